"""Pins for oracle/metrics.py, the comparator that decides pass or fail of every GPU parity test,
and for the two helper functions of the C oracle that no product test goes through
(oracle_smooth, oracle_dequant).

The comparator's figures are checked against values worked out by hand on rows whose rms is an
exact number, and a planted mistake in a private copy of its source (denominator inflated, rms
over the wrong axis or over the whole matrix, a missing absolute value, the floor dropped or
applied the wrong way round) has to fail one of them.  CPU only.
"""
import types
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

import oracle
import oracle.metrics as committed

TOL = 2e-3          # the bound of the parity tests (tests/gpu_common.py states the same number)
SRC = Path(committed.__file__).read_text()


# ---- hand-worked cases -------------------------------------------------------------------------
# Row [3, 4, 0, 0]: mean square 25/4, rms 2.5.   Row [6, 8, 0, 0] * 100: rms 500.

def check_error_at_the_tolerance_passes_and_above_it_fails(pe):
    Y = np.array([[3.0, 4.0, 0.0, 0.0]])
    # an element that cancels to zero: the denominator is the row rms (2.5), not |Y| = 0
    y = Y.copy(); y[0, 2] = 2e-3 * 2.5
    e = pe(y, Y)
    assert e["max_rel_floored"] == pytest.approx(2e-3, rel=1e-12) and e["max_rel_floored"] <= TOL * (1 + 1e-12)
    assert e["max_abs"] == pytest.approx(0.005, rel=1e-12)
    y = Y.copy(); y[0, 2] = 3e-3 * 2.5
    e = pe(y, Y)
    assert e["max_rel_floored"] == pytest.approx(3e-3, rel=1e-12) and e["max_rel_floored"] > TOL
    # an element above the rms: the denominator is |Y| = 4
    y = Y.copy(); y[0, 1] = 4.0 + 4.0 * 2e-3
    assert pe(y, Y)["max_rel_floored"] == pytest.approx(2e-3, rel=1e-9)
    y = Y.copy(); y[0, 1] = 4.0 + 4.0 * 3e-3
    assert pe(y, Y)["max_rel_floored"] > TOL


def check_negative_errors_count(pe):
    Y = np.array([[3.0, 4.0, 0.0, 0.0]])
    y = Y.copy(); y[0, 0] = 3.0 - 0.03          # only too-small values: 0.03 / 3 = 1e-2
    e = pe(y, Y)
    assert e["max_rel_floored"] == pytest.approx(1e-2, rel=1e-9)
    assert e["max_abs"] == pytest.approx(0.03, rel=1e-9)
    assert e["max_rel_large"] == pytest.approx(1e-2, rel=1e-9)
    # a negative reference value: the denominator is its magnitude
    Yn = -Y
    yn = Yn.copy(); yn[0, 1] = -4.0 - 0.04
    assert pe(yn, Yn)["max_rel_floored"] == pytest.approx(1e-2, rel=1e-9)


def check_every_token_has_its_own_rms(pe):
    # token 0 has rms 2.5, token 1 rms 500: an error of 0.05 on a cancelling element of token 0 is
    # 2 % of ITS rms; measured against token 1's rms, the rms over the tokens (axis 0) or the rms of
    # the whole matrix it would look 100 times smaller
    Y = np.array([[3.0, 4.0, 0.0, 0.0], [600.0, 800.0, 0.0, 0.0]])
    y = Y.copy(); y[0, 3] = 0.05
    e = pe(y, Y)
    assert e["max_rel_floored"] == pytest.approx(0.02, rel=1e-12)
    # and the other way round: 1.0 on token 1's cancelling element is 2e-3 of its rms, not 0.4 of token 0's
    y = Y.copy(); y[1, 2] = 1.0
    assert pe(y, Y)["max_rel_floored"] == pytest.approx(2e-3, rel=1e-12)


def check_floor_only_lifts_small_denominators(pe):
    Y = np.array([[3.0, 4.0, 0.0, 0.0]])
    # |Y| = 3 is above the rms 2.5: the floor must not replace it (0.03 / 3, not 0.03 / 2.5)
    y = Y.copy(); y[0, 0] = 3.03
    assert pe(y, Y)["max_rel_floored"] == pytest.approx(0.01, rel=1e-9)
    # |Y| = 1 below the rms of [1, 7, 0, 0] (sqrt(12.5)): floored
    Y2 = np.array([[1.0, 7.0, 0.0, 0.0]])
    y2 = Y2.copy(); y2[0, 0] = 1.01
    assert pe(y2, Y2)["max_rel_floored"] == pytest.approx(0.01 / np.sqrt(12.5), rel=1e-12)


def check_max_rel_large_on_a_known_pair(pe):
    # entries with |Y| >= rms only, pure element-wise ratio: [1, 7, 0, 0] has rms 3.5355; only the 7 counts
    Y = np.array([[1.0, 7.0, 0.0, 0.0]])
    y = np.array([[1.5, 7.07, 0.0, 0.0]])
    e = pe(y, Y)
    assert e["max_rel_large"] == pytest.approx(0.01, rel=1e-9)
    assert e["max_rel_floored"] == pytest.approx(0.5 / np.sqrt(12.5), rel=1e-12)
    assert e["max_abs"] == pytest.approx(0.5, rel=1e-12)


def check_exact_match_all_zero_and_empty(pe):
    Y = np.array([[3.0, 4.0, 0.0, 0.0]])
    assert pe(Y.copy(), Y) == {"max_rel_floored": 0.0, "max_rel_large": 0.0, "max_abs": 0.0}
    Z = np.zeros((2, 3))
    e = pe(Z + 0.25, Z)               # an all-zero reference row: absolute error, no division by zero
    assert e["max_rel_floored"] == 0.25 and e["max_abs"] == 0.25
    assert pe(np.zeros((0, 4)), np.zeros((0, 4)))["max_rel_floored"] == 0.0


def check_shape_mismatch_and_nan(pe):
    with pytest.raises(ValueError):
        pe(np.zeros((2, 3)), np.zeros((3, 2)))
    with pytest.raises(ValueError):          # shapes that numpy would broadcast silently
        pe(np.zeros((1, 3)), np.zeros((2, 3)))
    with pytest.raises(ValueError):
        pe(np.zeros(3), np.zeros((2, 3)))
    # a NaN in the computed output (an output that was never written) must not pass a "<= TOL" test
    Y = np.array([[3.0, 4.0, 0.0, 0.0]])
    y = Y.copy(); y[0, 1] = np.nan
    assert not (pe(y, Y)["max_rel_floored"] <= TOL)


def check_rational_evaluation_on_random_data(pe):
    # the definition, max |y - Y| / max(|Y|, rms_n Y[m, :]), redone with rationals (the rms through
    # its square, so no square root is taken): the reported figure r must satisfy
    # (diff / |Y|) or (diff^2 / meansq) as appropriate, element by element
    rng = np.random.default_rng(3)
    Y = np.round(rng.standard_normal((3, 7)) * 8) / 4
    y = Y + np.round(rng.standard_normal((3, 7)) * 4) / 64
    best = Fraction(0)
    for m in range(3):
        meansq = sum(Fraction(float(v)) ** 2 for v in Y[m]) / 7
        for n in range(7):
            d, a = abs(Fraction(float(y[m, n])) - Fraction(float(Y[m, n]))), abs(Fraction(float(Y[m, n])))
            r2 = d * d / (a * a if a * a >= meansq else meansq)          # squared ratio, exact
            best = max(best, r2)
    got = pe(y, Y)["max_rel_floored"]
    assert got * got == pytest.approx(float(best), rel=1e-12)


CHECKS = [v for k, v in sorted(globals().items()) if k.startswith("check_")]


@pytest.mark.parametrize("check", CHECKS, ids=[c.__name__[6:] for c in CHECKS])
def test_parity_errors(check):
    check(oracle.parity_errors)


# ---- do these pins bite? -----------------------------------------------------------------------
MUTATIONS = [
    ("denominator ten times too large",
     "den = np.maximum(np.abs(Y), rms)",
     "den = 10.0 * np.maximum(np.abs(Y), rms)"),
    ("rms over the tokens instead of over the outputs of one token",
     "rms = np.sqrt(np.mean(Y * Y, axis=-1, keepdims=True))",
     "rms = np.sqrt(np.mean(Y * Y, axis=0, keepdims=True))"),
    ("one rms for the whole matrix",
     "rms = np.sqrt(np.mean(Y * Y, axis=-1, keepdims=True))",
     "rms = np.sqrt(np.mean(Y * Y))"),
    ("mean absolute value instead of the rms",
     "rms = np.sqrt(np.mean(Y * Y, axis=-1, keepdims=True))",
     "rms = np.mean(np.abs(Y), axis=-1, keepdims=True)"),
    ("root of the sum of squares (no mean)",
     "rms = np.sqrt(np.mean(Y * Y, axis=-1, keepdims=True))",
     "rms = np.sqrt(np.sum(Y * Y, axis=-1, keepdims=True))"),
    ("signed difference",
     "diff = np.abs(y - Y)",
     "diff = y - Y"),
    ("denominator is the rms everywhere (no element-wise part)",
     "den = np.maximum(np.abs(Y), rms)",
     "den = np.maximum(rms, rms)"),
    ("floor dropped (pure element-wise ratio)",
     "den = np.maximum(np.abs(Y), rms)",
     "den = np.abs(Y)"),
    ("floor applied the wrong way round",
     "den = np.maximum(np.abs(Y), rms)",
     "den = np.minimum(np.abs(Y), rms)"),
    ("signed reference in the denominator",
     "den = np.maximum(np.abs(Y), rms)",
     "den = np.maximum(Y, rms)"),
    ("NaNs ignored by the maximum",
     '"max_rel_floored": float(np.max(diff / den)),',
     '"max_rel_floored": float(np.nanmax(diff / den)),'),
    ("shapes broadcast instead of being compared",
     "if y.shape != Y.shape:",
     "if False:"),
    ("max_rel_large over all entries",
     "large = np.abs(Y) >= rms",
     "large = np.abs(Y) >= 0"),
    ("mean error instead of the maximum",
     '"max_rel_floored": float(np.max(diff / den)),',
     '"max_rel_floored": float(np.mean(diff / den)),'),
]


def _failed(pe):
    out = []
    for c in CHECKS:
        try:
            with np.errstate(all="ignore"):
                c(pe)
        except (AssertionError, pytest.fail.Exception):      # pytest.raises reports "did not raise" through the latter
            out.append(c.__name__)
        except Exception as e:          # a mutant may also crash a pin: that counts as caught
            out.append(c.__name__ + " (" + type(e).__name__ + ")")
    return out


def test_the_committed_comparator_passes_the_harness():
    assert _failed(committed.parity_errors) == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_in_the_comparator_is_caught(name, old, new):
    assert SRC.count(old) == 1, f"mutation text not found exactly once: {name}"
    mutant = types.ModuleType("metrics_mutant")
    exec(compile(SRC.replace(old, new), "metrics_mutant", "exec"), mutant.__dict__)
    failed = _failed(mutant.parity_errors)
    assert failed, f"no pin noticed: {name}"


def test_the_gpu_tests_use_this_tolerance():
    import gpu_common          # imports the product binding only lazily at call time
    assert gpu_common.TOL == TOL
