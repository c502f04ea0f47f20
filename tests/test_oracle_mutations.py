"""Do the oracle's pins bite?  Each case plants one plausible mistake in a private copy of the
oracle's C source (the committed oracle is untouched), builds it, and runs the pin tests of
test_oracle_pins.py against it: at least one pin must fail for every mistake.  CPU only.
"""
import ctypes
import importlib
import subprocess
from pathlib import Path

import pytest

import oracle.lcd_oracle as wrapper
import test_oracle_pins as pins

SRC = Path(wrapper.__file__).resolve().parent / "lcd_oracle.c"

# (name, text in lcd_oracle.c, replacement) -- every text must occur in the source
MUTATIONS = [
    ("smoothing multiplies instead of divides (product)",
     "double xs = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];",
     "double xs = oracle_half_to_double(x[(size_t)m * K + k]) * (double)s[k];"),
    ("smoothing dropped (product)",
     "double xs = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];",
     "double xs = oracle_half_to_double(x[(size_t)m * K + k]);"),
    ("codebook of the wrong row",
     "cent[c] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);",
     "cent[c] = oracle_half_to_double(codebook[(size_t)(n > 0 ? n - 1 : 0) * ncent + c]);"),
    ("index matrix read transposed",
     "int c = idx[(size_t)n * K + k];\n                if (c >= ncent) { bad = 1; c = 0; }\n                double xs",
     "int c = idx[((size_t)n * K + k) % ((size_t)N * K) == (size_t)n * K + k ? ((size_t)k * N + n) % ((size_t)N * K) : 0];\n                if (c >= ncent) { bad = 1; c = 0; }\n                double xs"),
    ("last column dropped from the sum",
     "for (int k = 0; k < K; k++) {\n                int c = idx[(size_t)n * K + k];\n                if (c >= ncent) { bad = 1; c = 0; }\n                double xs",
     "for (int k = 0; k < K - 1; k++) {\n                int c = idx[(size_t)n * K + k];\n                if (c >= ncent) { bad = 1; c = 0; }\n                double xs"),
    ("output written transposed",
     "            Y[(size_t)m * N + n] = acc;\n        }\n    }\n    return bad;\n}\n\n/* Same result in centroid-bucket order",
     "            Y[(size_t)(M == N ? n * N + m : m * N + n)] = acc;\n        }\n    }\n    return bad;\n}\n\n/* Same result in centroid-bucket order"),
    ("sign of the product flipped",
     "acc += xs * cent[c];",
     "acc -= xs * cent[c];"),
    ("bucket form ignores the smoothing factor",
     "S[c] += oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];",
     "S[c] += oracle_half_to_double(x[(size_t)m * K + k]);"),
    ("bucket form uses centroid c+1",
     "acc += oracle_half_to_double(codebook[(size_t)n * ncent + c]) * S[c];",
     "acc += oracle_half_to_double(codebook[(size_t)n * ncent + (c + 1) % ncent]) * S[c];"),
    ("fp16 exponent bias off by one",
     "v = ldexp((double)(1024 + frac), expo - 25);",
     "v = ldexp((double)(1024 + frac), expo - 24);"),
    ("fp16 subnormals flushed to zero",
     "v = ldexp((double)frac, -24);",
     "v = 0.0;"),
    ("fp16 sign ignored",
     "return sign ? -v : v;",
     "return v;"),
    ("input transformation rounds half away from zero",
     "double r = nearbyint(v);",
     "double r = round(v);"),
    ("input transformation clips to the printed range",
     "double lo = -ldexp(1.0, b - 1), hi = ldexp(1.0, b - 1) - 1.0;",
     "double lo = -ldexp(1.0, b), hi = ldexp(1.0, b) - 1.0;"),
    ("binary32 quantiser divides in double precision",
     "volatile float v = xf / d;",
     "volatile float v = (float)((double)xf / ((double)s_m[k] * (double)s_q));"),
    ("binary32 quantiser multiplies by a rounded reciprocal",
     "volatile float v = xf / d;",
     "volatile float rcp = 1.0f / d; volatile float v = xf * rcp;"),
    ("binary32 quantiser rounds half away from zero",
     "float r = nearbyintf(v);",
     "float r = roundf(v);"),
    ("binary32 quantiser clips symmetrically",
     "float lo = -ldexpf(1.0f, b - 1), hi = ldexpf(1.0f, b - 1) - 1.0f;",
     "float lo = -ldexpf(1.0f, b - 1) + 1.0f, hi = ldexpf(1.0f, b - 1) - 1.0f;"),
    ("smoothed input multiplied instead of divided",
     "xs[(size_t)m * K + k] = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];",
     "xs[(size_t)m * K + k] = oracle_half_to_double(x[(size_t)m * K + k]) * (double)s[k];"),
    ("smoothed input takes the factor of the token, not of the channel",
     "xs[(size_t)m * K + k] = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];",
     "xs[(size_t)m * K + k] = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[m];"),
    ("smoothed input divides in single precision",
     "xs[(size_t)m * K + k] = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];",
     "xs[(size_t)m * K + k] = (float)oracle_half_to_double(x[(size_t)m * K + k]) / s[k];"),
    ("dequantised weight from the codebook of row 0",
     "What[(size_t)n * K + k] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);",
     "What[(size_t)n * K + k] = oracle_half_to_double(codebook[c]);"),
    ("dequantised weights written transposed",
     "What[(size_t)n * K + k] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);",
     "What[((size_t)k * N + n) % ((size_t)N * K)] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);"),
    ("dequantised weight of the wrong centroid",
     "What[(size_t)n * K + k] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);",
     "What[(size_t)n * K + k] = oracle_half_to_double(codebook[(size_t)n * ncent + (c ^ 1)]);"),
]


def pin_calls():
    """Every pin of test_oracle_pins.py as a zero-argument call (parametrised ones expanded)."""
    calls = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn, {}))
            continue
        combos = [{}]
        for m in marks:
            names = [a.strip() for a in m.args[0].split(",")]
            new = []
            for values in m.args[1]:
                if len(names) == 1:
                    values = (values,)
                for c in combos:
                    d = dict(c)
                    d.update(dict(zip(names, values)))
                    new.append(d)
            combos = new
        calls.extend((name, fn, c) for c in combos)
    return calls


@pytest.mark.parametrize("case", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(case, tmp_path):
    name, old, new = case
    text = SRC.read_text()
    assert text.count(old) >= 1, "the mutation target is not in the oracle source any more"
    mutated = tmp_path / "mutant.c"
    mutated.write_text(text.replace(old, new, 1))
    lib_path = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-o", str(lib_path), str(mutated), "-lm"])
    saved_lib, saved_path = wrapper._lib, wrapper._LIB
    failures = []
    try:
        wrapper._lib, wrapper._LIB = None, lib_path      # the wrapper loads the mutant from here
        wrapper.build_oracle = lambda force=False: lib_path
        for pin, fn, kwargs in pin_calls():
            try:
                fn(**kwargs)
            except AssertionError:
                failures.append(pin)
            except Exception as e:                      # a mutant may also crash a pin: that counts
                failures.append(pin + " (" + type(e).__name__ + ")")
    finally:
        importlib.reload(wrapper)                        # restores build_oracle and the paths
        wrapper._lib = saved_lib
    assert failures, "no pin noticed: " + name


def test_the_unmutated_oracle_passes_the_same_harness():
    for pin, fn, kwargs in pin_calls():
        fn(**kwargs)
