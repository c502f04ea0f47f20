"""Do the clustering oracle's pins bite?  Each case plants one plausible mistake in a private copy of
oracle/cluster_oracle.py (the committed file is untouched), puts the mutant's functions in place of
the oracle's for the duration of the test, and runs the pins of test_oracle_cluster_pins.py: at
least one must fail for every mistake.  CPU only."""
import types
from pathlib import Path

import pytest

import oracle
import oracle.cluster_oracle as committed
import test_oracle_cluster_pins as pins

SRC = Path(committed.__file__).read_text()

# (name, text in cluster_oracle.py, replacement) -- every text must occur in the source
MUTATIONS = [
    ("equal distances go to the upper centroid",
     "return np.argmin(dist, axis=2).astype(np.uint8)",
     "return (dist.shape[2] - 1 - np.argmin(dist[:, :, ::-1], axis=2)).astype(np.uint8)"),
    ("unused table entries take part in the assignment",
     "c64 = np.asarray(codebook, dtype=np.float16).astype(np.float64)[:, :ncent]\n    dist",
     "c64 = np.asarray(codebook, dtype=np.float16).astype(np.float64)\n    dist"),
    ("signed distance instead of absolute",
     "dist = np.abs(w64[:, :, None] - c64[:, None, :])",
     "dist = w64[:, :, None] - c64[:, None, :]"),
    ("cluster sizes shifted by one bin",
     "np.bincount(row, minlength=nslots)[:nslots]",
     "np.bincount(row + 1, minlength=nslots + 1)[:nslots]"),
    ("merge weights crossed, as the formula is printed",
     "new = (na * c64[n, a] + nb * c64[n, a + 1]) / (na + nb)",
     "new = (nb * c64[n, a] + na * c64[n, a + 1]) / (na + nb)"),
    ("merge takes the plain mean",
     "new = (na * c64[n, a] + nb * c64[n, a + 1]) / (na + nb) if na + nb > 0 else",
     "new = 0.5 * (c64[n, a] + c64[n, a + 1]) if na + nb > 0 else"),
    ("merge picks the widest gap",
     "a = int(np.argmin(gaps))",
     "a = int(np.argmax(gaps))"),
    ("re-numbering shifts the merged pair's upper index too late",
     "new_idx = idx - (idx > merged[:, None]).astype(np.uint8)",
     "new_idx = idx - (idx > merged[:, None] + 1).astype(np.uint8)"),
    ("rounding to fp16: ties go up",
     "if 2 * rem > ulp or (2 * rem == ulp and m % 2 == 1):",
     "if 2 * rem >= ulp:"),
    ("rounding to fp16: truncation",
     "if 2 * rem > ulp or (2 * rem == ulp and m % 2 == 1):",
     "if False:"),
    ("rounding to fp16: subnormals get the spacing of the first normal binade wrong",
     "e = -14\n    while e < 15",
     "e = -15\n    while e < 15"),
    ("stored merge rounds through binary32 first",
     "out[n, a] = round_to_half(new)",
     "out[n, a] = np.float16(np.float32(float(new)))"),
    ("stored merge takes the plain mean",
     "new = (na * ca + nb * cb_) / (na + nb) if na + nb > 0 else (ca + cb_) / 2",
     "new = (ca + cb_) / 2"),
    ("stored merge crosses the counts",
     "new = (na * ca + nb * cb_) / (na + nb) if na + nb > 0 else (ca + cb_) / 2",
     "new = (nb * ca + na * cb_) / (na + nb) if na + nb > 0 else (ca + cb_) / 2"),
    ("stored merge drops a centroid behind the pair",
     "out[n, a + 1:ncent - 1] = cb[n, a + 2:ncent]",
     "out[n, a + 1:ncent - 2] = cb[n, a + 3:ncent]"),
    ("merged centroid written one slot too far",
     "row = np.concatenate([c64[n, :a], [new], c64[n, a + 2:ncent]])",
     "row = np.concatenate([c64[n, :a + 1], [new], c64[n, a + 3:ncent], [0.0]])[:ncent - 1]"),
]

PINS = [getattr(pins, name) for name in dir(pins) if name.startswith("test_")]


def _run_pins():
    """Names of the pins that fail (parametrised pins run over all their cases)."""
    failed = []
    for fn in PINS:
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        cases = [()]
        for m in marks:
            names = [n.strip() for n in m.args[0].split(",")]
            cases = [c + (dict(zip(names, v if isinstance(v, (tuple, list)) else (v,))),) for c in cases for v in m.args[1]]
        for case in cases:
            kwargs = {}
            for d in case:
                kwargs.update(d)
            try:
                fn(**kwargs)
            except AssertionError:
                failed.append(fn.__name__)
                break
            except Exception:            # a mutant may also crash a pin: that counts as caught
                failed.append(fn.__name__)
                break
    return failed


def test_the_committed_oracle_passes_the_harness():
    assert _run_pins() == []


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, monkeypatch):
    assert SRC.count(old) == 1, f"mutation text not found exactly once: {name}"
    mutant = types.ModuleType("cluster_oracle_mutant")
    exec(compile(SRC.replace(old, new), "cluster_oracle_mutant", "exec"), mutant.__dict__)
    for fn in ("assign_nearest", "cluster_counts", "merge_closest", "merge_closest_stored", "round_to_half"):
        monkeypatch.setattr(oracle, fn, getattr(mutant, fn))
    failed = _run_pins()
    assert failed, f"no pin noticed: {name}"
    print(name, "->", failed)
