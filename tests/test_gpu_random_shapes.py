"""GPU: seeded random shapes through every product entry point against the fp64 oracle.

The fixed-shape tests pick their cases by hand; this one draws (N, K, M, bits, group make-up) from a
seeded generator so that tile counts, segment tails, visit boundaries and workgroup splits that
nobody thought of get exercised too.  Sizes stay small enough for the oracle to finish in seconds."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, check_layer, to_dev

pytestmark = pytest.mark.gpu


def _draw(rng, max_weights=3_000_000):
    while True:
        N = 16 * int(rng.integers(1, 200))
        K = 256 * int(rng.integers(1, 60))
        if N * K <= max_weights:
            return N, K


@pytest.mark.parametrize("seed", range(24))
def test_random_single_layer(seed):
    rng = np.random.default_rng(1000 + seed)
    N, K = _draw(rng)
    bits = int(rng.integers(2, 5))
    M = int(rng.choice([1, 1, 2, 3, 7, 8, 13, 16, 40, 129]))
    entry = "gemv" if M <= 16 else "gemm"
    layer = synth.make_layer(0, seed, N, K, bits, M, seed_offset=seed)
    err = check_layer(layer, bits, entry)
    print(seed, N, K, bits, M, entry, err["max_rel_floored"])


@pytest.mark.parametrize("seed", range(32))
def test_random_groups(seed):
    import torch
    rng = np.random.default_rng(2000 + seed)
    count = int(rng.integers(1, 9))
    bits = int(rng.integers(2, 5))
    M = int(rng.choice([1, 1, 2, 3, 4, 5, 16]))
    quantised = bool(rng.integers(0, 2))
    problems, refs, steps = [], [], []
    for i in range(count):
        N, K = _draw(rng, max_weights=600_000)
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=100 * seed + i)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, N))
        if quantised:
            s_q = float(np.float32(np.quantile(np.abs(layer["x"].astype(np.float64) / layer["s"]), 0.99) / 127.0))
            steps.append(s_q)
            refs.append(oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, bits))
        else:
            refs.append(oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits))
    from paper_2506_12038_amd.binding import GemvGroup
    GemvGroup(problems, bits, s_q=steps if quantised else None)()
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), Y in zip(problems, refs):
        err = oracle.parity_errors(y.cpu().numpy(), Y)
        assert err["max_rel_floored"] <= (1e-3 if quantised else TOL), (seed, N, err)


@pytest.mark.parametrize("seed", range(8))
def test_random_prefill_groups(seed):
    # grouped prefill with random shapes, token counts, index widths; some layers read the input of the
    # layer before them (same tensors), with fp16 activations or INT8 codes
    import torch
    from paper_2506_12038_amd.binding import GemmGroup
    rng = np.random.default_rng(3000 + seed)
    count = int(rng.integers(1, 7))
    bits = int(rng.integers(2, 5))
    M = int(rng.choice([1, 17, 64, 100, 128, 129, 300]))
    quantised = bool(rng.integers(0, 2))
    problems, refs, steps = [], [], []
    prev = None
    for i in range(count):
        N, K = _draw(rng, max_weights=400_000)
        share = prev is not None and bool(rng.integers(0, 2))
        if share:                                   # same K, same x and s tensors as the layer before
            K, src, x, s, s_q = prev
        else:
            src = synth.make_layer(3, i, 16, K, bits, M, seed_offset=100 * seed + i)
            x, s = to_dev(src["x"]), to_dev(src["s"])
            s_q = float(np.float32(np.quantile(np.abs(src["x"].astype(np.float64) / src["s"]), 0.99) / 127.0))
        prev = (K, src, x, s, s_q)
        w = synth.make_layer(3, 20 + i, N, K, bits, 1, seed_offset=100 * seed + i)
        packed = lcd.lcd_pack_indices(to_dev(w["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(w["codebook"]), bits)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        steps.append(s_q)
        if quantised:
            refs.append(oracle.quantised_lut_matmul(w["codebook"], w["idx"], src["x"], src["s"], s_q, bits))
        else:
            refs.append(oracle.lut_matmul(w["codebook"], w["idx"], src["x"], src["s"], bits))
    GemmGroup(problems, bits, s_q=steps if quantised else None)()
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), Y in zip(problems, refs):
        got = y.cpu().numpy()
        assert np.all(np.isfinite(got.astype(np.float32)))
        err = oracle.parity_errors(got, Y)
        assert err["max_rel_floored"] <= (1e-3 if quantised else TOL), (seed, N, M, bits, err)


@pytest.mark.parametrize("M,N,K,bits", [(5000, 48, 512, 3), (8192 + 33, 16, 256, 2), (4097, 272, 768, 4)])
def test_prefill_many_tokens(M, N, K, bits):
    # token counts far beyond one workgroup's 128-token tile, ragged at the end, on matrices small
    # enough for the oracle: every token block of the grid is compared
    layer = synth.make_layer(4, M % 97, N, K, bits, M, seed_offset=M)
    err = check_layer(layer, bits, "gemm")
    print(M, N, K, bits, err["max_rel_floored"])
