"""GPU: the prefill path with the input transformation of Sec. 4.1 (Eq. 10-11, b = 8) in front
(lcd_lut_gemm_q8, lcd_lut_gemm_q8_grouped) against the oracle's quantised product, the codes bit for
bit; and the grouped prefill call sharing one smoothed copy between layers that read the same input."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, assert_parity, to_dev

pytestmark = pytest.mark.gpu

Q8_TOL = 1e-3   # codes are exact matrix operands: only the fp32 accumulation and the fp16 store differ from the fp64 sum


def _step(layer):
    # the quantisation step puts the 99th percentile of |x/s| at code 127 (about 1 % of the codes clip)
    xs = layer["x"].astype(np.float64) / layer["s"].astype(np.float64)
    return float(np.float32(np.quantile(np.abs(xs), 0.99) / 127.0))


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [1, 64, 130, 257])
@pytest.mark.parametrize("shape", [(48, 768), (272, 1024), (1040, 512)])
def test_gemm_q8_matches_the_quantised_oracle(bits, M, shape):
    import torch
    N, K = shape
    layer = synth.make_layer(3, 0, N, K, bits, M, seed_offset=N + K + M + 3)
    s_q = _step(layer)
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    lcd.lcd_lut_gemm_q8(packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), s_q, N, bits, y=y)
    Y = oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, bits)
    assert_parity(y.cpu().numpy(), Y, Q8_TOL)


def test_gemm_q8_full_width_2048_tokens_sampled():
    # M = 2048 on a 7B-shaped layer: every row for sampled tokens, every token for sampled rows
    import torch
    bits, M, N, K = 3, 2048, 4096, 4096
    layer = synth.make_layer(3, 0, N, K, bits, M)
    s_q = _step(layer)
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    lcd.lcd_lut_gemm_q8(packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), s_q, N, bits, y=y)
    y = y.cpu().numpy()
    assert np.all(np.isfinite(y.astype(np.float32)))
    rng = np.random.default_rng(4)
    ms = np.sort(rng.choice(M, size=8, replace=False)); ms[0] = 0; ms[-1] = M - 1
    assert_parity(y[ms], oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"][ms], layer["s"], s_q, bits), Q8_TOL)
    rs = np.sort(rng.choice(N, size=96, replace=False)); rs[0] = 0; rs[-1] = N - 1
    assert_parity(y[:, rs], oracle.quantised_lut_matmul(layer["codebook"][rs], layer["idx"][rs], layer["x"], layer["s"], s_q, bits), Q8_TOL)


@pytest.mark.parametrize("M", [1, 70, 128, 300])
def test_gemm_q8_codes_are_bit_exact(M):
    # identity layer (row n reads column n through a one-hot codebook): y[m][n] = s_q * q[m][n] with a
    # power-of-two step, so every integer decision of the quantiser is visible; ties, clips and the
    # inputs on which the order of roundings decides the code are planted
    bits, N, K = 2, 1024, 1024
    codebook = np.zeros((N, 4), dtype=np.float16); codebook[:, 0] = 1.0
    idx = np.ones((N, K), dtype=np.uint8); idx[np.arange(N), np.arange(K)] = 0
    rng = np.random.default_rng(21 + M)
    x = (rng.standard_normal((M, K)) * 6).astype(np.float16)
    s = (0.25 + rng.random(K) * 3).astype(np.float32)
    s_q = 0.125
    s[:8] = 1.0
    x[0, :8] = np.array([0.0625, 0.1875, -0.0625, -0.1875, 15.9375, 100.0, -100.0, 16.0], dtype=np.float16)
    q = oracle.input_transform(x, s, s_q, 8, single_precision=True)
    assert q[0, :8].tolist() == [0, 2, 0, -2, 127, 127, -128, 127]
    packed = lcd.lcd_pack_indices(to_dev(idx), bits)
    lut = lcd.lcd_build_lut(to_dev(codebook), bits)
    y = lcd.lcd_lut_gemm_q8(packed, lut, to_dev(x), to_dev(s), s_q, N, bits).cpu().numpy()
    assert np.array_equal(y.astype(np.float64) / s_q, q.astype(np.float64))
    # the decode entry point quantises the same way
    if M <= 16:
        y2 = lcd.lcd_lut_gemv_q8(packed, lut, to_dev(x), to_dev(s), s_q, N, bits).cpu().numpy()
        assert np.array_equal(y, y2)


def test_gemm_q8_decides_hard_cases_like_the_binary32_oracle():
    cases = [(49119, 2.232786178588867, 0.028895359486341476), (51926, 1.3333886861801147, 0.08302413672208786),
             (52416, 2.515049934387207, 0.0709344744682312), (18075, 2.6308062076568604, 0.05176938697695732),
             (51858, 2.7504186630249023, 0.048504382371902466), (49771, 0.9853012561798096, 0.038542672991752625),
             (51873, 1.5403376817703247, 0.0839715301990509), (52298, 1.627970814704895, 0.0839715301990509),
             (50758, 1.0950627326965332, 0.04875607416033745), (17859, 2.0101850032806396, 0.0320252850651741)]
    bits, N, K, M = 2, 256, 256, 40
    codebook = np.zeros((N, 4), dtype=np.float16); codebook[:, 0] = 1.0
    idx = np.ones((N, K), dtype=np.uint8); idx[np.arange(N), np.arange(K)] = 0
    packed = lcd.lcd_pack_indices(to_dev(idx), bits)
    lut = lcd.lcd_build_lut(to_dev(codebook), bits)
    for bits16, s0, s_q in cases:
        x = np.zeros((M, K), dtype=np.float16)
        x[:, 0] = np.array([bits16], dtype=np.uint16).view(np.float16)[0]
        s = np.ones(K, dtype=np.float32); s[0] = s0
        expect = oracle.input_transform(x, s, s_q, 8, single_precision=True)
        y = lcd.lcd_lut_gemm_q8(packed, lut, to_dev(x), to_dev(s), s_q, N, bits).cpu().numpy()
        got = np.rint(y.astype(np.float64) / s_q).astype(np.int32)
        assert np.array_equal(got, expect), (bits16, s0, s_q, got[:, 0], expect[:, 0])


@pytest.mark.parametrize("bits,M", [(2, 200), (3, 64), (4, 129)])
def test_grouped_gemm_q8_matches_single_calls_and_oracle(bits, M):
    import torch
    from paper_2506_12038_amd.binding import GemmGroup
    shapes = [(272, 1024), (1040, 512), (48, 2816), (16, 4352)]
    problems, layers, singles, steps = [], [], [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(3, i, N, K, bits, M, seed_offset=7 * i + bits + M)
        s_q = _step(layer)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        layers.append(layer); steps.append(s_q)
        singles.append(lcd.lcd_lut_gemm_q8(packed, lut, x, s, s_q, N, bits))
    GemmGroup(problems, bits, s_q=steps)()
    torch.cuda.synchronize()
    for p, layer, single, s_q in zip(problems, layers, singles, steps):
        assert torch.equal(p[4], single)
        Y = oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, bits)
        assert_parity(p[4].cpu().numpy(), Y, Q8_TOL)


@pytest.mark.parametrize("quantised", [False, True])
def test_grouped_prefill_layers_that_share_an_input(quantised):
    # q/k/v-like: three layers read ONE x and s (same pointers) and get one smoothed copy; a fourth
    # layer with the same K but its own input, and (quantised) a fifth that shares x with another step,
    # must not be mixed up.  Every output against the oracle and against the single calls.
    import torch
    from paper_2506_12038_amd.binding import GemmGroup
    bits, M, K = 3, 150, 1024
    base = synth.make_layer(3, 0, 64, K, bits, M, seed_offset=1)
    other = synth.make_layer(3, 1, 64, K, bits, M, seed_offset=2)
    x0, s0, x1, s1 = to_dev(base["x"]), to_dev(base["s"]), to_dev(other["x"]), to_dev(other["s"])
    step0, step1 = _step(base), _step(other)
    specs = [(272, x0, s0, base, step0), (48, x0, s0, base, step0), (1040, x0, s0, base, step0), (64, x1, s1, other, step1),
             (96, x0, s0, base, step0 * 1.5)]
    problems, refs = [], []
    for i, (N, x, s, src, s_q) in enumerate(specs):
        w = synth.make_layer(3, 10 + i, N, K, bits, 1, seed_offset=i)
        packed = lcd.lcd_pack_indices(to_dev(w["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(w["codebook"]), bits)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        if quantised:
            refs.append((oracle.quantised_lut_matmul(w["codebook"], w["idx"], src["x"], src["s"], s_q, bits),
                         lcd.lcd_lut_gemm_q8(packed, lut, x, s, s_q, N, bits)))
        else:
            refs.append((oracle.lut_matmul(w["codebook"], w["idx"], src["x"], src["s"], bits), lcd.lcd_lut_gemm(packed, lut, x, s, N, bits)))
    GemmGroup(problems, bits, s_q=[sp[4] for sp in specs] if quantised else None)()
    torch.cuda.synchronize()
    for p, (Y, single) in zip(problems, refs):
        assert torch.equal(p[4], single)
        assert_parity(p[4].cpu().numpy(), Y, Q8_TOL if quantised else TOL)
