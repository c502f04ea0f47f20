"""GPU: batched decode (2 <= M <= 16) and prefill (lcd_lut_gemm) against the fp64 CPU oracle."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, assert_parity, check_layer, config_layers, run_hip, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [2, 3, 8, 16])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (80, 2304), (64, 11008), (32, 28672), (96, 5120), (48, 6656), (32, 13824), (8208, 1280)])
def test_gemv_batched_small(bits, M, shape):
    N, K = shape
    layer = synth.make_layer(2, 0, N, K, bits, M, seed_offset=N + K + M)
    check_layer(layer, bits, "gemv")


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [1, 5, 64, 130, 257])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (272, 1024), (1040, 512)])
def test_gemm_small(bits, M, shape):
    N, K = shape
    layer = synth.make_layer(3, 0, N, K, bits, M, seed_offset=N + K + M)
    check_layer(layer, bits, "gemm")


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("entry", ["gemv", "gemm"])
def test_batched_one_hot_rows_are_exact(bits, entry):
    # token m has x = e_{k_m}, s = 1: y[m][n] = C[n][idx[n][k_m]] exactly
    import torch
    N, K, M = 32, 512, 16
    layer = synth.make_layer(0, 0, N, K, bits, 1, seed_offset=9)
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    s = torch.ones(K, dtype=torch.float32, device="cuda")
    fn = lcd.lcd_lut_gemv if entry == "gemv" else lcd.lcd_lut_gemm
    for base in range(0, 256, 16):
        ks = [base + m for m in range(M)]
        x = torch.zeros((M, K), dtype=torch.float16, device="cuda")
        for m, k in enumerate(ks):
            x[m, k] = 1.0
        y = fn(packed, lut, x, s, N, bits).cpu().numpy()
        for m, k in enumerate(ks):
            assert np.array_equal(y[m], layer["codebook"][np.arange(N), layer["idx"][:, k]]), (m, k)


def _grouped_outputs(cfg_index, M, entry):
    """All matrices of a config through ONE grouped call (the launch configuration bench.py times);
    returns [(spec, layer, y)] with y as numpy.  Outputs start as NaN."""
    import torch
    config = synth.get_config(cfg_index)
    problems, keep = [], []
    for mid, spec, layer in config_layers(cfg_index, M, distinct_shapes_only=False):
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), config.bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), config.bits)
        y = torch.full((M, spec.N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, spec.N))
        keep.append((spec, layer))
    (lcd.lcd_lut_gemv_grouped if entry == "gemv" else lcd.lcd_lut_gemm_grouped)(problems, config.bits)
    torch.cuda.synchronize()
    return [(spec, layer, p[4].cpu().numpy()) for (spec, layer), p in zip(keep, problems)]


def _check_every_output(cfg_index, M):
    """Every output of every matrix of a decode config against the oracle: the grouped call over the
    whole set, and the single call on the first matrix of each shape."""
    bits = synth.get_config(cfg_index).bits
    seen = set()
    for spec, layer, y in _grouped_outputs(cfg_index, M, "gemv"):
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        assert_parity(y, Y, what=("grouped call", cfg_index, M, spec))
        if (spec.N, spec.K) not in seen:
            seen.add((spec.N, spec.K))
            assert_parity(run_hip(layer, bits, "gemv"), Y, what=("single call", cfg_index, M, spec))


def test_config2_batched_decode_full_size_every_output():
    _check_every_output(2, 16)


def test_config2_shapes_two_tokens_full_size_every_output():
    # two tokens at 2 bits run on the sparse-matrix-core kernel (one pass per token)
    _check_every_output(2, 2)


@pytest.mark.parametrize("M", [1, 3, 4])
def test_config2_shapes_int8_codes_full_size_every_output(M):
    # 2 bits with the INT8 codes of Sec. 4.1: up to four tokens run on the sparse-matrix-core kernel with
    # int8 operands.  One grouped call over the whole set, every output against the quantised oracle.
    import torch
    from paper_2506_12038_amd.binding import GemvGroup
    config = synth.get_config(2)
    problems, keep, steps = [], [], []
    for mid, spec, layer in config_layers(2, M, distinct_shapes_only=False):
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), config.bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), config.bits)
        y = torch.full((M, spec.N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, spec.N))
        steps.append(float(np.float32(np.quantile(np.abs(layer["x"].astype(np.float64) / layer["s"]), 0.99) / 127.0)))
        keep.append((spec, layer))
    GemvGroup(problems, config.bits, s_q=steps)()
    torch.cuda.synchronize()
    for (spec, layer), p, s_q in zip(keep, problems, steps):
        got = p[4].cpu().numpy()
        assert np.all(np.isfinite(got.astype(np.float32))), spec
        Y = oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, config.bits)
        err = oracle.parity_errors(got, Y)
        assert err["max_rel_floored"] <= 1e-3, (spec, M, err)


@pytest.mark.parametrize("M", [1, 8])
def test_config4_70b_mlp_full_size_every_output(M):
    _check_every_output(4, M)


def _check_prefill_sample(spec, layer, y, bits, mid, M):
    """Prefill outputs are too many for the oracle (2048 tokens): every row for 8 sampled tokens and
    every token for 96 sampled rows, both with the first and the last one; finite everywhere."""
    assert np.all(np.isfinite(y.astype(np.float32))), spec
    rng = np.random.default_rng(99 + mid)
    ms = np.sort(rng.choice(M, size=8, replace=False)); ms[0] = 0; ms[-1] = M - 1
    Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"][ms], layer["s"], bits)
    assert_parity(y[ms], Y, what=("all rows of sampled tokens", spec))
    rs = np.sort(rng.choice(spec.N, size=96, replace=False)); rs[0] = 0; rs[-1] = spec.N - 1
    Y = oracle.lut_matmul(layer["codebook"][rs], layer["idx"][rs], layer["x"], layer["s"], bits)
    # rms over the sampled rows stands in for the row rms (rows are i.i.d. by construction)
    assert_parity(y[:, rs], Y, what=("all tokens of sampled rows", spec))


def test_config3_prefill_full_size_single_calls():
    bits, M = synth.get_config(3).bits, 2048
    for mid, spec, layer in config_layers(3, M, distinct_shapes_only=True):
        _check_prefill_sample(spec, layer, run_hip(layer, bits, "gemm"), bits, mid, M)


def test_config3_prefill_full_size_grouped_call():
    bits, M = synth.get_config(3).bits, 2048
    for mid, (spec, layer, y) in enumerate(_grouped_outputs(3, M, "gemm")):
        _check_prefill_sample(spec, layer, y, bits, mid, M)


@pytest.mark.parametrize("bits,ncent", [(3, 5), (3, 6), (4, 10), (4, 13)])
@pytest.mark.parametrize("M,entry", [(1, "gemv"), (6, "gemv"), (70, "gemm")])
def test_codebooks_with_fewer_centroids_than_the_container_holds(bits, ncent, M, entry):
    # centroid counts that are no power of two (the paper's per-layer counts: 5, 6, 10, ...) live in the
    # next container; the codes above the count are never used and their table entries are zero
    N, K = 80, 1280
    layer = synth.make_layer(1, 3, N, K, bits, M, seed_offset=bits + ncent + M)
    layer["idx"] = (layer["idx"] % ncent).astype(np.uint8)
    layer["codebook"] = layer["codebook"].copy()
    layer["codebook"][:, ncent:] = 0
    assert int(layer["idx"].max()) == ncent - 1
    check_layer(layer, bits, entry)


@pytest.mark.parametrize("bits,M", [(2, 200), (3, 64), (3, 300), (4, 129)])
def test_grouped_prefill_matches_single_calls_and_oracle(bits, M):
    # several layers of different N and K in one pair of launches: the same bits as lcd_lut_gemm layer by layer
    import torch
    shapes = [(272, 1024), (1040, 512), (48, 2816), (4112, 256), (16, 4352)]
    problems, layers, singles = [], [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(3, i, N, K, bits, M, seed_offset=5 * i + bits + M)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        layers.append(layer)
        singles.append(lcd.lcd_lut_gemm(packed, lut, x, s, N, bits))
    lcd.lcd_lut_gemm_grouped(problems, bits)
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), layer, single in zip(problems, layers, singles):
        assert torch.equal(y, single)
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        assert oracle.parity_errors(y.cpu().numpy(), Y)["max_rel_floored"] <= TOL


def test_grouped_prefill_config3_sampled_and_replayed_from_a_hip_graph():
    # the launch configuration bench.py times for the prefill config: the whole 7B set in one grouped
    # call, captured once and replayed; sampled rows against the oracle, every replay against the eager call
    import torch
    from paper_2506_12038_amd.binding import GemmGroup
    config = synth.get_config(3)
    M = 256
    problems, samples = [], []
    for mid, spec in config.matrices():
        layer = synth.make_layer(3, mid, spec.N, spec.K, config.bits, M)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), config.bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), config.bits)
        y = torch.zeros((M, spec.N), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, spec.N))
        rs = np.sort(np.random.default_rng(mid).choice(spec.N, size=64, replace=False))
        rs[0] = 0; rs[-1] = spec.N - 1
        samples.append((rs, oracle.lut_matmul(layer["codebook"][rs], layer["idx"][rs], layer["x"], layer["s"], config.bits)))
        del layer
    group = GemmGroup(problems, config.bits)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        group(stream)
    torch.cuda.synchronize()
    eager = [p[4].clone() for p in problems]
    for (rs, Y), e in zip(samples, eager):
        assert oracle.parity_errors(e.cpu().numpy()[:, rs], Y)["max_rel_floored"] <= TOL
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        group(stream)
    for rep in range(3):
        for p in problems:
            p[4].fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        for p, e in zip(problems, eager):
            assert torch.equal(p[4], e), rep


@pytest.mark.parametrize("count", [1, 16])
def test_grouped_prefill_smallest_and_largest_group(count):
    # one layer (the grouped call degenerates to lcd_lut_gemm) and the largest group the entry point takes
    import torch
    bits, M = 3, 70
    problems, singles = [], []
    for i in range(count):
        N, K = 16 * (1 + i % 5), 256 * (1 + (3 * i) % 4)
        layer = synth.make_layer(3, i, N, K, bits, M, seed_offset=11 * i + count)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        singles.append(lcd.lcd_lut_gemm(packed, lut, x, s, N, bits))
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        assert oracle.parity_errors(singles[-1].cpu().numpy(), Y)["max_rel_floored"] <= TOL
    lcd.lcd_lut_gemm_grouped(problems, bits)
    torch.cuda.synchronize()
    for p, single in zip(problems, singles):
        assert torch.equal(p[4], single)

