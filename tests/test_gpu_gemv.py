"""GPU: decode path (lcd_lut_gemv) against the fp64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, assert_parity, check_layer, config_layers, run_hip, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (80, 2304), (256, 4096), (64, 11008), (96, 8192), (32, 28672), (16, 69632), (1088, 4352), (139264, 512), (64, 5120), (48, 13824)])
def test_gemv_m1_small(bits, shape):
    N, K = shape
    layer = synth.make_layer(0, 0, N, K, bits, 1, variant="B", seed_offset=N + K)
    err = check_layer(layer, bits)
    print(shape, bits, err)


@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("tiles_per_workgroup,K", [(3, 4352), (5, 4352), (6, 4352), (7, 4352), (3, 8704), (33, 512)])
def test_gemv_m1_runs_of_every_length_modulo_four(bits, tiles_per_workgroup, K):
    # The single-token kernel loads packed words three steps ahead through four register sets; a run of
    # row tiles (one visit in one K segment) whose length is no multiple of four ends in a short turn and
    # hands the next run its loads in other sets.  One layer over all compute units gives every workgroup
    # the same run length: 3, 5, 6, 7 (remainders 3, 1, 2, 3) with two or three segments, and 33 = a full
    # visit of 32 plus one tile.  M = 2 takes the two-token variant of that kernel at 2 bits and the
    # dequantising kernel at 3 bits over the same sequence; M = 3 the dequantising kernel.
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    N = cus * tiles_per_workgroup * 16
    for M in (1, 2, 3):
        layer = synth.make_layer_uniform(N, K, bits, M, seed=100 * tiles_per_workgroup + bits + M)
        err = check_layer(layer, bits)
        print(N, K, bits, M, err)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gemv_m1_one_hot_reads_single_centroids(bits):
    # x = e_k, s = 1: y[n] must be exactly C[n][idx[n,k]] -- sweeps every bit position of a tile
    import torch
    N, K = 32, 512
    layer = synth.make_layer(0, 0, N, K, bits, 1, seed_offset=5)
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    s = torch.ones(K, dtype=torch.float32, device="cuda")
    for k in list(range(0, 256)) + [300, 511]:
        x = torch.zeros((1, K), dtype=torch.float16, device="cuda")
        x[0, k] = 1.0
        y = lcd.lcd_lut_gemv(packed, lut, x, s, N, bits).cpu().numpy()[0]
        expect = layer["codebook"][np.arange(N), layer["idx"][:, k]]
        assert np.array_equal(y, expect), k


@pytest.mark.parametrize("cfg", [0, 1])
def test_gemv_m1_config_matrices(cfg):
    config = synth.get_config(cfg)
    seen = set()
    for mid, spec in config.matrices():
        if (spec.N, spec.K) in seen:
            continue
        seen.add((spec.N, spec.K))
        layer = synth.make_layer(cfg, mid, spec.N, spec.K, config.bits, 1)
        err = check_layer(layer, config.bits)
        print(cfg, spec, err)


def test_gemv_is_deterministic():
    layer = synth.make_layer(1, 6, 4096, 11008, 3, 1)
    y1 = run_hip(layer, 3)
    y2 = run_hip(layer, 3)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))


@pytest.mark.parametrize("bits,M", [(3, 1), (2, 1), (2, 2), (3, 2), (2, 4), (4, 1), (4, 7)])
def test_grouped_launch_matches_oracle_and_single_calls(bits, M):
    # a mixed group: different N and K per layer, one launch
    import torch
    shapes = [(64, 1024), (208, 512), (48, 2816), (16, 256), (96, 4352)]
    problems, layers, singles = [], [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=3 * i + bits)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        layers.append(layer)
        singles.append(lcd.lcd_lut_gemv(packed, lut, x, s, N, bits))
    lcd.lcd_lut_gemv_grouped(problems, bits)
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), layer, single in zip(problems, layers, singles):
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        err = oracle.parity_errors(y.cpu().numpy(), Y)
        assert err["max_rel_floored"] <= TOL, err
        assert torch.equal(y, single)  # same kernel, same reduction order: bit-identical


@pytest.mark.parametrize("cfg", [0, 1])
def test_grouped_config_full_size_every_output(cfg):
    # the launch configuration bench.py times (config 1: the whole 7B set in one grouped call), every
    # output of every matrix against the oracle, outputs NaN before the launch
    import torch
    config = synth.get_config(cfg)
    problems, layers = [], []
    for mid, spec, layer in config_layers(cfg, 1, distinct_shapes_only=False):
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), config.bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), config.bits)
        y = torch.full((1, spec.N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, spec.N))
        layers.append((spec, layer))
    lcd.lcd_lut_gemv_grouped(problems, config.bits)
    torch.cuda.synchronize()
    for p, (spec, layer) in zip(problems, layers):
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], config.bits)
        assert_parity(p[4].cpu().numpy(), Y, what=(cfg, spec))


@pytest.mark.parametrize("bits,M,quantised", [(3, 1, False), (2, 16, False), (2, 16, True), (4, 3, True), (3, 1, True), (2, 2, False), (2, 2, True), (2, 3, True), (2, 1, True)])
def test_grouped_launch_replayed_from_a_hip_graph(bits, M, quantised):
    # the launch configuration bench.py times: the grouped call captured once, replayed several times
    # with eager work and synchronisations in between; every replay must reproduce the eager result
    import torch
    from paper_2506_12038_amd.binding import GemvGroup
    shapes = [(256, 4096), (176, 2816), (64, 11008)]
    problems, eager, steps = [], [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=17 * i + bits + M)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        if quantised:   # two kernels per call for several tokens: the activation pre-pass, then the product
            s_q = float(np.float32(np.quantile(np.abs(layer["x"].astype(np.float64) / layer["s"]), 0.99) / 127.0))
            steps.append(s_q)
            Y = oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, bits)
            ref = lcd.lcd_lut_gemv_q8(packed, lut, x, s, s_q, N, bits)
            assert oracle.parity_errors(ref.cpu().numpy(), Y)["max_rel_floored"] <= 1e-3
        else:
            Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
            ref = lcd.lcd_lut_gemv(packed, lut, x, s, N, bits)
            assert oracle.parity_errors(ref.cpu().numpy(), Y)["max_rel_floored"] <= TOL
        eager.append(ref)
    group = GemvGroup(problems, bits, s_q=steps if quantised else None)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        group(stream)                      # first call outside capture (lazy module load)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        group(stream)
    for rep in range(3):
        for p in problems:
            p[4].fill_(float("nan"))       # eager work between the replays
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        for p, ref in zip(problems, eager):
            assert torch.equal(p[4], ref), rep


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 16])
@pytest.mark.parametrize("shape", [(64, 1024), (48, 11008)])
def test_gemv_q8_matches_the_quantised_oracle(bits, M, shape):
    # input transformation (Eq. 10-11, b = 8) in front of the product; s_q such that ~1 % of the codes clip
    N, K = shape
    layer = synth.make_layer(1, 0, N, K, bits, M, seed_offset=N + K + M + 7)
    xs = layer["x"].astype(np.float64) / layer["s"].astype(np.float64)
    s_q = float(np.float32(np.quantile(np.abs(xs), 0.99) / 127.0))
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    y = lcd.lcd_lut_gemv_q8(packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), s_q, N, bits).cpu().numpy()
    Y = oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, bits)
    err = oracle.parity_errors(y, Y)
    assert err["max_rel_floored"] <= 1e-3, err      # only fp32 accumulation and the fp16 store differ


@pytest.mark.parametrize("M", [1, 2, 3, 4, 16])
def test_gemv_q8_codes_are_bit_exact(M):
    # identity layer (row n reads column n through a one-hot codebook): y[m][n] = s_q * q[m][n], so the
    # quantiser's integer decisions are visible one by one; s_q = 2^-3 keeps the scaling exact.
    import torch
    bits, N, K = 2, 2048, 2048
    codebook = np.zeros((N, 4), dtype=np.float16); codebook[:, 0] = 1.0
    idx = np.ones((N, K), dtype=np.uint8); idx[np.arange(N), np.arange(K)] = 0
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((M, K)) * 6).astype(np.float16)
    s = (0.25 + rng.random(K) * 3).astype(np.float32)
    s_q = 0.125
    # plant exact ties and clip cases: s = 1 -> x / s_q = 8x
    s[:8] = 1.0
    x[0, :8] = np.array([0.0625, 0.1875, -0.0625, -0.1875, 15.9375, 100.0, -100.0, 16.0], dtype=np.float16)
    q = oracle.input_transform(x, s, s_q, 8, single_precision=True)
    assert q[0, :8].tolist() == [0, 2, 0, -2, 127, 127, -128, 127]
    packed = lcd.lcd_pack_indices(to_dev(idx), bits)
    lut = lcd.lcd_build_lut(to_dev(codebook), bits)
    y = lcd.lcd_lut_gemv_q8(packed, lut, to_dev(x), to_dev(s), s_q, N, bits).cpu().numpy()
    assert np.array_equal(y.astype(np.float64) / s_q, q.astype(np.float64))


@pytest.mark.parametrize("bits,M", [(3, 1), (2, 1), (2, 2), (2, 3), (2, 4), (2, 8), (4, 1), (4, 5)])
def test_grouped_q8_matches_oracle_and_single_calls(bits, M):
    # one launch over layers with different shapes and different quantisation steps
    import torch
    from paper_2506_12038_amd.binding import GemvGroup
    shapes = [(64, 1024), (208, 512), (48, 2816), (96, 4352)]
    problems, layers, singles, steps = [], [], [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=5 * i + bits + M)
        xs = layer["x"].astype(np.float64) / layer["s"].astype(np.float64)
        s_q = float(np.float32(np.quantile(np.abs(xs), 0.99) / 127.0))
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        layers.append(layer)
        steps.append(s_q)
        singles.append(lcd.lcd_lut_gemv_q8(packed, lut, x, s, s_q, N, bits))
    GemvGroup(problems, bits, s_q=steps)()
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), layer, single, s_q in zip(problems, layers, singles, steps):
        Y = oracle.quantised_lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], s_q, bits)
        err = oracle.parity_errors(y.cpu().numpy(), Y)
        assert err["max_rel_floored"] <= 1e-3, err
        assert torch.equal(y, single)


@pytest.mark.parametrize("bits,M", [(2, 3), (3, 16), (4, 1), (4, 9)])
def test_grouped_wide_and_narrow_layers(bits, M):
    # a group with one layer wide enough for the activations to be smoothed ahead of the product:
    # then all its layers take that route, while the single calls of the narrow ones smooth inside
    # the kernel; both round the same way, so the outputs must agree bit for bit
    import torch
    shapes = [(32, 16384), (64, 1024), (48, 2816)]
    problems, layers, singles = [], [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=11 * i + bits + M)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        layers.append(layer)
        singles.append(lcd.lcd_lut_gemv(packed, lut, x, s, N, bits))
    lcd.lcd_lut_gemv_grouped(problems, bits)
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), layer, single in zip(problems, layers, singles):
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        assert oracle.parity_errors(y.cpu().numpy(), Y)["max_rel_floored"] <= TOL
        assert torch.equal(y, single)


@pytest.mark.parametrize("M", [1, 6])
def test_grouped_layers_of_mixed_index_widths(M):
    # per-layer centroid counts: 4, 6 (3-bit container), 10 (4-bit container), 8, 16 in one call
    import torch
    from paper_2506_12038_amd.binding import GemvGroup
    specs = [(64, 1024, 2, 4), (208, 512, 3, 6), (48, 2816, 4, 10), (96, 1280, 3, 8), (32, 768, 4, 16)]
    problems, layers = [], []
    for i, (N, K, bits, ncent) in enumerate(specs):
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=13 * i + M)
        layer["idx"] = (layer["idx"] % ncent).astype(np.uint8)
        layer["codebook"] = layer["codebook"].copy()
        layer["codebook"][:, ncent:] = 0
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, N))
        layers.append((layer, bits))
    GemvGroup(problems, [b for _, _, b, _ in specs])()
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), (layer, bits) in zip(problems, layers):
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        assert oracle.parity_errors(y.cpu().numpy(), Y)["max_rel_floored"] <= TOL
        assert torch.equal(y, lcd.lcd_lut_gemv(packed, lut, x, s, N, bits))


def test_gemv_q8_decides_hard_cases_like_the_binary32_oracle():
    # inputs on which the order of roundings decides the code (a double-precision quotient, or a
    # product with a rounded reciprocal, gives the neighbouring integer): the kernel's split division
    # must land on the correctly rounded binary32 quotient
    import torch
    cases = [(49119, 2.232786178588867, 0.028895359486341476), (51926, 1.3333886861801147, 0.08302413672208786),
             (52416, 2.515049934387207, 0.0709344744682312), (18075, 2.6308062076568604, 0.05176938697695732),
             (51858, 2.7504186630249023, 0.048504382371902466), (49771, 0.9853012561798096, 0.038542672991752625),
             (51873, 1.5403376817703247, 0.0839715301990509), (52298, 1.627970814704895, 0.0839715301990509),
             (50758, 1.0950627326965332, 0.04875607416033745), (17859, 2.0101850032806396, 0.0320252850651741)]
    bits, N, K = 2, 256, 256
    codebook = np.zeros((N, 4), dtype=np.float16); codebook[:, 0] = 1.0
    idx = np.ones((N, K), dtype=np.uint8); idx[np.arange(N), np.arange(K)] = 0     # row n reads column n
    packed = lcd.lcd_pack_indices(to_dev(idx), bits)
    lut = lcd.lcd_build_lut(to_dev(codebook), bits)
    for M in (1, 3):
        for bits16, s0, s_q in cases:
            x = np.zeros((M, K), dtype=np.float16)
            x[:, 0] = np.array([bits16], dtype=np.uint16).view(np.float16)[0]
            s = np.ones(K, dtype=np.float32); s[0] = s0
            expect = oracle.input_transform(x, s, s_q, 8, single_precision=True)
            y = lcd.lcd_lut_gemv_q8(packed, lut, to_dev(x), to_dev(s), s_q, N, bits).cpu().numpy()
            got = np.rint(y.astype(np.float64) / s_q).astype(np.int32)      # y = fp16(s_q * q): q is recoverable
            assert np.array_equal(got, expect), (M, bits16, s0, s_q, got[:, 0], expect[:, 0])


@pytest.mark.parametrize("bits,M,quantised", [(2, 4, True), (3, 16, False), (4, 2, True), (2, 1, True)])
def test_grouped_decode_layers_that_share_an_input(bits, M, quantised):
    # q/k/v-like: three layers read ONE x and s (same pointers), so the ahead-of-time transformation keeps
    # one copy for them; a fourth layer with the same K has its own input and (quantised) a fifth shares x
    # with another step.  Not quantised: one layer is wide enough (K >= 16384) to send the whole group through
    # the ahead-of-time route.  Every output against the oracle and against the single calls.
    import torch
    from paper_2506_12038_amd.binding import GemvGroup
    K = 1024 if quantised else 16384
    base = synth.make_layer(2, 0, 64, K, bits, M, seed_offset=1)
    other = synth.make_layer(2, 1, 64, K, bits, M, seed_offset=2)
    x0, s0, x1, s1 = to_dev(base["x"]), to_dev(base["s"]), to_dev(other["x"]), to_dev(other["s"])
    step = lambda L: float(np.float32(np.quantile(np.abs(L["x"].astype(np.float64) / L["s"]), 0.99) / 127.0))
    specs = [(48, x0, s0, base, step(base)), (16, x0, s0, base, step(base)), (80, x0, s0, base, step(base)),
             (32, x1, s1, other, step(other)), (64, x0, s0, base, step(base) * 1.5)]
    problems, refs = [], []
    for i, (N, x, s, src, s_q) in enumerate(specs):
        w = synth.make_layer(2, 10 + i, N, K, bits, 1, seed_offset=i)
        packed = lcd.lcd_pack_indices(to_dev(w["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(w["codebook"]), bits)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        if quantised:
            refs.append((oracle.quantised_lut_matmul(w["codebook"], w["idx"], src["x"], src["s"], s_q, bits),
                         lcd.lcd_lut_gemv_q8(packed, lut, x, s, s_q, N, bits), 1e-3))
        else:
            refs.append((oracle.lut_matmul(w["codebook"], w["idx"], src["x"], src["s"], bits), lcd.lcd_lut_gemv(packed, lut, x, s, N, bits), TOL))
    GemvGroup(problems, bits, s_q=[sp[4] for sp in specs] if quantised else None)()
    torch.cuda.synchronize()
    for p, (Y, single, tol) in zip(problems, refs):
        assert torch.equal(p[4], single)
        assert_parity(p[4].cpu().numpy(), Y, tol)
