"""GPU: decode path (lcd_lut_gemv) against the fp64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, check_layer, run_hip, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (80, 2304), (256, 4096), (64, 11008), (96, 8192), (32, 28672), (16, 69632), (1088, 4352), (139264, 512), (64, 5120), (48, 13824)])
def test_gemv_m1_small(bits, shape):
    N, K = shape
    layer = synth.make_layer(0, 0, N, K, bits, 1, variant="B", seed_offset=N + K)
    err = check_layer(layer, bits)
    print(shape, bits, err)


@pytest.mark.parametrize("bits", [2, 3])
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


@pytest.mark.parametrize("bits,M", [(3, 1), (2, 1), (2, 4)])
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


def test_grouped_config1_full_size_sampled():
    import torch
    config = synth.get_config(1)
    problems, layers = [], []
    for mid, spec in config.matrices():
        layer = synth.make_layer(1, mid, spec.N, spec.K, config.bits, 1)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), config.bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), config.bits)
        y = torch.empty((1, spec.N), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), y, spec.N))
        rs = np.sort(np.random.default_rng(mid).choice(spec.N, size=256, replace=False))
        rs[0] = 0; rs[-1] = spec.N - 1
        layers.append((rs, oracle.lut_matmul(layer["codebook"][rs], layer["idx"][rs], layer["x"], layer["s"], config.bits)))
        del layer
    lcd.lcd_lut_gemv_grouped(problems, config.bits)
    torch.cuda.synchronize()
    for (packed, lut, x, s, y, N), (rs, Y) in zip(problems, layers):
        err = oracle.parity_errors(y.cpu().numpy()[:, rs], Y)
        assert err["max_rel_floored"] <= TOL, err


@pytest.mark.parametrize("bits,M", [(3, 1), (2, 16)])
def test_grouped_launch_replayed_from_a_hip_graph(bits, M):
    # the launch configuration bench.py times: the grouped call captured once, replayed several times
    # with eager work and synchronisations in between; every replay must reproduce the eager result
    import torch
    from paper_2506_12038_amd.binding import GemvGroup
    shapes = [(256, 4096), (176, 2816), (64, 11008)]
    problems, eager = [], []
    for i, (N, K) in enumerate(shapes):
        layer = synth.make_layer(1, i, N, K, bits, M, seed_offset=17 * i + bits + M)
        packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
        lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
        x, s = to_dev(layer["x"]), to_dev(layer["s"])
        y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
        problems.append((packed, lut, x, s, y, N))
        Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
        ref = lcd.lcd_lut_gemv(packed, lut, x, s, N, bits)
        assert oracle.parity_errors(ref.cpu().numpy(), Y)["max_rel_floored"] <= TOL
        eager.append(ref)
    group = GemvGroup(problems, bits)
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
