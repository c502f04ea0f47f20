"""GPU: decode path (lcd_lut_gemv) against the fp64 CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, check_layer, run_hip, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (80, 2304), (256, 4096), (64, 11008), (96, 8192), (32, 28672)])
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
