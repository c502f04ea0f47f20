"""Helpers for the GPU parity tests: run the HIP path through the Python binding of the C ABI
and the CPU oracle on the same seeded arrays."""
from __future__ import annotations

import numpy as np

import oracle
import paper_2506_12038_amd as lcd

TOL = 2e-3  # max |y - Y| / max(|Y|, rms_n Y): fp16 operands, fp32 accumulation, one fp16 store


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_hip(layer, bits, entry="gemv"):
    """pack -> build_lut -> gemv/gemm, everything on the GPU through the C ABI."""
    import torch
    N, K = layer["idx"].shape
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    x, s = to_dev(layer["x"]), to_dev(layer["s"])
    fn = lcd.lcd_lut_gemv if entry == "gemv" else lcd.lcd_lut_gemm
    # the output starts as NaN: an element the kernels never write fails every comparison
    y = torch.full((x.shape[0], N), float("nan"), dtype=torch.float16, device="cuda")
    fn(packed, lut, x, s, N, bits, y=y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check_layer(layer, bits, entry="gemv", tol=TOL):
    y = run_hip(layer, bits, entry)
    Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
    err = oracle.parity_errors(y, Y)
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert err["max_rel_floored"] <= tol, err
    return err


def assert_parity(y, Y, tol=TOL, what=None):
    """Every element of y against the oracle's Y (NaN or an unwritten element fails)."""
    assert y.shape == Y.shape, (y.shape, Y.shape)
    assert np.all(np.isfinite(y.astype(np.float32))), what
    err = oracle.parity_errors(y, Y)
    assert err["max_rel_floored"] <= tol, (what, err)
    return err


def config_layers(cfg_index, M, distinct_shapes_only):
    """(matrix id, spec, layer) for the matrices of a benchmark config at full size."""
    import synth
    config = synth.get_config(cfg_index)
    seen = set()
    for mid, spec in config.matrices():
        if distinct_shapes_only and (spec.N, spec.K) in seen:
            continue
        seen.add((spec.N, spec.K))
        yield mid, spec, synth.make_layer(cfg_index, mid, spec.N, spec.K, config.bits, M)
