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
    y = fn(packed, lut, x, s, N, bits)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def check_layer(layer, bits, entry="gemv", tol=TOL):
    y = run_hip(layer, bits, entry)
    Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
    err = oracle.parity_errors(y, Y)
    assert np.all(np.isfinite(y.astype(np.float32)))
    assert err["max_rel_floored"] <= tol, err
    return err
