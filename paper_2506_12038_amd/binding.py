"""Thin Python binding of the C ABI in include/lcd.h: argument marshalling only.

Every step of the path runs in the HIP library; this file only turns torch tensors into
pointers and sizes, allocates outputs with torch (device memory is PyTorch's job here), and
turns a status code into an exception.  There is no CPU fallback: if liblcd.so is missing
the import of a function fails loudly.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "liblcd.so"
_lib = None

EXPORTS = (
    "lcd_version", "lcd_layout_revision", "lcd_last_error_string", "lcd_status_string",
    "lcd_packed_bytes", "lcd_lut_bytes", "lcd_workspace_bytes",
    "lcd_pack_indices", "lcd_unpack_indices", "lcd_pack_indices_host", "lcd_unpack_indices_host",
    "lcd_build_lut", "lcd_lut_gemv", "lcd_lut_gemm", "lcd_lut_gemv_q8", "lcd_lut_gemv_noalloc",
    "lcd_workspace_bytes_grouped", "lcd_lut_gemv_grouped", "lcd_lut_gemv_q8_grouped", "lcd_lut_gemv_grouped_mixed",
    "lcd_workspace_bytes_gemm_grouped", "lcd_lut_gemm_grouped", "lcd_lut_gemm_q8", "lcd_lut_gemm_q8_grouped",
    "lcd_assign_indices", "lcd_cluster_counts", "lcd_merge_closest",
)


class _Problem(ctypes.Structure):
    _fields_ = [("packed", ctypes.c_void_p), ("lut", ctypes.c_void_p), ("x", ctypes.c_void_p), ("s", ctypes.c_void_p),
                ("y", ctypes.c_void_p), ("N", ctypes.c_int), ("K", ctypes.c_int)]


class LcdError(RuntimeError):
    def __init__(self, status: int, name: str, message: str):
        super().__init__(f"{name} ({status}): {message}")
        self.status = status
        self.name = name


def load_library():
    """dlopen liblcd.so (built by paper_2506_12038_amd/build.py).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2506_12038_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(str(LIB_PATH))
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.lcd_version.restype = ci
    lib.lcd_layout_revision.restype = ci
    lib.lcd_last_error_string.restype = ctypes.c_char_p
    lib.lcd_status_string.restype = ctypes.c_char_p
    lib.lcd_status_string.argtypes = [ci]
    lib.lcd_packed_bytes.restype = sz
    lib.lcd_packed_bytes.argtypes = [ci, ci, ci]
    lib.lcd_lut_bytes.restype = sz
    lib.lcd_lut_bytes.argtypes = [ci, ci]
    lib.lcd_workspace_bytes.restype = sz
    lib.lcd_workspace_bytes.argtypes = [ci, ci, ci, ci]
    lib.lcd_pack_indices.restype = ci
    lib.lcd_pack_indices.argtypes = [vp, ci, ci, ci, vp, sz, vp]
    lib.lcd_unpack_indices.restype = ci
    lib.lcd_unpack_indices.argtypes = [vp, ci, ci, ci, vp, vp]
    lib.lcd_pack_indices_host.restype = ci
    lib.lcd_pack_indices_host.argtypes = [vp, ci, ci, ci, vp, sz]
    lib.lcd_unpack_indices_host.restype = ci
    lib.lcd_unpack_indices_host.argtypes = [vp, ci, ci, ci, vp]
    lib.lcd_build_lut.restype = ci
    lib.lcd_build_lut.argtypes = [vp, ci, ci, vp, sz, vp]
    for name in ("lcd_lut_gemv", "lcd_lut_gemm"):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, vp, sz, vp]
    lib.lcd_lut_gemv_noalloc.restype = ci
    lib.lcd_lut_gemv_noalloc.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    for name in ("lcd_lut_gemv_q8", "lcd_lut_gemm_q8"):
        fn = getattr(lib, name)
        fn.restype = ci
        fn.argtypes = [vp, vp, vp, vp, ctypes.c_float, vp, ci, ci, ci, ci, vp, sz, vp]
    lib.lcd_lut_gemm_q8_grouped.restype = ci
    lib.lcd_lut_gemm_q8_grouped.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(ctypes.c_float), ci, ci, ci, vp, sz, vp]
    lib.lcd_workspace_bytes_grouped.restype = sz
    lib.lcd_workspace_bytes_grouped.argtypes = [ctypes.POINTER(_Problem), ci, ci, ci]
    lib.lcd_lut_gemv_grouped.restype = ci
    lib.lcd_lut_gemv_grouped.argtypes = [ctypes.POINTER(_Problem), ci, ci, ci, vp, sz, vp]
    lib.lcd_workspace_bytes_gemm_grouped.restype = sz
    lib.lcd_workspace_bytes_gemm_grouped.argtypes = [ctypes.POINTER(_Problem), ci, ci, ci]
    lib.lcd_lut_gemm_grouped.restype = ci
    lib.lcd_lut_gemm_grouped.argtypes = [ctypes.POINTER(_Problem), ci, ci, ci, vp, sz, vp]
    lib.lcd_lut_gemv_q8_grouped.restype = ci
    lib.lcd_lut_gemv_q8_grouped.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(ctypes.c_float), ci, ci, ci, vp, sz, vp]
    lib.lcd_lut_gemv_grouped_mixed.restype = ci
    lib.lcd_lut_gemv_grouped_mixed.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(ci), ci, ci, vp, sz, vp]
    lib.lcd_assign_indices.restype = ci
    lib.lcd_assign_indices.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    lib.lcd_cluster_counts.restype = ci
    lib.lcd_cluster_counts.argtypes = [vp, ci, ci, ci, vp, vp]
    lib.lcd_merge_closest.restype = ci
    lib.lcd_merge_closest.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp, vp, vp, vp]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        lib = load_library()
        raise LcdError(status, lib.lcd_status_string(status).decode(), lib.lcd_last_error_string().decode())


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t, dtype, name):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")
    return ctypes.c_void_p(t.data_ptr())


def lcd_version() -> int:
    return load_library().lcd_version()


def lcd_layout_revision() -> int:
    return load_library().lcd_layout_revision()


def lcd_packed_bytes(N: int, K: int, bits: int) -> int:
    return load_library().lcd_packed_bytes(N, K, bits)


def lcd_lut_bytes(N: int, bits: int) -> int:
    return load_library().lcd_lut_bytes(N, bits)


def lcd_workspace_bytes(M: int, N: int, K: int, bits: int) -> int:
    return load_library().lcd_workspace_bytes(M, N, K, bits)


def lcd_pack_indices(idx, bits: int, out=None, stream=None):
    """idx: CUDA uint8 [N, K] -> packed CUDA uint8 [N*K*bits/8]."""
    import torch
    lib = load_library()
    N, K = idx.shape
    nbytes = lib.lcd_packed_bytes(N, K, bits)
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=idx.device)
    _check(lib.lcd_pack_indices(_dev(idx, torch.uint8, "idx"), N, K, bits, _dev(out, torch.uint8, "packed"),
                                out.numel(), _stream(stream)))
    return out[:nbytes] if nbytes else out[:0]


def lcd_unpack_indices(packed, N: int, K: int, bits: int, stream=None):
    import torch
    lib = load_library()
    idx = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib.lcd_unpack_indices(_dev(packed, torch.uint8, "packed"), N, K, bits, _dev(idx, torch.uint8, "idx"),
                                  _stream(stream)))
    return idx


def lcd_pack_indices_host(idx, bits: int):
    """numpy uint8 [N, K] -> numpy uint8 packed bytes (no GPU needed)."""
    import numpy as np
    lib = load_library()
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    N, K = idx.shape
    nbytes = lib.lcd_packed_bytes(N, K, bits)
    out = np.zeros(max(nbytes, 1), dtype=np.uint8)
    _check(lib.lcd_pack_indices_host(idx.ctypes.data_as(ctypes.c_void_p), N, K, bits,
                                     out.ctypes.data_as(ctypes.c_void_p), nbytes))
    return out[:nbytes]


def lcd_unpack_indices_host(packed, N: int, K: int, bits: int):
    import numpy as np
    lib = load_library()
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    need = lib.lcd_packed_bytes(N, K, bits)
    if need and packed.size < need:
        raise ValueError("packed buffer too small")
    idx = np.empty((N, K), dtype=np.uint8)
    _check(lib.lcd_unpack_indices_host(packed.ctypes.data_as(ctypes.c_void_p), N, K, bits,
                                       idx.ctypes.data_as(ctypes.c_void_p)))
    return idx


def lcd_build_lut(codebook, bits: int, stream=None):
    """codebook: CUDA float16 [N, 2**bits] -> opaque CUDA uint8 table."""
    import torch
    lib = load_library()
    N = codebook.shape[0]
    if codebook.shape[1] != (1 << bits):
        raise ValueError("codebook must be [N, 2**bits]")
    nbytes = lib.lcd_lut_bytes(N, bits)
    lut = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=codebook.device)
    _check(lib.lcd_build_lut(_dev(codebook, torch.float16, "codebook"), N, bits, _dev(lut, torch.uint8, "lut"),
                             lut.numel(), _stream(stream)))
    return lut


def _product(fn_name, packed, lut, x, s, N, bits, y, workspace, stream):
    import torch
    lib = load_library()
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(lib.lcd_workspace_bytes(M, N, K, bits), 256), dtype=torch.uint8, device=x.device)
    _check(getattr(lib, fn_name)(
        _dev(packed, torch.uint8, "packed"), _dev(lut, torch.uint8, "lut"), _dev(x, torch.float16, "x"),
        _dev(s, torch.float32, "s"), _dev(y, torch.float16, "y"), M, N, K, bits,
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))
    return y


def lcd_lut_gemv(packed, lut, x, s, N: int, bits: int, y=None, workspace=None, stream=None):
    """Decode path, x: CUDA float16 [M<=16, K] -> y float16 [M, N]."""
    return _product("lcd_lut_gemv", packed, lut, x, s, N, bits, y, workspace, stream)


def lcd_lut_gemv_noalloc(packed, lut, x, s, N: int, bits: int, y, stream=None):
    """lcd_lut_gemv without a workspace: the library's own static device array serves as scratch.
    The caller brings y (this wrapper allocates nothing either)."""
    import torch
    M, K = x.shape
    _check(load_library().lcd_lut_gemv_noalloc(
        _dev(packed, torch.uint8, "packed"), _dev(lut, torch.uint8, "lut"), _dev(x, torch.float16, "x"),
        _dev(s, torch.float32, "s"), _dev(y, torch.float16, "y"), M, N, K, bits, _stream(stream)))
    return y


def lcd_lut_gemv_q8(packed, lut, x, s, s_q: float, N: int, bits: int, y=None, workspace=None, stream=None):
    """Decode path with the INT8 input transformation in front: y = s_q * sum_k q_k * C[n][idx], M <= 16."""
    return _product_q8("lcd_lut_gemv_q8", packed, lut, x, s, s_q, N, bits, y, workspace, stream)


def lcd_lut_gemm_q8(packed, lut, x, s, s_q: float, N: int, bits: int, y=None, workspace=None, stream=None):
    """Prefill path with the INT8 input transformation in front (any M)."""
    return _product_q8("lcd_lut_gemm_q8", packed, lut, x, s, s_q, N, bits, y, workspace, stream)


def _product_q8(fn_name, packed, lut, x, s, s_q, N, bits, y, workspace, stream):
    import torch
    lib = load_library()
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(lib.lcd_workspace_bytes(M, N, K, bits), 256), dtype=torch.uint8, device=x.device)
    _check(getattr(lib, fn_name)(
        _dev(packed, torch.uint8, "packed"), _dev(lut, torch.uint8, "lut"), _dev(x, torch.float16, "x"),
        _dev(s, torch.float32, "s"), float(s_q), _dev(y, torch.float16, "y"), M, N, K, bits,
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)))
    return y


def lcd_lut_gemm(packed, lut, x, s, N: int, bits: int, y=None, workspace=None, stream=None):
    """Prefill path, x: CUDA float16 [M, K] -> y float16 [M, N]."""
    return _product("lcd_lut_gemm", packed, lut, x, s, N, bits, y, workspace, stream)


class GemvGroup:
    """Marshalled argument block of lcd_lut_gemv_grouped: build once per layer set, call many times.

    problems: sequence of (packed, lut, x, s, y, N) with CUDA tensors as in lcd_lut_gemv.
    bits: one index width for all layers, or a sequence with one width per layer
          (lcd_lut_gemv_grouped_mixed).
    s_q: optional sequence of per-layer activation quantisation steps (lcd_lut_gemv_q8_grouped).
    """

    def __init__(self, problems, bits: int, workspace=None, s_q=None):
        import torch
        lib = load_library()
        self.count = len(problems)
        self._bits_arr = None
        if not isinstance(bits, int):
            if len(bits) != self.count:
                raise ValueError("one index width per problem")
            if s_q is not None:
                raise ValueError("mixed index widths and quantised activations are separate entry points")
            self._bits_arr = (ctypes.c_int * self.count)(*[int(b) for b in bits])
            bits = int(bits[0])     # the workspace size does not depend on the width
        self.bits = bits
        self._keep = list(problems)
        M = problems[0][2].shape[0]
        self.M = M
        arr = (_Problem * self.count)()
        for i, (packed, lut, x, s, y, N) in enumerate(problems):
            if x.shape[0] != M:
                raise ValueError("all problems of a group share M")
            K = x.shape[1]
            arr[i] = _Problem(_dev(packed, torch.uint8, "packed").value, _dev(lut, torch.uint8, "lut").value,
                              _dev(x, torch.float16, "x").value, _dev(s, torch.float32, "s").value,
                              _dev(y, torch.float16, "y").value, N, K)
        self._arr = arr
        self._s_q = None
        if s_q is not None:
            if len(s_q) != self.count:
                raise ValueError("one s_q per problem")
            self._s_q = (ctypes.c_float * self.count)(*[float(v) for v in s_q])
        need = lib.lcd_workspace_bytes_grouped(arr, self.count, M, bits)
        if need == 0:
            raise ValueError("invalid group (shapes, M or bits)")
        self.workspace = workspace if workspace is not None else torch.empty(need, dtype=torch.uint8, device=problems[0][2].device)

    def __call__(self, stream=None):
        import torch
        ws = _dev(self.workspace, torch.uint8, "workspace")
        if self._bits_arr is not None:
            _check(load_library().lcd_lut_gemv_grouped_mixed(self._arr, self._bits_arr, self.count, self.M, ws,
                                                             self.workspace.numel(), _stream(stream)))
        elif self._s_q is None:
            _check(load_library().lcd_lut_gemv_grouped(self._arr, self.count, self.M, self.bits, ws, self.workspace.numel(),
                                                       _stream(stream)))
        else:
            _check(load_library().lcd_lut_gemv_q8_grouped(self._arr, self._s_q, self.count, self.M, self.bits, ws,
                                                          self.workspace.numel(), _stream(stream)))


class GemmGroup:
    """Marshalled argument block of lcd_lut_gemm_grouped (prefill, several layers, one pair of launches):
    problems = [(packed, lut, x, s, y, N), ...] with one token count and one index width."""

    def __init__(self, problems, bits: int, workspace=None, s_q=None):
        import torch
        lib = load_library()
        self.count, self.bits = len(problems), bits
        self._keep = list(problems)
        self.M = problems[0][2].shape[0]
        self._s_q = None
        if s_q is not None:      # one activation quantisation step per layer: lcd_lut_gemm_q8_grouped
            if len(s_q) != self.count:
                raise ValueError("one s_q per problem")
            self._s_q = (ctypes.c_float * self.count)(*[float(v) for v in s_q])
        arr = (_Problem * self.count)()
        for i, (packed, lut, x, s, y, N) in enumerate(problems):
            if x.shape[0] != self.M:
                raise ValueError("all problems of a group share M")
            arr[i] = _Problem(_dev(packed, torch.uint8, "packed").value, _dev(lut, torch.uint8, "lut").value,
                              _dev(x, torch.float16, "x").value, _dev(s, torch.float32, "s").value,
                              _dev(y, torch.float16, "y").value, N, x.shape[1])
        self._arr = arr
        need = lib.lcd_workspace_bytes_gemm_grouped(arr, self.count, self.M, bits)
        if need == 0:
            raise ValueError("invalid group (shapes, M or bits)")
        self.workspace = workspace if workspace is not None else torch.empty(need, dtype=torch.uint8, device=problems[0][2].device)

    def __call__(self, stream=None):
        import torch
        ws = _dev(self.workspace, torch.uint8, "workspace")
        if self._s_q is None:
            _check(load_library().lcd_lut_gemm_grouped(self._arr, self.count, self.M, self.bits, ws, self.workspace.numel(), _stream(stream)))
        else:
            _check(load_library().lcd_lut_gemm_q8_grouped(self._arr, self._s_q, self.count, self.M, self.bits, ws,
                                                          self.workspace.numel(), _stream(stream)))


def lcd_lut_gemm_grouped(problems, bits: int, workspace=None, stream=None):
    """Prefill for several layers at once: problems = [(packed, lut, x, s, y, N), ...]; writes every y."""
    GemmGroup(problems, bits, workspace)(stream)


def lcd_workspace_bytes_grouped(problems, bits: int) -> int:
    return GemvGroup(problems, bits).workspace.numel()


def lcd_lut_gemv_grouped(problems, bits: int, workspace=None, stream=None):
    """One launch for several layers: problems = [(packed, lut, x, s, y, N), ...]; writes every y."""
    GemvGroup(problems, bits, workspace)(stream)


def lcd_assign_indices(w, codebook, ncent: int, bits: int, stream=None):
    """w: CUDA float16 [N, K], codebook: CUDA float16 [N, 2**bits] -> CUDA uint8 [N, K] nearest-centroid indices."""
    import torch
    N, K = w.shape
    if tuple(codebook.shape) != (N, 1 << bits):
        raise ValueError("codebook must be [N, 2**bits]")
    idx = torch.empty((N, K), dtype=torch.uint8, device=w.device)
    _check(load_library().lcd_assign_indices(_dev(w, torch.float16, "w"), _dev(codebook, torch.float16, "codebook"), ncent,
                                             N, K, bits, _dev(idx, torch.uint8, "idx"), _stream(stream)))
    return idx


def lcd_cluster_counts(idx, bits: int, stream=None):
    """idx: CUDA uint8 [N, K] -> CUDA int32 [N, 2**bits] cluster sizes (the bit patterns are uint32)."""
    import torch
    N, K = idx.shape
    counts = torch.empty((N, 1 << bits), dtype=torch.int32, device=idx.device)
    _check(load_library().lcd_cluster_counts(_dev(idx, torch.uint8, "idx"), N, K, bits, _dev(counts, torch.int32, "counts"),
                                             _stream(stream)))
    return counts


def lcd_merge_closest(codebook, counts, idx, ncent: int, bits: int, idx_out=None, stream=None):
    """Merge the two closest centroids of every row; returns (codebook_out, idx_out, merged)."""
    import torch
    N, K = idx.shape
    cb_out = torch.empty_like(codebook)
    if idx_out is None:
        idx_out = torch.empty_like(idx)
    merged = torch.empty((N,), dtype=torch.uint8, device=idx.device)
    _check(load_library().lcd_merge_closest(_dev(codebook, torch.float16, "codebook"), _dev(counts, torch.int32, "counts"),
                                            _dev(idx, torch.uint8, "idx"), ncent, N, K, bits,
                                            _dev(cb_out, torch.float16, "codebook_out"), _dev(idx_out, torch.uint8, "idx_out"),
                                            _dev(merged, torch.uint8, "merged"), _stream(stream)))
    return cb_out, idx_out, merged
