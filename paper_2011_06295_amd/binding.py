"""Thin ctypes binding of libsparseconv.so (include/sparse_conv.h).

Argument marshalling only: every step of direct sparse convolution (CSR
encoding, per-geometry plan, LDS staging, gather-FMA, store) runs inside the
library.  PyTorch appears only as the owner of device buffers and streams.
There is no fallback: if the library is not built, importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

SC_OK, SC_EINVAL, SC_EUNSUPPORTED, SC_ENOMEM, SC_EHIP, SC_ETOOBIG = 0, -1, -2, -3, -4, -5
SC_STATIC_SCRATCH_BYTES = 16 << 20
SC_F32, SC_F16 = 0, 1
SC_FLAG_UNIFY_NNZ = 1
SC_EPILOGUE_RELU = 1
SC_EPILOGUE_MAXPOOL2 = 2

# SPARSECONV_LIBRARY names another build of the same library (e.g. an instrumented one)
LIB_PATH = os.environ.get("SPARSECONV_LIBRARY") or os.path.join(
    os.path.dirname(os.path.abspath(__file__)), "libsparseconv.so")

EXPORTS = (
    "sparse_conv_create", "sparse_conv_output_shape", "sparse_conv_forward", "sparse_conv_forward_static",
    "sparse_conv_get_csr", "sparse_conv_set_launch", "sparse_conv_get_launch", "sparse_conv_set_epilogue", "sparse_conv_autotune",
    "sparse_conv_create_codebook", "sparse_conv_get_codebook", "sparse_conv_check_plan", "sparse_conv_rank_launches",
    "sparse_conv_probe_lds_read", "sparse_conv_probe_copy",
    "sparse_conv_last_hip_error", "sparse_conv_strerror", "sparse_conv_destroy",
)


class SparseConvError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code = code
        self.hip = hip
        msg = _lib.sparse_conv_strerror(code).decode() if _lib is not None else str(code)
        super().__init__(f"{where}: {msg} (status {code}" + (f", hip error {hip})" if hip else ")"))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2011_06295_amd.build` "
            "(there is no CPU fallback)")
    # PyTorch bundles its own HIP runtime (same SONAME as the system one).  It has
    # to be in the process before this library is loaded, so that both resolve to
    # one runtime and device pointers and streams can be shared.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, ip = C.c_void_p, C.POINTER(C.c_int)
    lib.sparse_conv_create.argtypes = [C.POINTER(vp), vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint]
    lib.sparse_conv_create_codebook.argtypes = [C.POINTER(vp), vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                                C.c_uint]
    lib.sparse_conv_get_codebook.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
    lib.sparse_conv_output_shape.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, ip, ip]
    lib.sparse_conv_forward.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp]
    lib.sparse_conv_forward_static.argtypes = lib.sparse_conv_forward.argtypes
    lib.sparse_conv_get_csr.argtypes = [vp, ip, C.POINTER(C.c_longlong), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
    lib.sparse_conv_set_launch.argtypes = [vp, ip, C.c_int]
    lib.sparse_conv_get_launch.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, ip]
    lib.sparse_conv_set_epilogue.argtypes = [vp, vp, C.c_uint]
    lib.sparse_conv_check_plan.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, ip]
    lib.sparse_conv_rank_launches.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, ip, ip]
    lib.sparse_conv_autotune.argtypes = [vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_int,
                                         C.POINTER(C.c_float)]
    lib.sparse_conv_probe_lds_read.argtypes = [vp, C.c_int, C.c_int, vp, C.POINTER(C.c_longlong)]
    lib.sparse_conv_probe_copy.argtypes = [vp, vp, C.c_longlong, vp]
    lib.sparse_conv_last_hip_error.argtypes = [vp]
    lib.sparse_conv_strerror.argtypes = [C.c_int]
    lib.sparse_conv_strerror.restype = C.c_char_p
    lib.sparse_conv_destroy.argtypes = [vp]
    lib.sparse_conv_destroy.restype = None
    for name in EXPORTS:
        if name not in ("sparse_conv_strerror", "sparse_conv_destroy"):
            getattr(lib, name).restype = C.c_int
    return lib


_lib = None
_lib = _load()


def _check(rc: int, where: str, handle=None):
    if rc != SC_OK:
        hip = _lib.sparse_conv_last_hip_error(handle) if handle else 0
        raise SparseConvError(rc, where, hip)


# ---------------------------------------------------------------- same-name functions

def sparse_conv_create(dense_w: np.ndarray, mask: np.ndarray, dtype: int = SC_F32, flags: int = 0) -> int:
    """Handle for the layer with HOST fp32 weights [K][C][R][S] and uint8 mask of the same shape."""
    w = np.ascontiguousarray(dense_w, dtype=np.float32)
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    if w.ndim != 4 or m.shape != w.shape:
        raise ValueError("dense_w and mask must both be [K][C][R][S]")
    K, Cc, R, S = w.shape
    h = C.c_void_p()
    _check(_lib.sparse_conv_create(C.byref(h), w.ctypes.data, m.ctypes.data, K, Cc, R, S, dtype, flags),
           "sparse_conv_create")
    return h.value


def sparse_conv_create_codebook(index: np.ndarray, centroids: np.ndarray, mask: np.ndarray, dtype: int = SC_F32,
                                flags: int = 0) -> int:
    """Handle for a cluster-quantised layer: HOST uint8 centroid numbers [K][C][R][S] (0..15), fp32 centroids [16]
    (stored as binary16) and the uint8 mask."""
    idx = np.ascontiguousarray(index, dtype=np.uint8)
    cen = np.ascontiguousarray(centroids, dtype=np.float32)
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    if idx.ndim != 4 or m.shape != idx.shape or cen.shape != (16,):
        raise ValueError("index and mask must both be [K][C][R][S], centroids [16]")
    K, Cc, R, S = idx.shape
    h = C.c_void_p()
    _check(_lib.sparse_conv_create_codebook(C.byref(h), idx.ctypes.data, cen.ctypes.data, m.ctypes.data, K, Cc, R, S,
                                            dtype, flags), "sparse_conv_create_codebook")
    return h.value


def sparse_conv_get_codebook(handle: int) -> Tuple[np.ndarray, np.ndarray]:
    """(packed 4-bit codes uint8 [(nnz + 1) // 2], centroid binary16 bits uint16 [16]) of a codebook handle (copies)."""
    nnz = C.c_longlong()
    _check(_lib.sparse_conv_get_csr(handle, None, C.byref(nnz), None, None, None), "sparse_conv_get_csr", handle)
    codes, cen = C.c_void_p(), C.c_void_p()
    _check(_lib.sparse_conv_get_codebook(handle, C.byref(codes), C.byref(cen)), "sparse_conv_get_codebook", handle)
    nbytes = (nnz.value + 1) // 2
    packed = np.ctypeslib.as_array(C.cast(codes, C.POINTER(C.c_uint8)), (nbytes,)).copy() if nbytes else np.zeros(0, np.uint8)
    bits = np.ctypeslib.as_array(C.cast(cen, C.POINTER(C.c_uint16)), (16,)).copy()
    return packed, bits


def sparse_conv_output_shape(handle: int, H: int, W: int, stride: int, pad: int) -> Tuple[int, int]:
    e, f = C.c_int(), C.c_int()
    _check(_lib.sparse_conv_output_shape(handle, H, W, stride, pad, C.byref(e), C.byref(f)),
           "sparse_conv_output_shape", handle)
    return e.value, f.value


def sparse_conv_forward(handle: int, input_ptr: int, output_ptr: int, N: int, H: int, W: int,
                        stride: int, pad: int, stream: int = 0) -> None:
    """Enqueue the convolution of DEVICE input [N][C][H][W] into DEVICE output [N][K][E][F]."""
    _check(_lib.sparse_conv_forward(handle, input_ptr, output_ptr, N, H, W, stride, pad, stream or None),
           "sparse_conv_forward", handle)


def sparse_conv_forward_static(handle: int, input_ptr: int, output_ptr: int, N: int, H: int, W: int,
                               stride: int, pad: int, stream: int = 0) -> None:
    """sparse_conv_forward without any device allocation: the layer's tables go through the GPU's static scratch."""
    _check(_lib.sparse_conv_forward_static(handle, input_ptr, output_ptr, N, H, W, stride, pad, stream or None),
           "sparse_conv_forward_static", handle)


def sparse_conv_get_csr(handle: int, dtype: int):
    """Copies of (rowptr int32, colidx int32, values float32|uint16 patterns)."""
    K, nnz = C.c_int(), C.c_longlong()
    rp, ci, va = C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(_lib.sparse_conv_get_csr(handle, C.byref(K), C.byref(nnz), C.byref(rp), C.byref(ci), C.byref(va)),
           "sparse_conv_get_csr", handle)
    n = nnz.value

    def arr(ptr, count, ctype, npdtype):
        if count == 0 or not ptr.value:
            return np.empty(0, dtype=npdtype)
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(ctype)), shape=(count,)).astype(npdtype, copy=True)

    rowptr = arr(rp, K.value + 1, C.c_int, np.int32)
    colidx = arr(ci, n, C.c_int, np.int32)
    values = arr(va, n, C.c_uint16, np.uint16) if dtype == SC_F16 else arr(va, n, C.c_float, np.float32)
    return rowptr, colidx, values


def sparse_conv_set_launch(handle: int, params: Sequence[int]) -> None:
    arr = (C.c_int * max(1, len(params)))(*params)
    _check(_lib.sparse_conv_set_launch(handle, arr, len(params)), "sparse_conv_set_launch", handle)


def sparse_conv_set_epilogue(handle: int, bias: Optional[np.ndarray], flags: int = 0) -> None:
    """bias: HOST fp32 [K] or None; flags: 0 or any of SC_EPILOGUE_RELU, SC_EPILOGUE_MAXPOOL2."""
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    ptr = None if b is None else b.ctypes.data_as(C.c_void_p)
    _check(_lib.sparse_conv_set_epilogue(handle, ptr, C.c_uint(flags)), "sparse_conv_set_epilogue", handle)


def sparse_conv_autotune(handle: int, input_ptr: int, output_ptr: int, N: int, H: int, W: int, stride: int, pad: int,
                         stream: int = 0, max_candidates: int = 0) -> float:
    """Measures the best-ranked launch configurations on the given device buffers; returns the kept one's us per launch."""
    us = C.c_float(0.0)
    _check(_lib.sparse_conv_autotune(handle, input_ptr, output_ptr, N, H, W, stride, pad, stream, max_candidates,
                                     C.byref(us)), "sparse_conv_autotune", handle)
    return float(us.value)


def sparse_conv_get_launch(handle: int, N: int, H: int, W: int, stride: int, pad: int) -> dict:
    arr = (C.c_int * 16)()
    _check(_lib.sparse_conv_get_launch(handle, N, H, W, stride, pad, arr), "sparse_conv_get_launch", handle)
    names = ("V", "WP", "WK", "KW", "Cc", "lds_budget", "grid", "lds_bytes", "threads", "entries", "LP", "kblocks", "store",
             "lanes", "csplit", "entry_bytes")
    return dict(zip(names, list(arr)))


def sparse_conv_rank_launches(handle: int, N: int, H: int, W: int, stride: int, pad: int, max_candidates: int = 8):
    """The best-ranked launch configurations for a geometry, each a list of 11 ints that sparse_conv_set_launch takes."""
    arr = (C.c_int * (11 * max_candidates))()
    n = C.c_int(0)
    _check(_lib.sparse_conv_rank_launches(handle, N, H, W, stride, pad, max_candidates, arr, C.byref(n)),
           "sparse_conv_rank_launches", handle)
    return [list(arr[11 * i:11 * i + 11]) for i in range(n.value)]


def sparse_conv_check_plan(handle: int, N: int, H: int, W: int, stride: int, pad: int) -> int:
    """Host-side consistency check of the geometry's plan: 0, or the number of the first failed check."""
    bad = C.c_int(-1)
    _check(_lib.sparse_conv_check_plan(handle, N, H, W, stride, pad, C.byref(bad)), "sparse_conv_check_plan", handle)
    return int(bad.value)


def sparse_conv_probe_lds_read(sink_ptr: int, workgroups: int, iterations: int, stream: int = 0) -> int:
    """Enqueues the LDS read probe; returns the LDS bytes the launch reads."""
    n = C.c_longlong(0)
    _check(_lib.sparse_conv_probe_lds_read(sink_ptr, workgroups, iterations, stream or None, C.byref(n)),
           "sparse_conv_probe_lds_read")
    return int(n.value)


def sparse_conv_probe_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    """Enqueues the copy probe (nbytes read, nbytes written)."""
    _check(_lib.sparse_conv_probe_copy(dst_ptr, src_ptr, nbytes, stream or None), "sparse_conv_probe_copy")


def sparse_conv_destroy(handle: Optional[int]) -> None:
    _lib.sparse_conv_destroy(handle)


def raw_library():
    """The loaded ctypes library (for tests of the raw ABI)."""
    return _lib


# ---------------------------------------------------------------- convenience wrapper

class SparseConv:
    """One pruned convolution layer on the GPU; owns a library handle."""

    def __init__(self, dense_w: np.ndarray, mask: np.ndarray, dtype: str = "f32", unify: bool = False):
        self.dtype = SC_F16 if dtype in ("f16", SC_F16) else SC_F32
        self.K, self.C, self.R, self.S = dense_w.shape
        self.handle = sparse_conv_create(dense_w, mask, self.dtype, SC_FLAG_UNIFY_NNZ if unify else 0)

    @classmethod
    def from_codebook(cls, index: np.ndarray, centroids: np.ndarray, mask: np.ndarray, dtype: str = "f32",
                      unify: bool = False) -> "SparseConv":
        """A layer whose weights are 4-bit centroid numbers into 16 binary16 centroids."""
        self = cls.__new__(cls)
        self.dtype = SC_F16 if dtype in ("f16", SC_F16) else SC_F32
        self.K, self.C, self.R, self.S = index.shape
        self.handle = sparse_conv_create_codebook(index, centroids, mask, self.dtype, SC_FLAG_UNIFY_NNZ if unify else 0)
        return self

    def csr(self):
        return sparse_conv_get_csr(self.handle, self.dtype)

    def codebook(self):
        return sparse_conv_get_codebook(self.handle)

    def output_shape(self, H: int, W: int, stride: int = 1, pad: int = 0):
        return sparse_conv_output_shape(self.handle, H, W, stride, pad)

    def check_plan(self, N: int, H: int, W: int, stride: int = 1, pad: int = 0) -> int:
        return sparse_conv_check_plan(self.handle, N, H, W, stride, pad)

    def rank_launches(self, N: int, H: int, W: int, stride: int = 1, pad: int = 0, max_candidates: int = 8):
        return sparse_conv_rank_launches(self.handle, N, H, W, stride, pad, max_candidates)

    def set_launch(self, params: Sequence[int]):
        sparse_conv_set_launch(self.handle, params)

    def set_epilogue(self, bias: Optional[np.ndarray] = None, relu: bool = False, maxpool: bool = False):
        sparse_conv_set_epilogue(self.handle, bias, (SC_EPILOGUE_RELU if relu else 0) | (SC_EPILOGUE_MAXPOOL2 if maxpool else 0))
        self._shapes = {}    # the output shape of a geometry depends on the pooling flag

    def get_launch(self, N, H, W, stride=1, pad=0):
        return sparse_conv_get_launch(self.handle, N, H, W, stride, pad)

    def _buffers(self, x, stride, pad, out):
        import torch
        want = torch.float16 if self.dtype == SC_F16 else torch.float32
        if not x.is_cuda or x.dtype != want or not x.is_contiguous() or x.dim() != 4 or x.shape[1] != self.C:
            raise ValueError("input must be a contiguous CUDA tensor [N][C][H][W] of the layer's dtype")
        N, _, H, W = x.shape
        try:      # the output shape of a geometry is asked of the library once (a forward call is a few microseconds)
            E, F = self._shapes[(H, W, stride, pad)]
        except (AttributeError, KeyError):
            if not hasattr(self, "_shapes"):
                self._shapes = {}
            E, F = self._shapes[(H, W, stride, pad)] = self.output_shape(H, W, stride, pad)
        if out is None:
            out = torch.empty((N, self.K, E, F), dtype=want, device=x.device)
        elif out.shape != (N, self.K, E, F) or out.dtype != want or not out.is_contiguous():
            raise ValueError("bad output tensor")
        return out, (N, H, W, stride, pad), torch.cuda.current_stream(x.device).cuda_stream

    def autotune(self, x, stride: int = 1, pad: int = 0, out=None, max_candidates: int = 0) -> float:
        """Picks the launch configuration for x's geometry by measurement (overwrites out); returns its us per launch."""
        out, geom, stream = self._buffers(x, stride, pad, out)
        return sparse_conv_autotune(self.handle, x.data_ptr(), out.data_ptr(), *geom, stream, max_candidates)

    def forward(self, x, stride: int = 1, pad: int = 0, out=None):
        """x: contiguous CUDA tensor [N][C][H][W] of the layer's dtype; returns [N][K][E][F]."""
        out, geom, stream = self._buffers(x, stride, pad, out)
        sparse_conv_forward(self.handle, x.data_ptr(), out.data_ptr(), *geom, stream)
        return out

    def prepare(self, x, stride: int = 1, pad: int = 0, out=None):
        """Checks the tensors once and returns a function without arguments that enqueues this convolution of x
        into out on the stream that is current now (its attribute `out` is the output tensor).  For loops that
        repeat a call on the same buffers: what is left per call is the library call itself."""
        out, geom, stream = self._buffers(x, stride, pad, out)
        fn, h, xp, op, st = _lib.sparse_conv_forward, self.handle, x.data_ptr(), out.data_ptr(), stream or None

        def enqueue(_keep=(x, out)):
            rc = fn(h, xp, op, *geom, st)
            if rc:
                _check(rc, "sparse_conv_forward", h)

        enqueue.out = out
        return enqueue

    def forward_static(self, x, stride: int = 1, pad: int = 0, out=None):
        """forward for callers that cannot allocate device memory (`out` should then be given)."""
        out, geom, stream = self._buffers(x, stride, pad, out)
        sparse_conv_forward_static(self.handle, x.data_ptr(), out.data_ptr(), *geom, stream)
        return out

    def close(self):
        if getattr(self, "handle", None):
            sparse_conv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
