"""ctypes front end of the CPU oracle (oracle/sparse_conv_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module,
and this module never imports the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sparse_conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, so float sums are the
    plain left-to-right ones)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
             "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_f32_to_f16.restype = C.c_uint16
        _lib.oracle_f32_to_f16.argtypes = [C.c_float]
        _lib.oracle_f16_to_f32.restype = C.c_float
        _lib.oracle_f16_to_f32.argtypes = [C.c_uint16]
        _lib.oracle_csr_rowptr.restype = C.c_longlong
        _lib.oracle_codebook_csr.restype = C.c_longlong
        _lib.oracle_unify_mask.restype = C.c_int
        _lib.oracle_output_dim.restype = C.c_int
        _lib.oracle_output_dim.argtypes = [C.c_int] * 4
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def output_dim(size: int, pad: int, filt: int, stride: int) -> int:
    return int(lib().oracle_output_dim(size, pad, filt, stride))


def f32_to_f16_bits(a) -> np.ndarray:
    a = _f32(a)
    out = np.empty(a.shape, dtype=np.uint16)
    lib().oracle_to_f16_bits(_p(a), _p(out), C.c_longlong(a.size))
    return out


def round_through_f16(a) -> np.ndarray:
    a = _f32(a)
    out = np.empty_like(a)
    lib().oracle_round_through_f16(_p(a), _p(out), C.c_longlong(a.size))
    return out


def unify_mask(mask) -> Tuple[np.ndarray, int]:
    """Extended mask (0 dropped / 1 kept / 2 explicit zero) with every row at the
    count of the fullest row, and that count."""
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    K = m.shape[0]
    m2 = m.reshape(K, -1)
    out = np.empty_like(m2)
    target = lib().oracle_unify_mask(_p(m2), K, m2.shape[1], _p(out))
    return out.reshape(m.shape), int(target)


def csr_encode(w, mask) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """CSR (rowptr int32 [K+1], colidx int32 [nnz], values float32 [nnz]) of w*mask."""
    w = _f32(w)
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    K = w.shape[0]
    L = w.size // K
    assert m.size == w.size
    rowptr = np.empty(K + 1, dtype=np.int32)
    nnz = lib().oracle_csr_rowptr(_p(m), K, L, _p(rowptr))
    colidx = np.empty(nnz, dtype=np.int32)
    values = np.empty(nnz, dtype=np.float32)
    lib().oracle_csr_fill(_p(w), _p(m), K, L, _p(colidx), _p(values))
    return rowptr, colidx, values


def codebook_csr_encode(index, centroids, mask):
    """CSR of cluster-quantised weights: (rowptr, colidx, packed 4-bit codes uint8 [ceil(nnz/2)],
    centroid binary16 bits uint16 [16], values float32 [nnz] = centroid of each stored entry).
    mask may hold 0/1/2 (2: explicit zero of the unify step)."""
    idx = np.ascontiguousarray(index, dtype=np.uint8)
    cen = _f32(centroids)
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    assert cen.size == 16 and m.size == idx.size
    K = idx.shape[0]
    L = idx.size // K
    rowptr = np.empty(K + 1, dtype=np.int32)
    nnz = lib().oracle_csr_rowptr(_p(m), K, L, _p(rowptr))
    colidx = np.empty(nnz, dtype=np.int32)
    unused = np.empty(nnz, dtype=np.float32)
    lib().oracle_csr_fill(_p(np.zeros(idx.size, dtype=np.float32)), _p(m), K, L, _p(colidx), _p(unused))
    bits = np.empty(16, dtype=np.uint16)
    packed = np.zeros((nnz + 1) // 2, dtype=np.uint8)
    values = np.empty(nnz, dtype=np.float32)
    got = lib().oracle_codebook_csr(_p(idx), _p(cen), _p(m), K, L, _p(bits), _p(packed), _p(values))
    if got < 0:
        raise ValueError("index above 15" if got == -1 else "an explicit zero needs a zero centroid")
    assert got == nnz
    return rowptr, colidx, packed, bits, values


def sparse_conv(csr, x, K: int, R: int, S: int, stride: int, pad: int,
                acc: str = "f64", want_abs: bool = False):
    """Direct sparse convolution of NCHW x with CSR weights; float32 [N][K][E][F]."""
    rowptr, colidx, values = csr
    x = _f32(x)
    N, Cc, H, W = x.shape
    E, F = output_dim(H, pad, R, stride), output_dim(W, pad, S, stride)
    if E < 0 or F < 0:
        raise ValueError("filter larger than padded input")
    out = np.empty((N, K, E, F), dtype=np.float32)
    aout = np.empty_like(out) if want_abs else None
    rc = lib().oracle_sparse_conv(
        _p(rowptr), _p(colidx), _p(values), _p(x), N, Cc, H, W, K, R, S, stride, pad,
        _p(out), _p(aout) if want_abs else None, 0 if acc == "f64" else 1)
    if rc != 0:
        raise ValueError("oracle_sparse_conv rc=%d" % rc)
    return (out, aout) if want_abs else out


def sparse_conv_points(csr, x, K: int, R: int, S: int, stride: int, pad: int, pts) -> np.ndarray:
    """Exact-order double sums at the output coordinates pts [npts][4] = (n,k,i,j)."""
    rowptr, colidx, values = csr
    x = _f32(x)
    N, Cc, H, W = x.shape
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 4)
    out = np.empty(pts.shape[0], dtype=np.float64)
    rc = lib().oracle_sparse_conv_points(
        _p(rowptr), _p(colidx), _p(values), _p(x), N, Cc, H, W, K, R, S, stride, pad,
        _p(pts), pts.shape[0], _p(out))
    if rc != 0:
        raise ValueError("oracle_sparse_conv_points rc=%d" % rc)
    return out


def dense_conv7(w, mask, x, stride: int, pad: int) -> np.ndarray:
    """Seven-loop dense convolution of w*mask (pin for sparse_conv on small layers)."""
    w = _f32(w)
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    x = _f32(x)
    K, Cc, R, S = w.shape
    N, C2, H, W = x.shape
    assert C2 == Cc
    E, F = output_dim(H, pad, R, stride), output_dim(W, pad, S, stride)
    out = np.empty((N, K, E, F), dtype=np.float32)
    rc = lib().oracle_dense_conv7(_p(w), _p(m), _p(x), N, Cc, H, W, K, R, S, stride, pad, _p(out))
    if rc != 0:
        raise ValueError("oracle_dense_conv7 rc=%d" % rc)
    return out


def relu(x) -> np.ndarray:
    y = _f32(x).copy()
    lib().oracle_relu(_p(y), C.c_longlong(y.size))
    return y


def maxpool2(x) -> np.ndarray:
    x = _f32(x)
    N, Cc, H, W = x.shape
    out = np.empty((N, Cc, H // 2, W // 2), dtype=np.float32)
    lib().oracle_maxpool2(_p(x), C.c_longlong(N * Cc), H, W, _p(out))
    return out
