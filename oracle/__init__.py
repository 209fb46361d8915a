"""CPU oracle: the plain definitions the HIP library is checked against.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg; the library and its Python binding never import it, and it imports neither
of them.  The C part (conv_oracle.c, gemm_oracle.c) is compiled by oracle/build.py.
"""
import ctypes
import os
import numpy as np

from . import build as _build
from .layouts import nchw_to_nchwc, nchwc_to_nchw, kcrs_to_kcrsck, kcrsck_to_kcrs  # noqa: F401
from .elementwise import bias_add, relu, relu6, bnorm_inference  # noqa: F401

ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2
_ACT = {None: 0, "none": 0, "relu": 1, "relu6": 2, 0: 0, 1: 1, 2: 2, False: 0, True: 1}

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        i, i64, dbl, ptr = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        _lib.oracle_conv2d_fwd.argtypes = [i] * 9 + [ptr, ptr, ptr, i, ptr, ptr]
        _lib.oracle_conv2d_fwd_at.argtypes = [i] * 9 + [ptr, ptr, ptr, i, i64, ptr, ptr, ptr]
        _lib.oracle_gemm.argtypes = [i64] * 3 + [ptr, ptr, ptr, dbl, dbl, ptr, ptr]
        _lib.oracle_gemm_at.argtypes = [i64] * 3 + [ptr, ptr, ptr, dbl, dbl, i64, ptr, ptr, ptr]
        for f in (_lib.oracle_conv2d_fwd, _lib.oracle_conv2d_fwd_at, _lib.oracle_gemm,
                  _lib.oracle_gemm_at):
            f.restype = i
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def conv2d_fwd(x, w, bias=None, stride=1, pad=0, act=None, at=None):
    """Forward convolution of x (NCHW) with w (KCRS); see conv_oracle.c for the definition.

    Returns (out, absum) as float64: the NKPQ tensor, or, when ``at`` lists flat NKPQ indices,
    only those elements.  float32 inputs are widened exactly (bf16 data is passed already widened).
    """
    lib = _load()
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    b = None if bias is None else _f32(bias)
    if b is not None and b.shape != (K,):
        raise ValueError("bias shape")
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    if at is None:
        out = np.empty((N, K, P, Q), dtype=np.float64)
        ab = np.empty_like(out)
        rc = lib.oracle_conv2d_fwd(N, C, H, W, K, R, S, stride, pad, _p(x), _p(w), _p(b),
                                   _ACT[act], _p(out), _p(ab))
    else:
        idx = np.ascontiguousarray(at, dtype=np.int64)
        out = np.empty(idx.shape, dtype=np.float64)
        ab = np.empty_like(out)
        rc = lib.oracle_conv2d_fwd_at(N, C, H, W, K, R, S, stride, pad, _p(x), _p(w), _p(b),
                                      _ACT[act], idx.size, _p(idx), _p(out), _p(ab))
    if rc != 0:
        raise ValueError("oracle_conv2d_fwd rejected the shape (rc=%d)" % rc)
    return out, ab


def gemm(A, B, C0=None, alpha=1.0, beta=1.0, at=None):
    """C = beta*C0 + alpha*A@B in float64 (k ascending); returns (C, absum).  See gemm_oracle.c."""
    lib = _load()
    A, B = _f32(A), _f32(B)
    M, K = A.shape
    K2, N = B.shape
    if K2 != K:
        raise ValueError("inner dimension mismatch")
    c0 = None if C0 is None else _f32(C0)
    if c0 is not None and c0.shape != (M, N):
        raise ValueError("C0 shape")
    if at is None:
        C = np.empty((M, N), dtype=np.float64)
        ab = np.empty_like(C)
        rc = lib.oracle_gemm(M, N, K, _p(A), _p(B), _p(c0), alpha, beta, _p(C), _p(ab))
    else:
        idx = np.ascontiguousarray(at, dtype=np.int64)
        C = np.empty(idx.shape, dtype=np.float64)
        ab = np.empty_like(C)
        rc = lib.oracle_gemm_at(M, N, K, _p(A), _p(B), _p(c0), alpha, beta, idx.size, _p(idx),
                                _p(C), _p(ab))
    if rc != 0:
        raise ValueError("oracle_gemm rejected the shape (rc=%d)" % rc)
    return C, ab


def scaled_error(got, want, absum):
    """The parity metric: max over outputs of |got - want| / absum, where absum is the sum of the
    magnitudes of the terms that make up the output.  Where absum is 0 the output must be 0."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    absum = np.asarray(absum, dtype=np.float64)
    diff = np.abs(got - want)
    zero = absum == 0
    if np.any(diff[zero] != 0):
        return float("inf")
    if np.all(zero):
        return 0.0
    return float(np.max(diff[~zero] / absum[~zero]))
