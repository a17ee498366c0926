"""CPU oracle (test infrastructure only).

Thin ctypes wrapper over ``oracle.c``: plain nested-loop definitions of the fp32 GEMM
(Section 2.1, Fig. 1), the 2-D convolution (Section 2.1, list of contractions) and the
signed 8-bit GEMM with 32-bit sums, accumulated in double / 64-bit integers.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this package; it
imports nothing from the GPU package and shares no code with it.

Every fp32 function returns ``(value, absum)`` as float64 arrays where ``absum`` is
``|C_in| + sum |a*b|`` per element, the scale the acceptance tolerance is stated in.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from .build import LIB, build as _build_lib

_lib = None

_i64 = ctypes.c_int64
_ptr = ctypes.c_void_p


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        src = os.path.join(os.path.dirname(LIB), "oracle.c")
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(src):
            _build_lib()
        L = ctypes.CDLL(LIB, mode=ctypes.RTLD_LOCAL)
        L.oracle_sgemm.argtypes = [_i64] * 3 + [_ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr, _ptr]
        L.oracle_sgemm_op.argtypes = ([ctypes.c_int] * 2 + [_i64] * 3
                                      + [_ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr, _ptr])
        L.oracle_sgemm_points.argtypes = ([_i64] * 3 + [_ptr, _i64, _ptr, _i64, _ptr, _i64, _i64]
                                          + [_ptr] * 4)
        L.oracle_igemm_s8s32.argtypes = [_i64] * 3 + [_ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr]
        L.oracle_igemm_s8s32_bt.argtypes = [_i64] * 3 + [_ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr]
        L.oracle_conv2d_nhwc.argtypes = [_i64] * 9 + [_ptr] * 4
        L.oracle_sgemm_fused.argtypes = ([_i64] * 3 + [_ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr]
                                         + [ctypes.c_int] * 2 + [_ptr] * 2)
        L.oracle_conv2d_nhwc_fused.argtypes = [_i64] * 9 + [_ptr] * 3 + [ctypes.c_int] + [_ptr] * 2
        L.oracle_dwconv2d_nhwc.argtypes = [_i64] * 8 + [_ptr] * 3 + [ctypes.c_int] + [_ptr] * 2
        L.oracle_tensor_copy.argtypes = [_i64, _ptr, _ptr, _ptr, _ptr]
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().oracle_num_threads()


def set_threads(n: int) -> None:
    lib().oracle_set_threads(int(n))


def _p(a: np.ndarray):
    return a.ctypes.data_as(_ptr)


def _check2d(a: np.ndarray, dtype, name: str):
    if a.dtype == dtype and a.ndim == 2 and a.size == 0:
        return max(a.shape[1], 1)
    if a.dtype != dtype or a.ndim != 2 or a.strides[1] != a.itemsize or a.strides[0] % a.itemsize:
        raise ValueError(f"{name}: need a row-major 2-D {np.dtype(dtype)} array (row stride allowed)")
    return a.strides[0] // a.itemsize


def sgemm(A: np.ndarray, B: np.ndarray, C: np.ndarray):
    """value = C + A @ B per the Fig. 1 loop nest; A, B, C may be row-strided views."""
    lda, ldb, ldc = _check2d(A, np.float32, "A"), _check2d(B, np.float32, "B"), _check2d(C, np.float32, "C")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or C.shape != (M, N):
        raise ValueError("shape mismatch")
    out = np.empty((M, N), np.float64)
    absum = np.empty((M, N), np.float64)
    rc = lib().oracle_sgemm(M, N, K, _p(A), max(lda, 1), _p(B), max(ldb, 1), _p(C), max(ldc, 1),
                            _p(out), _p(absum))
    if rc:
        raise RuntimeError(f"oracle_sgemm failed: {rc}")
    return out, absum


def sgemm_op(ta: bool, tb: bool, A: np.ndarray, B: np.ndarray, C: np.ndarray):
    """value = C + op(A) @ op(B); with ta the array A holds the K x M transpose of the left
    operand, with tb the array B holds the N x K transpose of the right one (Section 2.1)."""
    lda, ldb, ldc = _check2d(A, np.float32, "A"), _check2d(B, np.float32, "B"), _check2d(C, np.float32, "C")
    K, M = A.shape if ta else A.shape[::-1]
    K2, N = B.shape[::-1] if tb else B.shape
    if K2 != K or C.shape != (M, N):
        raise ValueError("shape mismatch")
    out = np.empty((M, N), np.float64)
    absum = np.empty((M, N), np.float64)
    rc = lib().oracle_sgemm_op(int(ta), int(tb), M, N, K, _p(A), max(lda, 1), _p(B), max(ldb, 1),
                               _p(C), max(ldc, 1), _p(out), _p(absum))
    if rc:
        raise RuntimeError(f"oracle_sgemm_op failed: {rc}")
    return out, absum


PRE_ACCUMULATE, PRE_ZERO, PRE_BIAS = 0, 1, 2
POST_NONE, POST_RELU = 0, 1


def sgemm_fused(A: np.ndarray, B: np.ndarray, C: np.ndarray, bias=None, pre: int = PRE_ACCUMULATE,
                post: int = POST_NONE):
    """value = post(pre(C) + A @ B) with the pre/post-operations of Section 2.1."""
    lda, ldb, ldc = _check2d(A, np.float32, "A"), _check2d(B, np.float32, "B"), _check2d(C, np.float32, "C")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or C.shape != (M, N):
        raise ValueError("shape mismatch")
    if pre == PRE_BIAS:
        bias = np.ascontiguousarray(bias, np.float32)
        if bias.shape != (N,):
            raise ValueError("bias must hold N values")
    out = np.empty((M, N), np.float64)
    absum = np.empty((M, N), np.float64)
    rc = lib().oracle_sgemm_fused(M, N, K, _p(A), max(lda, 1), _p(B), max(ldb, 1), _p(C), max(ldc, 1),
                                  _p(bias) if pre == PRE_BIAS else None, pre, post, _p(out), _p(absum))
    if rc:
        raise RuntimeError(f"oracle_sgemm_fused failed: {rc}")
    return out, absum


def sgemm_points(A: np.ndarray, B: np.ndarray, C: np.ndarray, ii, jj):
    """The same element formula at the coordinates (ii[t], jj[t]) only."""
    lda, ldb, ldc = _check2d(A, np.float32, "A"), _check2d(B, np.float32, "B"), _check2d(C, np.float32, "C")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or C.shape != (M, N):
        raise ValueError("shape mismatch")
    ii = np.ascontiguousarray(ii, np.int64)
    jj = np.ascontiguousarray(jj, np.int64)
    out = np.empty(ii.shape, np.float64)
    absum = np.empty(ii.shape, np.float64)
    rc = lib().oracle_sgemm_points(M, N, K, _p(A), lda, _p(B), ldb, _p(C), ldc, ii.size, _p(ii),
                                   _p(jj), _p(out), _p(absum))
    if rc:
        raise RuntimeError(f"oracle_sgemm_points failed: {rc}")
    return out, absum


def igemm_s8s32(A: np.ndarray, B: np.ndarray, C: np.ndarray) -> np.ndarray:
    """(C + A @ B) mod 2^32 with signed 8-bit A, B and int32 C."""
    lda, ldb, ldc = _check2d(A, np.int8, "A"), _check2d(B, np.int8, "B"), _check2d(C, np.int32, "C")
    M, K = A.shape
    K2, N = B.shape
    if K2 != K or C.shape != (M, N):
        raise ValueError("shape mismatch")
    out = np.empty((M, N), np.int32)
    rc = lib().oracle_igemm_s8s32(M, N, K, _p(A), max(lda, 1), _p(B), max(ldb, 1), _p(C),
                                  max(ldc, 1), _p(out))
    if rc:
        raise RuntimeError(f"oracle_igemm_s8s32 failed: {rc}")
    return out


def igemm_s8s32_bt(A: np.ndarray, Bt: np.ndarray, C: np.ndarray) -> np.ndarray:
    """(C + A @ Bt.T) mod 2^32 with signed 8-bit A (M x K), Bt (N x K) and int32 C."""
    lda, ldbt, ldc = _check2d(A, np.int8, "A"), _check2d(Bt, np.int8, "Bt"), _check2d(C, np.int32, "C")
    M, K = A.shape
    N, K2 = Bt.shape
    if K2 != K or C.shape != (M, N):
        raise ValueError("shape mismatch")
    out = np.empty((M, N), np.int32)
    rc = lib().oracle_igemm_s8s32_bt(M, N, K, _p(A), max(lda, 1), _p(Bt), max(ldbt, 1), _p(C),
                                     max(ldc, 1), _p(out))
    if rc:
        raise RuntimeError(f"oracle_igemm_s8s32_bt failed: {rc}")
    return out


def conv_out_shape(x_shape, w_shape, stride: int, pad: int):
    N, H, W, _ = x_shape
    K, R, S, _ = w_shape
    return N, (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1, K


def conv2d_nhwc(x: np.ndarray, w: np.ndarray, stride: int = 1, pad: int = 0, bias=None,
                post: int = POST_NONE):
    """out[n,p,q,k] = post(bias[k] + sum_{r,s,c} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[k,r,s,c])."""
    if x.dtype != np.float32 or w.dtype != np.float32 or x.ndim != 4 or w.ndim != 4:
        raise ValueError("x (NHWC) and w (KRSC) must be 4-D float32")
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    shape = conv_out_shape(x.shape, w.shape, stride, pad)
    out = np.empty(shape, np.float64)
    absum = np.empty(shape, np.float64)
    if bias is not None:
        bias = np.ascontiguousarray(bias, np.float32)
        if bias.shape != (K,):
            raise ValueError("bias must hold K values")
    rc = lib().oracle_conv2d_nhwc_fused(N, H, W, C, K, R, S, stride, pad, _p(x), _p(w),
                                        _p(bias) if bias is not None else None, post, _p(out), _p(absum))
    if rc:
        raise RuntimeError(f"oracle_conv2d_nhwc failed: {rc}")
    return out, absum


def dwconv2d_nhwc(x: np.ndarray, w: np.ndarray, stride: int = 1, pad: int = 0, bias=None,
                  post: int = POST_NONE):
    """out[n,p,q,c] = post(bias[c] + sum_{r,s} x[n, p*stride-pad+r, q*stride-pad+s, c] * w[r,s,c])."""
    if x.dtype != np.float32 or w.dtype != np.float32 or x.ndim != 4 or w.ndim != 3:
        raise ValueError("x (NHWC) must be 4-D and w (RSC) 3-D float32")
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w)
    N, H, W, C = x.shape
    R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    shape = (N, (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1, C)
    out = np.empty(shape, np.float64)
    absum = np.empty(shape, np.float64)
    if bias is not None:
        bias = np.ascontiguousarray(bias, np.float32)
        if bias.shape != (C,):
            raise ValueError("bias must hold C values")
    rc = lib().oracle_dwconv2d_nhwc(N, H, W, C, R, S, stride, pad, _p(x), _p(w),
                                    _p(bias) if bias is not None else None, post, _p(out), _p(absum))
    if rc:
        raise RuntimeError(f"oracle_dwconv2d_nhwc failed: {rc}")
    return out, absum


def tensor_copy(x: np.ndarray, dims, strides, offset: int = 0) -> np.ndarray:
    """out[i0,i1,i2,i3] = x.ravel()[offset + i0*s0 + i1*s1 + i2*s2 + i3*s3], dense, for
    float32 or int8 ``x`` (any shape: only its flat buffer is addressed)."""
    if x.dtype not in (np.float32, np.int8):
        raise ValueError("float32 or int8 only")
    flat = np.ascontiguousarray(x).ravel()
    d = np.asarray(dims, np.int64)
    s = np.asarray(strides, np.int64)
    if d.shape != (4,) or s.shape != (4,):
        raise ValueError("four extents and four strides")
    if np.all(d > 0) and offset + int(((d - 1) * s).sum()) >= flat.size:
        raise ValueError("addresses past the end of x")
    out = np.empty(tuple(int(v) for v in d), x.dtype)
    rc = lib().oracle_tensor_copy(x.dtype.itemsize, _p(d), _p(s), flat[offset:].ctypes.data if flat.size > offset else None,
                                  _p(out))
    if rc:
        raise RuntimeError(f"oracle_tensor_copy failed: {rc}")
    return out
