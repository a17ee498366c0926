"""ctypes binding of liblsmi.so: argument marshalling only.

Function names and argument order are those of ``include/lsmi.h``.  The raw calls take
integers that are device addresses; the ``*_t`` helpers accept torch tensors that own
device memory and pass their ``data_ptr()`` and strides through unchanged.  No arithmetic
of the contractions happens here, and there is no fallback: if the library has not been
built, ``load()`` raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblsmi.so")

OK, ERR_DIM, ERR_LD, ERR_NULL, ERR_TOO_LARGE, ERR_NO_DEVICE, ERR_LAUNCH, ERR_OP = 0, -1, -2, -3, -4, -5, -6, -7
PRE_ACCUMULATE, PRE_ZERO, PRE_BIAS = 0, 1, 2
POST_NONE, POST_RELU = 0, 1

# every symbol include/lsmi.h and include/lsmi_tune.h declare
SYMBOLS = ("sgemm", "sgemm_fused", "igemm_s8s32", "conv2d_nhwc", "conv2d_nhwc_fused", "lsmi_set_stream", "lsmi_strerror",
           "lsmi_last_hip_error", "lsmi_version", "lsmi_last_variant", "lsmi_set_tuning",
           "lsmi_variant_name", "lsmi_tile_of_workgroup", "lsmi_set_conv_tuning",
           "dwconv2d_nhwc", "dwconv2d_nhwc_fused", "lsmi_set_dwconv_tuning", "lsmi_set_dwconv_tile",
           "lsmi_dwconv_variant_name", "lsmi_set_conv_split", "lsmi_conv_variant_name",
           "lsmi_set_igemm_tuning", "lsmi_igemm_variant_name", "tensor_copy_f32", "tensor_copy_s8", "igemm_s8s32_bt",
           "lsmi_set_conv_tail", "lsmi_mfma_rate", "sgemm_op", "sgemm_ws", "lsmi_sgemm_ws_bytes", "lsmi_last_split",
           "sgemm_static", "lsmi_fast_divide", "lsmi_set_tile_walk")

_lib = None
_i64, _ptr, _int = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int


class LsmiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status}, hip error {last_hip_error()})")


def load() -> ctypes.CDLL:
    """Open liblsmi.so (RTLD_LOCAL, so the bare name ``sgemm`` cannot interpose on a BLAS)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2205_00618_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH, mode=ctypes.RTLD_LOCAL)
        L.sgemm.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]
        L.igemm_s8s32.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]
        L.sgemm_op.argtypes = [_int, _int, _i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]
        L.sgemm_op.restype = _int
        L.sgemm_ws.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]
        L.sgemm_ws.restype = _int
        L.sgemm_static.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]
        L.sgemm_static.restype = _int
        L.lsmi_sgemm_ws_bytes.argtypes = [_i64, _i64, _i64]
        L.lsmi_sgemm_ws_bytes.restype = _i64
        L.lsmi_last_split.restype = _int
        L.lsmi_set_tile_walk.argtypes = [_int]
        L.lsmi_set_tile_walk.restype = _int
        L.lsmi_fast_divide.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
        L.lsmi_fast_divide.restype = ctypes.c_uint32
        L.igemm_s8s32_bt.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64]
        L.igemm_s8s32_bt.restype = _int
        L.conv2d_nhwc.argtypes = [_i64] * 9 + [_ptr] * 3
        L.sgemm_fused.argtypes = [_i64, _i64, _i64, _ptr, _i64, _ptr, _i64, _ptr, _i64, _ptr, _int, _int]
        L.conv2d_nhwc_fused.argtypes = [_i64] * 9 + [_ptr] * 4 + [_int]
        L.dwconv2d_nhwc.argtypes = [_i64] * 8 + [_ptr] * 3
        L.dwconv2d_nhwc_fused.argtypes = [_i64] * 8 + [_ptr] * 4 + [_int]
        L.lsmi_set_dwconv_tuning.argtypes = [_int, _int]
        L.tensor_copy_f32.argtypes = [_i64] * 8 + [_ptr] * 2
        L.tensor_copy_f32.restype = _int
        L.tensor_copy_s8.argtypes = [_i64] * 8 + [_ptr] * 2
        L.tensor_copy_s8.restype = _int
        L.lsmi_set_igemm_tuning.argtypes = [_int]
        L.lsmi_set_igemm_tuning.restype = _int
        L.lsmi_igemm_variant_name.argtypes = [_int]
        L.lsmi_igemm_variant_name.restype = ctypes.c_char_p
        L.lsmi_set_conv_tail.argtypes = [_int]
        L.lsmi_set_conv_tail.restype = _int
        L.lsmi_set_conv_split.argtypes = [_int]
        L.lsmi_set_conv_split.restype = _int
        L.lsmi_conv_variant_name.argtypes = [_int]
        L.lsmi_conv_variant_name.restype = ctypes.c_char_p
        L.lsmi_set_dwconv_tile.argtypes = [_int, _int, _int]
        L.lsmi_set_dwconv_tile.restype = _int
        L.lsmi_dwconv_variant_name.argtypes = [_int]
        L.lsmi_dwconv_variant_name.restype = ctypes.c_char_p
        L.lsmi_set_stream.argtypes = [_ptr]
        L.lsmi_strerror.argtypes = [_int]
        L.lsmi_strerror.restype = ctypes.c_char_p
        L.lsmi_last_variant.restype = ctypes.c_char_p
        L.lsmi_set_tuning.argtypes = [_int, _int]
        L.lsmi_set_conv_tuning.argtypes = [_int]
        L.lsmi_set_conv_tuning.restype = _int
        L.lsmi_variant_name.argtypes = [_int]
        L.lsmi_variant_name.restype = ctypes.c_char_p
        L.lsmi_tile_of_workgroup.argtypes = [_int] * 4 + [ctypes.POINTER(_int)] * 2
        L.lsmi_tile_of_workgroup.restype = _int
        L.lsmi_mfma_rate.argtypes = [_int, _int, _ptr, _i64, ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_double)]
        L.lsmi_mfma_rate.restype = _int
        for name in ("sgemm", "sgemm_fused", "conv2d_nhwc_fused", "igemm_s8s32", "conv2d_nhwc", "lsmi_set_stream", "lsmi_last_hip_error",
                     "lsmi_version", "lsmi_set_tuning", "dwconv2d_nhwc", "dwconv2d_nhwc_fused", "lsmi_set_dwconv_tuning"):
            getattr(L, name).restype = _int
        _lib = L
    return _lib


# ---- raw calls: integers are device addresses, return value is the library status ----

def sgemm(M, N, K, A, lda, B, ldb, C, ldc) -> int:
    return load().sgemm(M, N, K, A, lda, B, ldb, C, ldc)


def sgemm_op(transa, transb, M, N, K, A, lda, B, ldb, C, ldc) -> int:
    return load().sgemm_op(int(transa), int(transb), M, N, K, A, lda, B, ldb, C, ldc)


def sgemm_ws(M, N, K, A, lda, B, ldb, C, ldc, workspace, workspace_bytes) -> int:
    return load().sgemm_ws(M, N, K, A, lda, B, ldb, C, ldc, workspace, workspace_bytes)


def sgemm_static(M, N, K, A, lda, B, ldb, C, ldc) -> int:
    return load().sgemm_static(M, N, K, A, lda, B, ldb, C, ldc)


def sgemm_ws_bytes(M, N, K) -> int:
    return load().lsmi_sgemm_ws_bytes(M, N, K)


def fast_divide(n: int, d: int) -> int:
    return load().lsmi_fast_divide(n, d)


def last_split() -> int:
    return load().lsmi_last_split()


def sgemm_fused(M, N, K, A, lda, B, ldb, C, ldc, bias, pre, post) -> int:
    return load().sgemm_fused(M, N, K, A, lda, B, ldb, C, ldc, bias, pre, post)


def conv2d_nhwc_fused(N, H, W, C, K, R, S, stride, pad, inp, w, out, bias, post) -> int:
    return load().conv2d_nhwc_fused(N, H, W, C, K, R, S, stride, pad, inp, w, out, bias, post)


def igemm_s8s32(M, N, K, A, lda, B, ldb, C, ldc) -> int:
    return load().igemm_s8s32(M, N, K, A, lda, B, ldb, C, ldc)


def igemm_s8s32_bt(M, N, K, A, lda, Bt, ldbt, C, ldc) -> int:
    return load().igemm_s8s32_bt(M, N, K, A, lda, Bt, ldbt, C, ldc)


def conv2d_nhwc(N, H, W, C, K, R, S, stride, pad, inp, w, out) -> int:
    return load().conv2d_nhwc(N, H, W, C, K, R, S, stride, pad, inp, w, out)


def dwconv2d_nhwc(N, H, W, C, R, S, stride, pad, inp, w, out) -> int:
    return load().dwconv2d_nhwc(N, H, W, C, R, S, stride, pad, inp, w, out)


def dwconv2d_nhwc_fused(N, H, W, C, R, S, stride, pad, inp, w, out, bias, post) -> int:
    return load().dwconv2d_nhwc_fused(N, H, W, C, R, S, stride, pad, inp, w, out, bias, post)


def tensor_copy_f32(d0, d1, d2, d3, s0, s1, s2, s3, inp, out) -> int:
    return load().tensor_copy_f32(d0, d1, d2, d3, s0, s1, s2, s3, inp, out)


def tensor_copy_s8(d0, d1, d2, d3, s0, s1, s2, s3, inp, out) -> int:
    return load().tensor_copy_s8(d0, d1, d2, d3, s0, s1, s2, s3, inp, out)


def set_stream(hip_stream) -> int:
    return load().lsmi_set_stream(hip_stream)


def strerror(status: int) -> str:
    return load().lsmi_strerror(status).decode()


def last_hip_error() -> int:
    return load().lsmi_last_hip_error()


def version() -> int:
    return load().lsmi_version()


def last_variant() -> str:
    return load().lsmi_last_variant().decode()


def set_tuning(sgemm_variant: int = -1, split_k: int = 0) -> int:
    return load().lsmi_set_tuning(sgemm_variant, split_k)


def set_tile_walk(band_rows: int = 0) -> int:
    return load().lsmi_set_tile_walk(band_rows)


def set_conv_tuning(conv_variant: int = -1) -> int:
    return load().lsmi_set_conv_tuning(conv_variant)


def set_igemm_tuning(igemm_variant: int = -1) -> int:
    return load().lsmi_set_igemm_tuning(igemm_variant)


def igemm_variant_names():
    names, i = [], 0
    while True:
        s = load().lsmi_igemm_variant_name(i)
        if s is None:
            return names
        names.append(s.decode())
        i += 1


def set_conv_split(slices: int = 0) -> int:
    return load().lsmi_set_conv_split(slices)


def set_conv_tail(tile_rows: int = -1) -> int:
    return load().lsmi_set_conv_tail(tile_rows)


def conv_variant_names():
    names, i = [], 0
    while True:
        s = load().lsmi_conv_variant_name(i)
        if s is None:
            return names
        names.append(s.decode())
        i += 1


def set_dwconv_tuning(dwconv_variant: int = -1, strip: int = 0) -> int:
    return load().lsmi_set_dwconv_tuning(dwconv_variant, strip)


def set_dwconv_tile(cols: int = 0, channels: int = 0, depth: int = 0) -> int:
    return load().lsmi_set_dwconv_tile(cols, channels, depth)


def dwconv_variant_names():
    names, i = [], 0
    while True:
        s = load().lsmi_dwconv_variant_name(i)
        if s is None:
            return names
        names.append(s.decode())
        i += 1


def tile_of_workgroup(wg: int, tiles_m: int, tiles_n: int, group_m: int):
    tm, tn = _int(-1), _int(-1)
    status = load().lsmi_tile_of_workgroup(wg, tiles_m, tiles_n, group_m, ctypes.byref(tm),
                                           ctypes.byref(tn))
    if status != OK:
        raise LsmiError(status, "lsmi_tile_of_workgroup")
    return tm.value, tn.value


def variant_names():
    names, i = [], 0
    while True:
        s = load().lsmi_variant_name(i)
        if s is None:
            return names
        names.append(s.decode())
        i += 1


def mfma_rate(int8: bool, random_operands: bool, device_words: int, words: int):
    """(operations per second, shader clock in Hz) of a loop of matrix instructions on registers."""
    ops, hz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    status = load().lsmi_mfma_rate(int(int8), int(random_operands), device_words, words,
                                   ctypes.byref(ops), ctypes.byref(hz))
    if status != OK:
        raise LsmiError(status, "lsmi_mfma_rate")
    return ops.value, hz.value


# ---- tensor helpers: torch owns the memory and the stream, nothing else ----

def use_torch_stream() -> None:
    """Enqueue this thread's later calls on torch's current stream."""
    import torch
    set_stream(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise LsmiError(status, where)


def _rows(t, name: str) -> int:
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or not t.is_cuda:
        raise ValueError(f"{name}: need a 2-D device tensor with unit column stride")
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], 1)


def sgemm_t(A, B, C) -> None:
    """C += A @ B in place; A (MxK), B (KxN), C (MxN) fp32 device tensors (row stride free)."""
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _check(sgemm(M, N, K, A.data_ptr(), _rows(A, "A"), B.data_ptr(), _rows(B, "B"), C.data_ptr(),
                 _rows(C, "C")), "sgemm")


def sgemm_op_t(transa: bool, transb: bool, A, B, C) -> None:
    """C += op(A) @ op(B) in place; with transa A is the stored K x M transpose, with transb B is N x K."""
    K, M = A.shape if transa else (A.shape[1], A.shape[0])
    K2, N = (B.shape[1], B.shape[0]) if transb else B.shape
    if K2 != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _check(sgemm_op(transa, transb, M, N, K, A.data_ptr(), _rows(A, "A"), B.data_ptr(), _rows(B, "B"),
                    C.data_ptr(), _rows(C, "C")), "sgemm_op")


def sgemm_ws_t(A, B, C, workspace) -> None:
    """C += A @ B in place, partial sums of a cut reduction meeting in `workspace` (a device
    tensor whose first 65536 bytes were zero before its first use)."""
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _check(sgemm_ws(M, N, K, A.data_ptr(), _rows(A, "A"), B.data_ptr(), _rows(B, "B"), C.data_ptr(),
                    _rows(C, "C"), workspace.data_ptr() if workspace is not None else None,
                    workspace.numel() * workspace.element_size() if workspace is not None else 0), "sgemm_ws")


def sgemm_fused_t(A, B, C, bias=None, pre: int = PRE_ACCUMULATE, post: int = POST_NONE) -> None:
    """C = post(pre(C) + A @ B) in place; bias: N fp32 device values for PRE_BIAS."""
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != N or not bias.is_contiguous()):
        raise ValueError("bias must be a dense vector of N values")
    _check(sgemm_fused(M, N, K, A.data_ptr(), _rows(A, "A"), B.data_ptr(), _rows(B, "B"), C.data_ptr(),
                       _rows(C, "C"), bias.data_ptr() if bias is not None else None, pre, post),
           "sgemm_fused")


def igemm_s8s32_t(A, B, C) -> None:
    """C += A @ B in place; A, B int8 device tensors, C int32."""
    M, K = A.shape
    N = B.shape[1]
    if B.shape[0] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _check(igemm_s8s32(M, N, K, A.data_ptr(), _rows(A, "A"), B.data_ptr(), _rows(B, "B"),
                       C.data_ptr(), _rows(C, "C")), "igemm_s8s32")


def igemm_s8s32_bt_t(A, Bt, C) -> None:
    """C += A @ Bt.T in place; A (MxK), Bt (NxK) int8 device tensors, C (MxN) int32."""
    M, K = A.shape
    N = Bt.shape[0]
    if Bt.shape[1] != K or tuple(C.shape) != (M, N):
        raise ValueError("shape mismatch")
    _check(igemm_s8s32_bt(M, N, K, A.data_ptr(), _rows(A, "A"), Bt.data_ptr(), _rows(Bt, "Bt"),
                          C.data_ptr(), _rows(C, "C")), "igemm_s8s32_bt")


def conv2d_nhwc_t(x, w, out, stride: int, pad: int, bias=None, post: int = POST_NONE) -> None:
    """out[N,P,Q,K] = post(bias + conv(x[N,H,W,C], w[K,R,S,C])); dense fp32 device tensors."""
    if not (x.is_contiguous() and w.is_contiguous() and out.is_contiguous()):
        raise ValueError("conv2d_nhwc needs dense tensors")
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if tuple(out.shape) != (N, P, Q, K):
        raise ValueError(f"out must be {(N, P, Q, K)}")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != K or not bias.is_contiguous()):
        raise ValueError("bias must be a dense vector of K values")
    _check(conv2d_nhwc_fused(N, H, W, C, K, R, S, stride, pad, x.data_ptr(), w.data_ptr(),
                             out.data_ptr(), bias.data_ptr() if bias is not None else None, post),
           "conv2d_nhwc")


def dwconv2d_nhwc_t(x, w, out, stride: int, pad: int, bias=None, post: int = POST_NONE) -> None:
    """out[N,P,Q,C] = post(bias + depthwise_conv(x[N,H,W,C], w[R,S,C])); dense fp32 device tensors."""
    if not (x.is_contiguous() and w.is_contiguous() and out.is_contiguous()):
        raise ValueError("dwconv2d_nhwc needs dense tensors")
    N, H, W, C = x.shape
    R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    if tuple(out.shape) != (N, P, Q, C):
        raise ValueError(f"out must be {(N, P, Q, C)}")
    if bias is not None and (bias.dim() != 1 or bias.shape[0] != C or not bias.is_contiguous()):
        raise ValueError("bias must be a dense vector of C values")
    _check(dwconv2d_nhwc_fused(N, H, W, C, R, S, stride, pad, x.data_ptr(), w.data_ptr(),
                               out.data_ptr(), bias.data_ptr() if bias is not None else None, post),
           "dwconv2d_nhwc")


def tensor_copy_t(x, out) -> None:
    """out (dense, up to 4-D) = x, where x is any strided view (permute, slice, expand) of a
    float32 or int8 device tensor with non-negative strides."""
    import torch
    if x.dtype != out.dtype or x.dtype not in (torch.float32, torch.int8):
        raise ValueError("float32 or int8 tensors of one type")
    if tuple(x.shape) != tuple(out.shape) or x.dim() > 4 or not out.is_contiguous():
        raise ValueError("out must be dense with x's shape, at most four dimensions")
    pad = 4 - x.dim()
    d = [1] * pad + list(x.shape)
    s = [0] * pad + list(x.stride())
    fn = tensor_copy_f32 if x.dtype == torch.float32 else tensor_copy_s8
    _check(fn(*d, *s, x.data_ptr(), out.data_ptr()), "tensor_copy")
