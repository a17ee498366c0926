"""Helpers for the GPU parity tests: upload numpy arrays, call the C ABI, fetch results."""
import numpy as np
import torch

from paper_2205_00618_amd import binding as b

TOL = 1e-5  # |gpu - oracle| <= TOL * (|C_in| + sum |a*b|) per element


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_sgemm(A, B, C, lda=None, ldb=None, ldc=None, offset=0, ta=False, tb=False, workspace=None):
    """Runs the library's sgemm on (possibly row-padded, possibly offset) device copies and
    returns the resulting C as numpy.  Padding is NaN so that a stray read poisons C.
    ta / tb: A / B are the stored transposes (K x M, N x K) and the call is sgemm_op;
    workspace: a device tensor, and the call is sgemm_ws."""
    K, M = A.shape if ta else A.shape[::-1]
    N = B.shape[0] if tb else B.shape[1]
    lda, ldb, ldc = lda or A.shape[1], ldb or B.shape[1], ldc or N

    def place(a, ld, fill):
        buf = np.full(a.shape[0] * ld + offset, fill, a.dtype)
        view = buf[offset:].reshape(a.shape[0], ld)
        view[:, :a.shape[1]] = a
        return buf

    bufA, bufB, bufC = place(A, lda, np.nan), place(B, ldb, np.nan), place(C, ldc, 777.0)
    dA, dB, dC = dev(bufA), dev(bufB), dev(bufC)
    esz = 4
    ptrs = (dA.data_ptr() + offset * esz, lda, dB.data_ptr() + offset * esz, ldb, dC.data_ptr() + offset * esz, ldc)
    if workspace is not None:
        assert not (ta or tb)
        st = b.sgemm_ws(M, N, K, *ptrs, workspace.data_ptr(), workspace.numel() * workspace.element_size())
    elif ta or tb:
        st = b.sgemm_op(ta, tb, M, N, K, *ptrs)
    else:
        st = b.sgemm(M, N, K, *ptrs)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    full = out[offset:].reshape(M, ldc)
    assert np.all(full[:, N:] == 777.0), "wrote outside the N columns of C"
    assert np.all(out[:offset] == 777.0)
    return full[:, :N].copy()


def assert_close(got, ref, absum, tol=TOL, what=""):
    err = np.abs(got.astype(np.float64) - ref)
    bound = tol * absum
    bad = err > bound
    if np.any(bad):
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} elements out of tolerance, worst at {idx}: "
                             f"got {got[idx]!r} ref {ref[idx]!r} err {err[idx]:.3e} bound {bound[idx]:.3e}")
    return float(np.max(err / np.maximum(absum, 1e-300)))
