"""Pins of the oracle for products on transposed operands (not GPU): hand sums on rectangular
cases a wrong index map cannot reproduce, reduction to the plain product's oracle on
explicitly transposed copies, float64 matmul, leading dimensions with poisoned padding."""
import numpy as np
import pytest

import oracle
from golden_io import read_cases
from paper_2205_00618_amd import workloads as wl

CASES = read_cases("sgemm_op_hand.txt")


@pytest.mark.parametrize("name", sorted(CASES))
def test_hand_sums(name):
    c = CASES[name]
    A, B, Cin = (c[k].astype(np.float32) for k in ("A", "B", "Cin"))
    out, absum = oracle.sgemm_op(bool(c["ta"]), bool(c["tb"]), A, B, Cin)
    assert np.array_equal(out, c["expect"])
    assert np.all(absum >= np.abs(out))


def test_hand_cases_reject_the_untransposed_reading():
    # the same stored arrays read without the swap give something else (where shapes allow)
    c = CASES["tt_two_three_two"]
    A, B, Cin = (c[k].astype(np.float32) for k in ("A", "B", "Cin"))
    # (the same memory taken as a 2 x 3 and a 3 x 2 row-major matrix)
    wrong, _ = oracle.sgemm(np.ascontiguousarray(A).reshape(2, 3), np.ascontiguousarray(B).reshape(3, 2), Cin)
    assert not np.array_equal(wrong, c["expect"])


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_reduces_to_the_plain_product_on_transposed_copies(ta, tb):
    rng = np.random.default_rng(7 + 2 * ta + tb)
    M, N, K = 23, 17, 31
    a = wl.uniform_f32(rng, (M, K))
    b = wl.uniform_f32(rng, (K, N))
    c = wl.uniform_f32(rng, (M, N))
    A = np.ascontiguousarray(a.T) if ta else a
    B = np.ascontiguousarray(b.T) if tb else b
    out, absum = oracle.sgemm_op(ta, tb, A, B, c)
    ref, ref_abs = oracle.sgemm(a, b, c)
    assert np.array_equal(out, ref) and np.array_equal(absum, ref_abs)
    lib = c.astype(np.float64) + a.astype(np.float64) @ b.astype(np.float64)
    assert np.max(np.abs(out - lib)) <= 1e-12 * np.max(absum)


@pytest.mark.parametrize("ta,tb", [(True, False), (False, True), (True, True)])
def test_leading_dimensions_skip_poisoned_padding(ta, tb):
    rng = np.random.default_rng(11)
    M, N, K = 5, 7, 9
    a = np.round(wl.uniform_f32(rng, (M, K)) * 8)
    b = np.round(wl.uniform_f32(rng, (K, N)) * 8).astype(np.float32)
    a = a.astype(np.float32)
    c = np.round(wl.uniform_f32(rng, (M, N)) * 8).astype(np.float32)

    def padded(x, extra):
        buf = np.full((x.shape[0], x.shape[1] + extra), np.nan, np.float32)
        buf[:, :x.shape[1]] = x
        return buf[:, :x.shape[1]]

    A = padded(np.ascontiguousarray(a.T) if ta else a, 3)
    B = padded(np.ascontiguousarray(b.T) if tb else b, 2)
    C = padded(c, 5)
    out, _ = oracle.sgemm_op(ta, tb, A, B, C)
    assert np.array_equal(out, c.astype(np.float64) + a.astype(np.float64) @ b.astype(np.float64))


def test_rank_one_closed_form_on_transposed_storage():
    # op(A) = u 1^T, op(B) = 1 v^T  =>  C[i,j] = K u_i v_j, whatever the storage
    K = 13
    u = np.arange(1, 5, dtype=np.float32)
    v = np.arange(-2, 4, dtype=np.float32)
    A = np.tile(u, (K, 1))            # K x M, stored transposed
    B = np.tile(v[:, None], (1, K))   # N x K, stored transposed
    out, _ = oracle.sgemm_op(True, True, A, B, np.zeros((4, 6), np.float32))
    assert np.array_equal(out, K * np.outer(u, v))
