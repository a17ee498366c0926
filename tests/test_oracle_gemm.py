"""Pins for the GEMM oracles (fp32 and signed 8-bit): hand sums, invariants, closed forms,
and library cross-checks.  Each targets a mistake the plain loop nest could plausibly hold
(dropped C_in, swapped operands, wrong stride, wrong index order, lost sign, truncation)."""
import numpy as np
import pytest

import oracle
from golden_io import read_cases
from paper_2205_00618_amd import workloads as wl


@pytest.mark.parametrize("name", ["two_by_two", "three_by_three", "two_three_two", "row_vector"])
def test_sgemm_hand_sums(name):
    c = read_cases("sgemm_hand.txt")[name]
    val, absum = oracle.sgemm(c["A"].astype(np.float32), c["B"].astype(np.float32),
                              c["Cin"].astype(np.float32))
    assert np.array_equal(val, c["expect"])
    assert np.all(absum >= np.abs(val))


def test_sgemm_absum_hand():
    # |C_in| + sum|a b| for the 2x2 case: [1+5+14, 1+6+16; 0+15+28, 2+18+32]
    c = read_cases("sgemm_hand.txt")["two_by_two"]
    _, absum = oracle.sgemm(c["A"].astype(np.float32), c["B"].astype(np.float32),
                            c["Cin"].astype(np.float32))
    assert np.array_equal(absum, np.array([[20, 23], [43, 52]], np.float64))
    A = np.array([[1, -2]], np.float32)
    B = np.array([[3], [4]], np.float32)
    C = np.array([[-1]], np.float32)
    val, absum = oracle.sgemm(A, B, C)
    assert val[0, 0] == -6 and absum[0, 0] == 12


def test_sgemm_identity_and_zero():
    rng = np.random.default_rng(11)
    B = wl.uniform_f32(rng, (17, 23))
    C = wl.uniform_f32(rng, (17, 23))
    eye = np.eye(17, dtype=np.float32)
    val, _ = oracle.sgemm(eye, B, C)
    assert np.array_equal(val, C.astype(np.float64) + B.astype(np.float64))
    val, _ = oracle.sgemm(np.zeros((17, 17), np.float32), B, C)
    assert np.array_equal(val, C.astype(np.float64))
    A = wl.uniform_f32(rng, (17, 9))
    val, _ = oracle.sgemm(A, np.zeros((9, 23), np.float32), C)
    assert np.array_equal(val, C.astype(np.float64))
    # identity on the right
    A = wl.uniform_f32(rng, (17, 23))
    val, _ = oracle.sgemm(A, np.eye(23, dtype=np.float32), C)
    assert np.array_equal(val, C.astype(np.float64) + A.astype(np.float64))


def test_sgemm_k_zero_and_empty():
    C = np.arange(6, dtype=np.float32).reshape(2, 3)
    val, absum = oracle.sgemm(np.zeros((2, 0), np.float32), np.zeros((0, 3), np.float32), C)
    assert np.array_equal(val, C) and np.array_equal(absum, np.abs(C))
    val, _ = oracle.sgemm(np.zeros((0, 4), np.float32), np.zeros((4, 3), np.float32),
                          np.zeros((0, 3), np.float32))
    assert val.shape == (0, 3)


def test_sgemm_linearity_exact():
    rng = np.random.default_rng(5)
    A1, A2 = wl.small_int_f32(rng, (13, 31)), wl.small_int_f32(rng, (13, 31))
    B1, B2 = wl.small_int_f32(rng, (31, 7)), wl.small_int_f32(rng, (31, 7))
    Z = np.zeros((13, 7), np.float32)
    f = lambda a, b: oracle.sgemm(a, b, Z)[0]
    assert np.array_equal(f(A1 + A2, B1), f(A1, B1) + f(A2, B1))
    assert np.array_equal(f(A1, B1 + B2), f(A1, B1) + f(A1, B2))
    assert np.array_equal(f(3 * A1, B1), 3 * f(A1, B1))


def test_sgemm_rank_one_closed_form():
    # A = u 1^T, B = 1 v^T  =>  C[i,j] = K u_i v_j ; all ones => C = K
    K = 37
    u = np.arange(1, 6, dtype=np.float32)
    v = np.array([2, -3, 5, 7], np.float32)
    A = np.repeat(u[:, None], K, axis=1)
    B = np.repeat(v[None, :], K, axis=0)
    val, _ = oracle.sgemm(A, B, np.zeros((5, 4), np.float32))
    assert np.array_equal(val, K * np.outer(u, v).astype(np.float64))
    val, _ = oracle.sgemm(np.ones((3, K), np.float32), np.ones((K, 2), np.float32),
                          np.zeros((3, 2), np.float32))
    assert np.all(val == K)


def test_sgemm_single_entry_selects_one_product():
    # A has one non-zero at (i0,k0), B one at (k0,j0): only C[i0,j0] moves
    A = np.zeros((5, 6), np.float32)
    B = np.zeros((6, 4), np.float32)
    A[3, 2] = 2.0
    B[2, 1] = 7.0
    B[4, 1] = 100.0  # wrong k must not be picked up
    val, _ = oracle.sgemm(A, B, np.zeros((5, 4), np.float32))
    expect = np.zeros((5, 4))
    expect[3, 1] = 14.0
    assert np.array_equal(val, expect)


def test_sgemm_matches_float64_matmul_and_strides():
    rng = np.random.default_rng(7)
    A = wl.uniform_f32(rng, (33, 65))
    B = wl.uniform_f32(rng, (65, 29))
    C = wl.uniform_f32(rng, (33, 29))
    ref = C.astype(np.float64) + A.astype(np.float64) @ B.astype(np.float64)
    val, absum = oracle.sgemm(A, B, C)
    assert np.max(np.abs(val - ref) / absum) < 1e-14
    ref_abs = np.abs(C).astype(np.float64) + np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)
    assert np.max(np.abs(absum - ref_abs) / ref_abs) < 1e-14
    # leading dimensions larger than the row length, padding poisoned with NaN
    Ap = wl.with_ld(A, 70, fill=np.nan)[:, :65]
    Bp = wl.with_ld(B, 31, fill=np.nan)[:, :29]
    Cp = wl.with_ld(C, 40, fill=np.nan)[:, :29]
    val2, absum2 = oracle.sgemm(Ap, Bp, Cp)
    assert np.array_equal(val2, val) and np.array_equal(absum2, absum)


def test_sgemm_points_equal_full():
    rng = np.random.default_rng(9)
    A = wl.uniform_f32(rng, (40, 50))
    B = wl.uniform_f32(rng, (50, 30))
    C = wl.uniform_f32(rng, (40, 30))
    val, absum = oracle.sgemm(A, B, C)
    ii, jj = wl.sample_points(3, 40, 30, 50, tile=16)
    pv, pa = oracle.sgemm_points(A, B, C, ii, jj)
    assert np.array_equal(pv, val[ii, jj]) and np.array_equal(pa, absum[ii, jj])
    ref = C[ii, jj].astype(np.float64) + np.einsum("tk,kt->t", A[ii].astype(np.float64),
                                                   B[:, jj].astype(np.float64))
    assert np.max(np.abs(pv - ref)) < 1e-13


def test_sgemm_oracle_error_is_far_inside_tolerance():
    # exact rational check: with dyadic inputs the double accumulation is exact
    rng = np.random.default_rng(13)
    A = (rng.integers(-2**10, 2**10, size=(8, 300)) / 2.0**10).astype(np.float32)
    B = (rng.integers(-2**10, 2**10, size=(300, 8)) / 2.0**10).astype(np.float32)
    val, _ = oracle.sgemm(A, B, np.zeros((8, 8), np.float32))
    exact = (np.rint(A * 2**10).astype(np.int64) @ np.rint(B * 2**10).astype(np.int64)) / 2.0**20
    assert np.array_equal(val, exact)


# ---------------------------------------------------------------- signed 8-bit

@pytest.mark.parametrize("name", ["extremes", "with_cin"])
def test_igemm_hand_sums(name):
    c = read_cases("igemm_hand.txt")[name]
    out = oracle.igemm_s8s32(c["A"].astype(np.int8), c["B"].astype(np.int8), c["Cin"].astype(np.int32))
    assert out.dtype == np.int32 and np.array_equal(out, c["expect"].astype(np.int32))


def test_igemm_all_min_value():
    # (-128)^2 * 1024 = 2^24 exactly
    A = np.full((3, 1024), -128, np.int8)
    B = np.full((1024, 2), -128, np.int8)
    out = oracle.igemm_s8s32(A, B, np.zeros((3, 2), np.int32))
    assert np.all(out == 2**24)
    B[:] = 127
    out = oracle.igemm_s8s32(A, B, np.zeros((3, 2), np.int32))
    assert np.all(out == -128 * 127 * 1024)


def test_igemm_matches_int64_matmul_and_sgemm_oracle():
    A, B, C = wl.igemm_inputs(21, wl.GemmShape(37, 41, 129), c_zero=False)
    out = oracle.igemm_s8s32(A, B, C)
    ref = C.astype(np.int64) + A.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(out.astype(np.int64), ref)
    val, _ = oracle.sgemm(A.astype(np.float32), B.astype(np.float32), np.zeros((37, 41), np.float32))
    assert np.array_equal(val, (ref - C).astype(np.float64))


def test_igemm_wraps_modulo_2_32():
    A = np.full((1, 4), 127, np.int8)
    B = np.full((4, 1), 127, np.int8)
    C = np.array([[2**31 - 1]], np.int32)
    out = oracle.igemm_s8s32(A, B, C)
    assert out[0, 0] == np.int64(2**31 - 1 + 4 * 127 * 127 - 2**32)
    C = np.array([[-2**31]], np.int32)
    B[:] = -128
    out = oracle.igemm_s8s32(A, B, C)
    assert out[0, 0] == np.int64(-2**31 - 4 * 127 * 128 + 2**32)


def test_igemm_sign_of_both_operands():
    # would fail if either operand were read as unsigned bytes
    A = np.array([[-1]], np.int8)
    B = np.array([[1]], np.int8)
    assert oracle.igemm_s8s32(A, B, np.zeros((1, 1), np.int32))[0, 0] == -1
    assert oracle.igemm_s8s32(B, A, np.zeros((1, 1), np.int32))[0, 0] == -1
    assert oracle.igemm_s8s32(A, A, np.zeros((1, 1), np.int32))[0, 0] == 1


def test_igemm_strides():
    A, B, C = wl.igemm_inputs(22, wl.GemmShape(9, 11, 13), c_zero=False)
    ref = oracle.igemm_s8s32(A, B, C)
    Ap = wl.with_ld(A, 20, fill=99)[:, :13]
    Bp = wl.with_ld(B, 17, fill=99)[:, :11]
    Cp = wl.with_ld(C, 12, fill=99)[:, :11]
    assert np.array_equal(oracle.igemm_s8s32(Ap, Bp, Cp), ref)


@pytest.mark.parametrize("name", ["bt_with_cin", "bt_rectangular"])
def test_igemm_bt_hand_sums(name):
    c = read_cases("igemm_hand.txt")[name]
    out = oracle.igemm_s8s32_bt(c["A"].astype(np.int8), c["Bt"].astype(np.int8), c["Cin"].astype(np.int32))
    assert out.dtype == np.int32 and np.array_equal(out, c["expect"].astype(np.int32))


def test_igemm_bt_matches_int64_matmul_and_wraps():
    rng = np.random.default_rng(31)
    A = rng.integers(-128, 128, size=(9, 300), dtype=np.int8)
    Bt = rng.integers(-128, 128, size=(7, 300), dtype=np.int8)
    C = rng.integers(-2**31, 2**31, size=(9, 7), dtype=np.int64).astype(np.int32)
    want = (C.astype(np.int64) + A.astype(np.int64) @ Bt.astype(np.int64).T) & 0xFFFFFFFF
    got = oracle.igemm_s8s32_bt(A, Bt, C)
    assert np.array_equal(got.view(np.uint32).astype(np.int64), want)
    # padded rows are never read
    buf = np.full((7, 310), 99, np.int8)
    buf[:, :300] = Bt
    assert np.array_equal(oracle.igemm_s8s32_bt(A, buf[:, :300], C), got)
