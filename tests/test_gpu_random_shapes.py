"""Seeded sweeps of shapes, leading dimensions and base offsets through the built-in kernel
choice of every compute call: whatever kernel and cut of the reduction the library picks for a
shape, the result on small integers must equal the oracle bit for bit.  The hand-picked cases
of the other test files force kernels; here the choice itself is the thing under test."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_conv as tc
import test_gpu_dwconv as td
import test_gpu_igemm as ti
from gpu_util import dev, run_sgemm
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults():
    def reset():
        b.set_stream(None)
        b.set_tuning(-1, 0)
        b.set_igemm_tuning(-1)
        b.set_conv_tuning(-1)
        b.set_conv_split(0)
        b.set_conv_tail(-1)
        b.set_dwconv_tuning(-1, 0)
        b.set_dwconv_tile(0, 0, 0)
    reset()
    yield
    reset()


def gemm_cases(seed, count, lo, hi, k_hi, unit):
    """(M, N, K, lda - K, ldb - N, ldc - N, offset); `unit`: what the extents and paddings are
    rounded to in about half of the cases (the aligned kernels need whole vector loads)."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        M, N = (int(v) for v in rng.integers(lo, hi, 2))
        K = int(rng.integers(1, k_hi))
        pads = [int(v) for v in rng.choice([0, 0, 1, 3, unit, 2 * unit, 5 * unit], 3)]
        offset = int(rng.choice([0, 0, 1, unit]))
        if i % 2 == 0:      # vector-aligned rows: N, K, paddings and offset multiples of the unit
            N, K = max(unit, N // unit * unit), max(unit, K // unit * unit)
            pads = [p // unit * unit for p in pads]
            offset = offset // unit * unit
        cases.append((M, N, K, *pads, offset))
    return cases


SGEMM_SMALL = gemm_cases(1001, 40, 1, 600, 900, 4)
SGEMM_LARGE = gemm_cases(1002, 14, 1300, 3400, 300, 4)


def few_row_cases(seed, count, unit):
    """A few rows of C against a B of a million elements or more (the few-row kernels' range),
    aligned in two cases of three."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        M = int(rng.integers(1, 40))
        N, K = int(rng.integers(1024, 3000)), int(rng.integers(1024, 2100))
        pads = [int(v) for v in rng.choice([0, 0, 1, unit, 3 * unit], 3)]
        offset = int(rng.choice([0, 0, 1, unit]))
        if i % 3 != 0:
            K = K // unit * unit
            pads = [p // unit * unit for p in pads]
            pads[0] += (-K) % unit
            pads[1] += (-N) % unit      # N itself stays ragged, its row pitch is aligned
            offset = offset // unit * unit
        cases.append((M, N, K, *pads, offset))
    return cases


def few_col_cases(seed, count):
    """A few columns of C against an A of a million elements or more (a matrix-vector product and
    its relatives): K a multiple of 4, rows of A padded by multiples of 4, B and C by anything."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        M, N = int(rng.integers(1024, 6000)), int(rng.integers(1, 20))
        K = int(rng.integers(256, 2500)) // 4 * 4
        cases.append((M, N, K, int(rng.choice([0, 4, 8])), int(rng.choice([0, 1, 4])), int(rng.choice([0, 1, 3])), 0))
    return cases


SGEMM_FEW = few_row_cases(1007, 18, 4) + few_col_cases(1011, 16)
IGEMM_FEW = few_row_cases(1008, 12, 16)


@pytest.mark.parametrize("case", SGEMM_SMALL + SGEMM_LARGE + SGEMM_FEW, ids=lambda c: "x".join(map(str, c)))
def test_sgemm_built_in_choice_exact(case):
    M, N, K, pa, pb, pc, offset = case
    print("case: sgemm random shape", case, flush=True)
    A, B, C = wl.sgemm_inputs(M * 7 + N * 3 + K, wl.GemmShape(M, N, K), exact=True, c_zero=False)
    got = run_sgemm(A, B, C, lda=K + pa, ldb=N + pb, ldc=N + pc, offset=offset)
    ref, _ = oracle.sgemm(A, B, C)
    assert np.array_equal(got.astype(np.float64), ref), f"{case}: {b.last_variant()}"


IGEMM_SMALL = gemm_cases(1003, 40, 1, 600, 900, 16)
IGEMM_LARGE = gemm_cases(1004, 14, 1300, 3400, 300, 16)
# rows that are 4-byte aligned only (the 4-byte direct-to-LDS loads) in half of these
IGEMM_SMALL_4 = gemm_cases(1009, 30, 1, 600, 900, 4)
IGEMM_LARGE_4 = gemm_cases(1010, 8, 1300, 3400, 1200, 4)


@pytest.mark.parametrize("case", IGEMM_SMALL + IGEMM_LARGE + IGEMM_FEW + IGEMM_SMALL_4 + IGEMM_LARGE_4,
                         ids=lambda c: "x".join(map(str, c)))
def test_igemm_built_in_choice_exact(case):
    M, N, K, pa, pb, pc, offset = case
    print("case: igemm random shape", case, flush=True)
    ti.check((M, N, K), M + N + K, lda=K + pa, ldb=N + pb, ldc=N + pc, offset=offset)


@pytest.mark.parametrize("case", IGEMM_SMALL[:20] + IGEMM_LARGE[:6] + IGEMM_SMALL_4[:12] + IGEMM_LARGE_4[:4],
                         ids=lambda c: "x".join(map(str, c)))
def test_igemm_bt_built_in_choice_exact(case):
    M, N, K, pa, pb, pc, offset = case
    print("case: igemm bt random shape", case, flush=True)
    A, B, C = wl.igemm_inputs(M + N + K, wl.GemmShape(M, N, K), c_zero=False)
    Bt = np.ascontiguousarray(B.T)
    ldbt = K + pb
    bufB = np.full(N * ldbt + offset, 77, np.int8)
    bufB[offset:].reshape(N, ldbt)[:, :K] = Bt
    bufA = np.full(M * (K + pa) + offset, 77, np.int8)
    bufA[offset:].reshape(M, K + pa)[:, :K] = A
    ldc = N + pc
    bufC = np.full(M * ldc + offset, 777, np.int32)
    bufC[offset:].reshape(M, ldc)[:, :N] = C
    dA, dB, dC = dev(bufA), dev(bufB), dev(bufC)
    st = b.igemm_s8s32_bt(M, N, K, dA.data_ptr() + offset, K + pa, dB.data_ptr() + offset, ldbt,
                          dC.data_ptr() + 4 * offset, ldc)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    full = out[offset:].reshape(M, ldc)
    assert np.all(full[:, N:] == 777) and np.all(out[:offset] == 777), "wrote outside C"
    ref = oracle.igemm_s8s32(A, B, C)
    assert np.array_equal(full[:, :N], ref), f"{case}: {b.last_variant()}"


def conv_cases(seed, count, depthwise):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        N = int(rng.integers(1, 5))
        H, W = (int(v) for v in rng.integers(1, 41, 2))
        C = int(rng.choice([1, 3, 4, 5, 8, 12, 16, 20, 24, 32, 40, 48, 64, 72, 96, 130]))
        K = int(rng.integers(1, 200))
        R, S = (int(v) for v in rng.choice([1, 1, 2, 3, 3, 3, 5, 7], 2)) if not depthwise else \
            (int(v) for v in rng.choice([1, 2, 3, 3, 3, 5, 5, 7], 2))
        stride = int(rng.choice([1, 1, 2, 3]))
        pad = int(rng.integers(0, 4))
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        cases.append((N, H, W, C, R, S, stride, pad) if depthwise else (N, H, W, C, K, R, S, stride, pad))
    return cases


@pytest.mark.parametrize("case", conv_cases(1005, 60, False), ids=lambda c: "x".join(map(str, c)))
def test_conv2d_built_in_choice_exact(case):
    print("case: conv random shape", case, flush=True)
    tc.check(wl.ConvShape(*case), sum(case), exact=True)


@pytest.mark.parametrize("case", conv_cases(1006, 50, True), ids=lambda c: "x".join(map(str, c)))
def test_dwconv2d_built_in_choice_exact(case):
    print("case: dwconv random shape", case, flush=True)
    post = (b.POST_NONE, b.POST_RELU)[sum(case) % 2]
    td.check(wl.DwConvShape(*case), sum(case), exact=True, with_bias=sum(case) % 3 == 0, post=post)
