"""GPU parity of sgemm against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, assert_close, dev, run_sgemm
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    yield
    b.set_tuning(-1, 0)


def check(A, B, C, exact=False, **kw):
    got = run_sgemm(A, B, C, **kw)
    ref, absum = oracle.sgemm(A, B, C)
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), f"not bit-exact ({b.last_variant()})"
        return 0.0
    return assert_close(got, ref, absum, what=b.last_variant())


def test_config_small_64():
    seed, shape = wl.SGEMM_SMALL
    print("case: sgemm 64^3 seed", seed, flush=True)
    ratio = check(*wl.sgemm_inputs(seed, shape))
    assert ratio < TOL


def test_hand_sum_on_gpu():
    A = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    B = np.array([[7, 8], [9, 10], [11, 12]], np.float32)
    C = np.array([[1, -1], [0, 2]], np.float32)
    got = run_sgemm(A, B, C)
    assert np.array_equal(got, np.array([[59, 63], [139, 156]], np.float32))


N_VARIANTS = len(b.variant_names())


@pytest.mark.parametrize("variant", range(N_VARIANTS))
@pytest.mark.parametrize("split", [1, 3])
def test_every_variant_exact_integers(variant, split):
    # integers in [-8, 8]: every partial sum is exactly representable, so any summation
    # order (and split-K with atomics) must reproduce the oracle bit for bit.  The shape
    # spans several tiles of every variant and leaves a ragged tail in M, N and K.
    print("case: exact integers variant", variant, "split", split, flush=True)
    assert b.set_tuning(variant, split) == b.OK
    shape = wl.GemmShape(300, 290, 203)
    A, B, C = wl.sgemm_inputs(31, shape, exact=True, c_zero=False)
    check(A, B, C, exact=True)
    name = b.variant_names()[variant]
    # the aligned-only kernels cannot take this ragged shape: the built-in choice runs instead
    assert b.last_variant() == name or "dma" in name or "rows" in name or "cols" in name


@pytest.mark.parametrize("variant", range(N_VARIANTS))
@pytest.mark.parametrize("k", [16, 32, 48, 96, 112])
def test_every_variant_aligned_fast_path_exact(variant, k):
    # K of one to seven chunks exercises every fill level of the load pipeline
    print("case: aligned exact variant", variant, "K", k, flush=True)
    if "cols" in b.variant_names()[variant]:
        pytest.skip("the few-column kernel takes at most 16 columns")
    assert b.set_tuning(variant, 1) == b.OK
    shape = wl.GemmShape(512, 512, k)
    A, B, C = wl.sgemm_inputs(32 + k, shape, exact=True, c_zero=False)
    check(A, B, C, exact=True)
    assert b.last_variant() == b.variant_names()[variant]


@pytest.mark.parametrize("variant", range(2, N_VARIANTS))
def test_aligned_kernels_with_strides_and_random_values(variant):
    if "cols" in b.variant_names()[variant]:
        pytest.skip("the few-column kernel takes at most 16 columns")
    assert b.set_tuning(variant, 1) == b.OK
    A, B, C = wl.sgemm_inputs(33, wl.GemmShape(768, 640, 208), c_zero=False)
    check(A, B, C, lda=212, ldb=648, ldc=642)
    assert b.last_variant() == b.variant_names()[variant]


EDGE_VARIANTS = [i for i, n in enumerate(b.variant_names()) if "_dma_edge_" in n]


@pytest.mark.parametrize("variant", EDGE_VARIANTS)
@pytest.mark.parametrize("split", [1, 3])
@pytest.mark.parametrize("shape,ld", [((300, 292, 204), (204, 292, 292)), ((129, 67, 36), (40, 68, 71)),
                                      ((1, 4, 4), (4, 4, 4)), ((64, 64, 4), (4, 64, 64)),
                                      ((200, 131, 1000), (1004, 132, 131)), ((128, 128, 64), (64, 128, 128))])
def test_ragged_direct_to_lds_kernels_exact(variant, split, shape, ld):
    # rows 16-byte aligned and K % 4 == 0, everything else ragged: groups past M, N or the
    # end of a K slice must come from the zero block (the padding is NaN-poisoned)
    print("case: edge dma variant", variant, "split", split, shape, ld, flush=True)
    assert "edge" in b.variant_names()[variant]
    assert b.set_tuning(variant, split) == b.OK
    A, B, C = wl.sgemm_inputs(35, wl.GemmShape(*shape), exact=True, c_zero=False)
    check(A, B, C, exact=True, lda=ld[0], ldb=ld[1], ldc=ld[2])
    assert b.last_variant() == b.variant_names()[variant]


def test_ragged_aligned_shapes_take_the_direct_to_lds_kernel():
    A, B, C = wl.sgemm_inputs(36, wl.GemmShape(3000, 3000, 300), c_zero=False)
    assert check(A, B, C) < TOL
    assert "dma_edge" in b.last_variant()
    # K % 4 != 0 or rows that are not 16-byte aligned: the same kernels with 4-byte loads ...
    A, B, C = wl.sgemm_inputs(37, wl.GemmShape(500, 500, 502), c_zero=False)
    assert check(A, B, C) < TOL
    assert "dma_edge4" in b.last_variant()
    # ... and the register-staged kernel for reductions shorter than a step of those
    A, B, C = wl.sgemm_inputs(38, wl.GemmShape(100, 100, 30), c_zero=False)
    assert check(A, B, C) < TOL
    assert "dma" not in b.last_variant()


def test_identity_is_bit_exact_with_strides():
    rng = np.random.default_rng(41)
    n = 200
    B = wl.uniform_f32(rng, (n, 150))
    C = wl.uniform_f32(rng, (n, 150))
    got = run_sgemm(np.eye(n, dtype=np.float32), B, C, lda=n + 3, ldb=157, ldc=163)
    assert np.array_equal(got, C + B)


def test_zero_operand_and_k_zero_leave_c():
    rng = np.random.default_rng(42)
    C = wl.uniform_f32(rng, (70, 90))
    B = wl.uniform_f32(rng, (33, 90))
    got = run_sgemm(np.zeros((70, 33), np.float32), B, C)
    assert np.array_equal(got, C)
    dC = dev(C)
    assert b.sgemm(70, 90, 0, 0, 1, 0, 90, dC.data_ptr(), 90) == b.OK
    assert b.sgemm(0, 90, 5, 0, 5, 0, 90, dC.data_ptr(), 90) == b.OK
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C)


@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 257, 19), (257, 1, 19), (5, 7, 1), (33, 65, 33),
                                   (127, 129, 17), (128, 128, 16), (129, 127, 15)])
def test_degenerate_and_ragged_shapes(shape):
    print("case: ragged", shape, flush=True)
    A, B, C = wl.sgemm_inputs(50 + sum(shape), wl.GemmShape(*shape), c_zero=False)
    check(A, B, C)
    A, B, C = wl.sgemm_inputs(51 + sum(shape), wl.GemmShape(*shape), exact=True, c_zero=False)
    check(A, B, C, exact=True)


@pytest.mark.parametrize("lda,ldb,ldc,offset", [(260, 300, 301, 0), (259, 297, 299, 0),
                                                (256, 296, 296, 1), (256, 296, 296, 4)])
def test_leading_dimensions_and_misaligned_bases(lda, ldb, ldc, offset):
    # 16-byte aligned rows take the vector path, everything else the element-wise one
    print("case: ld", lda, ldb, ldc, "offset", offset, flush=True)
    A, B, C = wl.sgemm_inputs(61, wl.GemmShape(260, 296, 256), exact=True, c_zero=False)
    check(A, B, C, exact=True, lda=lda, ldb=ldb, ldc=ldc, offset=offset)


@pytest.mark.parametrize("n", [128, 256, 512])
def test_table1_matrix_sizes(n):
    A, B, C = wl.sgemm_inputs(70 + n, wl.GemmShape(n, n, n))
    assert check(A, B, C) < TOL


def test_config_ragged_four_shapes():
    for shape, A, B, C in wl.sgemm_ragged_inputs():
        print("case: ragged config", shape, flush=True)
        ratio = check(A, B, C)
        print("   variant", b.last_variant(), "max err/absum", ratio, flush=True)
        assert ratio < TOL


def test_accumulates_into_existing_c_twice():
    A, B, C = wl.sgemm_inputs(81, wl.GemmShape(256, 256, 64), exact=True, c_zero=False)
    dA, dB, dC = dev(A), dev(B), dev(C)
    for _ in range(2):
        b.sgemm_t(dA, dB, dC)
    torch.cuda.synchronize()
    ref, _ = oracle.sgemm(A, B, C)
    ref2 = ref + (ref - C)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref2)


def test_runs_on_the_stream_it_was_given():
    A, B, C = wl.sgemm_inputs(82, wl.GemmShape(512, 512, 512), exact=True)
    dA, dB = dev(A), dev(B)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        dC = torch.zeros(512, 512, device="cuda")
        b.use_torch_stream()
        b.sgemm_t(dA, dB, dC)
        done = torch.cuda.Event()
        done.record(s)
    done.synchronize()
    b.set_stream(None)
    ref, _ = oracle.sgemm(A, B, C)
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), ref)


def test_config_4096_sampled_outputs():
    seed, shape = wl.SGEMM_4096
    print("case: sgemm 4096^3 seed", seed, flush=True)
    A, B, C = wl.sgemm_inputs(seed, shape)
    dA, dB, dC = dev(A), dev(B), dev(C)
    b.sgemm_t(dA, dB, dC)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    ii, jj = wl.sample_points(5, shape.M, shape.N, 20000)
    ref, absum = oracle.sgemm_points(A, B, C, ii, jj)
    ratio = assert_close(got[ii, jj], ref, absum, what="sampled points")
    # 16 full rows spread over the matrix
    rows = np.linspace(0, shape.M - 1, 16).astype(np.int64)
    ref, absum = oracle.sgemm(A[rows], B, C[rows])
    ratio = max(ratio, assert_close(got[rows], ref, absum, what="full rows"))
    print("   variant", b.last_variant(), "max err/absum", ratio, flush=True)
    # a property that holds at any size: every row sum of C equals A (B 1) within tolerance
    ones = B.astype(np.float64).sum(axis=1)
    rs = A.astype(np.float64) @ ones
    bound = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64).sum(axis=1)
    assert np.all(np.abs(got.astype(np.float64).sum(axis=1) - rs) <= TOL * bound)


@pytest.mark.parametrize("shape,expect", [
    ((2304, 2304, 512), "sgemm_dma_edge_64x64x32_w2x1_k2"),   # 324 tiles of 128 x 128 fill 63 % of two rounds
    ((3000, 3000, 304), "sgemm_dma_edge_64x64x32_w2x1_k2"),   # ragged, 576 tiles of 128 x 128: 2.25 per CU
    ((1024, 1024, 128), "sgemm_dma_edge_64x64x32_w2x1_k2"),   # a 64 x 64 tile per CU, short reduction: two wave sets
    ((1024, 1024, 512), "sgemm_dma_edge_64x64x64_w2x1_k4"),   # the same tiles, a longer one: four wave sets
    ((4096, 2048, 256), "sgemm_dma_128x128x16"),              # 512 tiles: two whole rounds
    ((4096, 4096, 256), "sgemm_dma_128x128x16_w4x2"),         # four 128 x 128 tiles per CU: the eight-wave form, one launch
    ((4096, 4096, 4096), "sgemm_dma_256x128x16_w4x2"),        # a long reduction: 512 tiles of 256 x 128, two per CU
    ((2048, 2048, 256), "sgemm_dma_128x128x16_w4x2"),         # one 128 x 128 tile per CU, short reduction: eight waves
    ((1792, 2048, 1024), "sgemm_dma_128x128x16_w4x2"),        # 224 tiles: seven eighths of the CUs
    ((2048, 2048, 3072), "sgemm_dma_edge_64x64x64_w2x1_k4"),  # a long reduction: 64 x 64 tiles, four wave sets
    ((4096, 3072, 2048), "sgemm_dma_128x128x16_w4x2"),        # 384 of those: 1.5 per CU, so 768 of 128 x 128 instead
    ((4000, 4000, 64), "sgemm_dma_edge_128x128x16"),          # ragged, 1024 tiles: four whole rounds
])
def test_built_in_tile_size_follows_the_fill_of_the_cu_rounds(shape, expect):
    """The kernel the library picks by itself for tile counts that do and do not fill whole
    rounds of the 256 CUs, checked on sampled points and full rows against the oracle."""
    M, N, K = shape
    print("case: sgemm built-in choice", shape, flush=True)
    A, B, C = wl.sgemm_inputs(91, wl.GemmShape(M, N, K))
    dA, dB, dC = dev(A), dev(B), dev(C)
    b.sgemm_t(dA, dB, dC)
    torch.cuda.synchronize()
    assert b.last_variant().startswith(expect), b.last_variant()
    got = dC.cpu().numpy()
    ii, jj = wl.sample_points(6, M, N, 5000)
    ref, absum = oracle.sgemm_points(A, B, C, ii, jj)
    assert_close(got[ii, jj], ref, absum, what="sampled points")
    rows = np.unique(np.concatenate([np.linspace(0, M - 1, 8).astype(np.int64), [63, 64, 127, 128, M - 65, M - 64]]))
    ref, absum = oracle.sgemm(A[rows], B, C[rows])
    assert_close(got[rows], ref, absum, what="full rows")


@pytest.mark.parametrize("shape,name,tail", [
    ((1100, 1100, 1024), "sgemm_dma_edge_64x64x32_w2x1_k2_s3", True),    # 324 tiles: 68 left over, three slices each
    ((1100, 1100, 1024), "sgemm_dma_edge_128x128x16_w2x2_s2", False),    # 81 tiles: fewer than CUs
    ((2181, 2176, 1024), "sgemm_dma_edge_128x128x16_w2x2_s2", True),     # 306 tiles, ragged rows: 50 left over, five slices
    ((2181, 2176, 1024), "sgemm_dma_edge_64x64x32_w2x1_k2_s3", False),   # 1190 tiles: 166 left over, no room for two slices
    ((1283, 1092, 516), "sgemm_dma_edge_64x64x32_w2x1_k2_s3", True),     # 378 tiles, 122 left over in two slices (19.4 against 23.0 us)
    ((1283, 1092, 132), "sgemm_dma_edge_64x64x32_w2x1_k2_s3", False),    # the same tiles, five chunks: too short to cut
])
def test_tail_split_exact(shape, name, tail):
    """More tiles than CUs and an incomplete last round: the left-over tiles run as slices of
    the reduction that add their partial sums atomically (on the 256 CUs of an MI355X, when
    that saves more than the atomics cost).  Small integers: bit-exact in any order."""
    M, N, K = shape
    print("case: sgemm tail split", shape, name, flush=True)
    variant = b.variant_names().index(name)
    A, B, C = wl.sgemm_inputs(95, wl.GemmShape(M, N, K), exact=True, c_zero=False)
    assert b.set_tuning(variant, 0) == b.OK
    got = run_sgemm(A, B, C)
    ran = b.last_variant()
    b.set_tuning(-1, 0)
    assert ran == name + ("_tail" if tail else ""), ran
    ref, _ = oracle.sgemm(A, B, C)
    assert np.array_equal(got.astype(np.float64), ref), ran
    # the same call with every split switched off gives the same values
    assert b.set_tuning(variant, 1) == b.OK
    again = run_sgemm(A, B, C)
    assert b.last_variant() == name, b.last_variant()
    b.set_tuning(-1, 0)
    assert np.array_equal(again, got)


def test_reduction_kept_in_one_workgroup_is_reproducible():
    """With the split switched off (split_k = 1) no partial sums meet in atomics: two runs of
    a shape that would otherwise take the tail split agree bit for bit, and the default run
    agrees with them within the tolerance."""
    M, N, K = 1100, 1100, 1024
    A, B, C = wl.sgemm_inputs(96, wl.GemmShape(M, N, K), c_zero=False)
    assert b.set_tuning(-1, 1) == b.OK
    first = run_sgemm(A, B, C)
    assert not b.last_variant().endswith("_tail"), b.last_variant()
    second = run_sgemm(A, B, C)
    b.set_tuning(-1, 0)
    assert np.array_equal(first, second)
    default = run_sgemm(A, B, C)
    assert b.last_variant().endswith("_tail"), b.last_variant()
    ref, absum = oracle.sgemm(A, B, C)
    assert_close(first, ref, absum, what="no split")
    assert_close(default, ref, absum, what="tail split")


DWORD_VARIANTS = [i for i, n in enumerate(b.variant_names()) if "_dma_edge4_" in n]


@pytest.mark.parametrize("variant", DWORD_VARIANTS)
@pytest.mark.parametrize("split", [0, 1, 3])
@pytest.mark.parametrize("offset", [0, 1, 3])
@pytest.mark.parametrize("shape,ld", [((300, 291, 203), (205, 293, 291)), ((129, 67, 37), (41, 69, 71)),
                                      ((1, 1, 1), (1, 1, 1)), ((64, 64, 5), (5, 64, 64)),
                                      ((200, 131, 1001), (1003, 133, 131)), ((128, 128, 64), (64, 128, 128)),
                                      ((1100, 1090, 515), (515, 1090, 1090)), ((2180, 2177, 130), (131, 2179, 2177))])
def test_direct_to_lds_kernel_with_4_byte_loads_exact(variant, split, offset, shape, ld):
    """Rows that start at any element: odd lda, ldb, ldc and K, bases 4 and 12 bytes off a
    16-byte boundary, ragged M and N, with and without a cut of the reduction (the last shape
    has more tiles than CUs: the tail split).  Padding is NaN-poisoned; small integers: exact."""
    print("case: dword dma", variant, split, offset, shape, ld, flush=True)
    assert b.set_tuning(variant, split) == b.OK
    A, B, C = wl.sgemm_inputs(38, wl.GemmShape(*shape), exact=True, c_zero=False)
    check(A, B, C, exact=True, lda=ld[0], ldb=ld[1], ldc=ld[2], offset=offset)
    assert b.last_variant().startswith("sgemm_dma_edge4_"), b.last_variant()


def test_unaligned_rows_take_the_4_byte_loads_when_large():
    """The ragged shape of the workload list (4097 x 129 x 511, lda = 511): built-in choice."""
    A, B, C = wl.sgemm_inputs(39, wl.GemmShape(4097, 129, 511), c_zero=False)
    assert check(A, B, C) < TOL
    assert b.last_variant().startswith("sgemm_dma_edge4_"), b.last_variant()
    A, B, C = wl.sgemm_inputs(40, wl.GemmShape(1000, 1000, 1001), c_zero=False)
    assert check(A, B, C, lda=1001, ldb=1003, ldc=1001) < TOL
    assert b.last_variant().startswith("sgemm_dma_edge4_"), b.last_variant()


ROWS_VARIANTS = [i for i, n in enumerate(b.variant_names()) if "_rows_" in n]


@pytest.mark.parametrize("variant", ROWS_VARIANTS)
@pytest.mark.parametrize("split", [0, 1, 3])
@pytest.mark.parametrize("shape,ld,offset", [
    ((1, 64, 64), (64, 64, 64), 0), ((5, 100, 200), (200, 100, 101), 0), ((16, 1028, 1000), (1004, 1032, 1029), 4),
    ((17, 67, 36), (36, 68, 67), 0), ((32, 64, 4), (4, 64, 64), 8), ((40, 130, 520), (524, 132, 131), 0),
    ((8, 4096, 512), (512, 4096, 4096), 0), ((3, 1, 12), (12, 4, 1), 0),
])
def test_few_row_kernels_exact(variant, split, shape, ld, offset):
    """The kernels for a few rows against a large B (operands straight into registers, MFMA
    16x16x4): M below, at and above their 16 or 32 rows, N not a multiple of 4 or 64, K not a
    multiple of the 16-deep step or the 64-deep slice unit, padded leading dimensions (NaN in
    the padding), with and without a cut of the reduction.  Small integers: exact."""
    print("case: few rows", variant, split, shape, ld, offset, flush=True)
    assert b.set_tuning(variant, split) == b.OK
    A, B, C = wl.sgemm_inputs(41, wl.GemmShape(*shape), exact=True, c_zero=False)
    check(A, B, C, exact=True, lda=ld[0], ldb=ld[1], ldc=ld[2], offset=offset)
    assert b.last_variant() == b.variant_names()[variant], b.last_variant()


def test_few_rows_against_a_large_b_take_the_row_kernels():
    """Built-in choice: 8 and 16 rows against a 1024 x 1024 B run on the 16-row kernel; 24 rows
    (two row tiles), a B below 4 MB, an odd lda, and a caller who keeps the reduction in one
    workgroup do not."""
    for shape, lda, expect in (((8, 1024, 1024), 1024, "sgemm_rows_16x64"), ((16, 1024, 1024), 1024, "sgemm_rows_16x64"),
                               ((24, 1024, 1024), 1024, None), ((8, 512, 1024), 1024, None),
                               ((8, 1024, 1024), 1025, None)):
        A, B, C = wl.sgemm_inputs(42, wl.GemmShape(*shape), exact=True, c_zero=False)
        check(A, B, C, exact=True, lda=lda)
        if expect is None:
            assert "_rows_" not in b.last_variant(), (shape, b.last_variant())
        else:
            assert b.last_variant().startswith(expect), (shape, b.last_variant())
    assert b.set_tuning(-1, 1) == b.OK
    A, B, C = wl.sgemm_inputs(43, wl.GemmShape(8, 1024, 1024), exact=True, c_zero=False)
    check(A, B, C, exact=True)
    assert "_rows_" not in b.last_variant(), b.last_variant()


@pytest.mark.parametrize("shape", [(6144, 4096, 64), (8192, 4096, 64), (4096, 4224, 64), (6100, 4000, 2048), (6101, 4001, 2051)])
def test_outputs_larger_than_one_generation_of_workgroups_exact(shape):
    """More 128 x 128 tiles of the four-wave kernels than the CUs hold at once: 1536 tiles run as launches of 1024 and
    512, 2048 as two of 1024; 1056 tiles as 1024 and 32, the short last generation on the form of
    the tile that requests C at the start.  Every element is compared: a tile computed twice or not at
    all shows."""
    print("case: sgemm generations", shape, flush=True)
    A, B, C = wl.sgemm_inputs(44, wl.GemmShape(*shape), exact=True, c_zero=False)
    # (the library's own choice for these shapes is the eight-wave form of the tile, in one launch)
    if shape[1] in (4096, 4224):
        assert b.set_tuning(b.variant_names().index("sgemm_dma_128x128x16_w2x2_s2_c0"), 0) == b.OK
    if shape[1] == 4000:
        assert b.set_tuning(b.variant_names().index("sgemm_dma_edge_128x128x16_w2x2_s2"), 0) == b.OK
    check(A, B, C, exact=True)
    if shape[1] == 4096:
        assert b.last_variant() == "sgemm_dma_128x128x16_w2x2_s2_c0", b.last_variant()
    if shape[1] == 4000:    # ragged: the buffer-load form of the tile, 1536 tiles as 1024 + 512
        assert b.last_variant() == "sgemm_dma_edge_128x128x16_w2x2_s2", b.last_variant()
    if shape[1] == 4001:    # rows that start at any element: its 4-byte-load form
        assert b.last_variant() == "sgemm_dma_edge4_128x128x16_w2x2_s2", b.last_variant()


@pytest.mark.parametrize("kernel", ["sgemm_dma_128x128x16_w4x2_s2_c0", "sgemm_dma_256x128x16_w4x2_s2_c0"])
@pytest.mark.parametrize("shape", [(4096, 4096, 272), (6144, 4096, 256), (8192, 4096, 512), (512, 65536, 256)])
def test_eight_wave_tiles_in_one_launch_exact(shape, kernel):
    """The tiles on eight waves, two workgroups per CU -- 128 x 128, the library's choice for these
    shapes, and 256 x 128, its choice from K = 4096, forced here: two to sixteen tiles per CU in one
    launch, the CUs' two slots refilling as tiles finish.  Every element is compared: a tile
    computed twice or not at all shows."""
    print("case: sgemm eight-wave tiles", shape, kernel, flush=True)
    A, B, C = wl.sgemm_inputs(46, wl.GemmShape(*shape), exact=True, c_zero=False)
    if kernel.startswith("sgemm_dma_256"):
        assert b.set_tuning(b.variant_names().index(kernel), 0) == b.OK
    check(A, B, C, exact=True)
    assert b.last_variant() == kernel, b.last_variant()

