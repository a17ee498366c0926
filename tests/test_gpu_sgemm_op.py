"""GPU parity of sgemm_op (products on operands stored transposed) against the CPU oracle,
through the C ABI: every kernel variant on every combination of layouts."""
import numpy as np
import pytest

import oracle
from golden_io import read_cases
from gpu_util import TOL, assert_close, run_sgemm
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu

OPS = [(False, True), (True, False), (True, True)]
N_VARIANTS = len(b.variant_names())
SUFFIX = {(False, False): "", (False, True): "_nt", (True, False): "_tn", (True, True): "_tt"}


@pytest.fixture(autouse=True)
def _defaults():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    yield
    b.set_tuning(-1, 0)


def transposed(x):
    out = np.empty(x.shape[::-1], x.dtype)   # fresh row-major storage, also for a single row or column
    out[...] = x.T
    return out


def stored(a, bm, ta, tb):
    return (transposed(a) if ta else a), (transposed(bm) if tb else bm)


def check(a, bm, c, ta, tb, exact=False, **kw):
    """a (M x K), bm (K x N): the operands; the call gets their stored forms."""
    A, B = stored(a, bm, ta, tb)
    got = run_sgemm(A, B, c, ta=ta, tb=tb, **kw)
    ref, absum = oracle.sgemm_op(ta, tb, A, B, c)
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), f"not bit-exact ({b.last_variant()})"
        return 0.0
    return assert_close(got, ref, absum, what=b.last_variant())


@pytest.mark.parametrize("name", sorted(read_cases("sgemm_op_hand.txt")))
def test_hand_sums_on_gpu(name):
    c = read_cases("sgemm_op_hand.txt")[name]
    A, B, Cin = (c[k].astype(np.float32) for k in ("A", "B", "Cin"))
    got = run_sgemm(A, B, Cin, ta=bool(c["ta"]), tb=bool(c["tb"]))
    assert np.array_equal(got.astype(np.float64), c["expect"])


@pytest.mark.parametrize("ta,tb", OPS)
@pytest.mark.parametrize("variant", range(N_VARIANTS))
@pytest.mark.parametrize("split", [1, 3])
def test_every_variant_exact_integers(ta, tb, variant, split):
    # ragged in M, N and K, rows that start at any element: the aligned-only kernels hand over
    # to the built-in choice, everything else must reproduce the oracle bit for bit
    print("case: op exact integers", ta, tb, "variant", variant, "split", split, flush=True)
    assert b.set_tuning(variant, split) == b.OK
    a, bm, c = wl.sgemm_inputs(51, wl.GemmShape(300, 290, 203), exact=True, c_zero=False)
    check(a, bm, c, ta, tb, exact=True)
    name = b.variant_names()[variant]
    assert b.last_variant() == name + SUFFIX[ta, tb] or "dma" in name or "rows" in name or "cols" in name


@pytest.mark.parametrize("ta,tb", OPS)
@pytest.mark.parametrize("variant", range(N_VARIANTS))
@pytest.mark.parametrize("k", [16, 48, 112])
def test_every_variant_whole_tiles_exact(ta, tb, variant, k):
    print("case: op aligned exact", ta, tb, "variant", variant, "K", k, flush=True)
    if "rows" in b.variant_names()[variant] and ta:
        pytest.skip("the few-row kernels take A as given only")
    if "cols" in b.variant_names()[variant]:
        pytest.skip("the few-column kernel takes at most 16 columns")
    assert b.set_tuning(variant, 1) == b.OK
    a, bm, c = wl.sgemm_inputs(52 + k, wl.GemmShape(512, 512, k), exact=True, c_zero=False)
    check(a, bm, c, ta, tb, exact=True)
    assert b.last_variant() == b.variant_names()[variant] + SUFFIX[ta, tb]


EDGE = [i for i, n in enumerate(b.variant_names()) if "_dma_edge" in n]


@pytest.mark.parametrize("ta,tb", OPS)
@pytest.mark.parametrize("variant", EDGE)
@pytest.mark.parametrize("split", [1, 3])
@pytest.mark.parametrize("shape", [(300, 292, 204), (129, 67, 36), (1, 4, 4), (64, 64, 4), (200, 131, 1000),
                                   (128, 128, 64), (77, 260, 132)])
def test_ragged_buffer_load_kernels_exact(ta, tb, variant, split, shape):
    # stored rows 16-byte aligned (padded to a multiple of four elements, the padding
    # NaN-poisoned), K % 4 == 0: groups past M, N or the end of a K slice must arrive as zeros
    print("case: op edge", ta, tb, "variant", variant, "split", split, shape, flush=True)
    assert b.set_tuning(variant, split) == b.OK
    M, N, K = shape
    a, bm, c = wl.sgemm_inputs(53, wl.GemmShape(M, N, K), exact=True, c_zero=False)
    pad4 = lambda n: (n + 3) // 4 * 4 + 4
    lda = pad4(M if ta else K)
    ldb = pad4(K if tb else N)
    check(a, bm, c, ta, tb, exact=True, lda=lda, ldb=ldb, ldc=N + 1)
    assert b.last_variant() == b.variant_names()[variant] + SUFFIX[ta, tb]


@pytest.mark.parametrize("ta,tb", OPS)
def test_tn_needs_no_multiple_of_four_in_k(ta, tb):
    # with neither operand k-contiguous (A transposed, B plain) the 16-byte kernels take any K
    a, bm, c = wl.sgemm_inputs(54, wl.GemmShape(1024, 1024, 1023), exact=True, c_zero=False)
    check(a, bm, c, ta, tb, exact=True)
    assert ("edge4" in b.last_variant()) == (not ta or tb)


@pytest.mark.parametrize("ta,tb", OPS)
@pytest.mark.parametrize("shape,ld", [((768, 640, 208), (4, 8, 2)), ((1000, 1000, 1000), (0, 0, 0)),
                                      ((2048, 2048, 256), (0, 0, 0)), ((1001, 517, 333), (3, 1, 5)),
                                      ((64, 64, 64), (0, 0, 0)), ((5, 4096, 2048), (0, 0, 0))])
def test_built_in_choice_random_values(ta, tb, shape, ld):
    print("case: op random", ta, tb, shape, ld, flush=True)
    M, N, K = shape
    a, bm, c = wl.sgemm_inputs(55, wl.GemmShape(M, N, K), c_zero=False)
    lda = (M if ta else K) + ld[0]
    ldb = (K if tb else N) + ld[1]
    assert check(a, bm, c, ta, tb, lda=lda, ldb=ldb, ldc=N + ld[2]) < TOL
    assert b.last_variant().endswith(SUFFIX[ta, tb])


@pytest.mark.parametrize("ta,tb", OPS)
def test_base_offsets_off_sixteen_bytes(ta, tb):
    a, bm, c = wl.sgemm_inputs(56, wl.GemmShape(260, 200, 132), exact=True, c_zero=False)
    check(a, bm, c, ta, tb, exact=True, offset=3)


def test_validation_uses_the_stored_row_lengths():
    P = 4096
    assert b.sgemm_op(1, 0, 8, 4, 2, P, 7, P, 4, P, 4) == b.ERR_LD     # stored A is 2 x 8: lda >= 8
    assert b.sgemm_op(1, 0, 8, 4, 2, P, 8, P, 3, P, 4) == b.ERR_LD
    assert b.sgemm_op(0, 1, 8, 4, 2, P, 2, P, 1, P, 4) == b.ERR_LD     # stored B is 4 x 2: ldb >= 2
    assert b.sgemm_op(0, 1, 8, 4, 2, P, 2, P, 2, P, 3) == b.ERR_LD
    assert b.sgemm_op(1, 1, -1, 4, 2, P, 8, P, 2, P, 4) == b.ERR_DIM
    assert b.sgemm_op(1, 1, 8, 4, 2, 0, 8, P, 2, P, 4) == b.ERR_NULL
    assert b.sgemm_op(1, 1, 0, 4, 2, 0, 1, 0, 2, 0, 4) == b.OK


@pytest.mark.parametrize("shape,ld", [((1, 2048, 1024), (0, 0, 0)), ((8, 1100, 1028), (4, 8, 3)), ((16, 1091, 2052), (0, 12, 0)),
                                      ((13, 4096, 516), (8, 0, 1)), ((3, 1101, 1300), (4, 8, 3)), ((4, 2050, 772), (0, 4, 2))])
def test_a_few_rows_against_a_transposed_b_take_the_streaming_kernel(shape, ld):
    """A fully connected layer at a small batch with its weights stored output-major (N x K): the
    kernel that streams the weights into registers, exact on small integers; N ragged, K a
    multiple of 4 and not of the 32-element step, padded rows."""
    M, N, K = shape
    a, bm, c = wl.sgemm_inputs(61 + M, wl.GemmShape(M, N, K), exact=True, c_zero=False)
    check(a, bm, c, False, True, exact=True, lda=K + ld[0], ldb=K + ld[1], ldc=N + ld[2])
    assert b.last_variant().startswith("sgemm_rows_16x64x64_w4_nt"), b.last_variant()
    a, bm, c = wl.sgemm_inputs(62 + M, wl.GemmShape(M, N, K), c_zero=False)
    assert check(a, bm, c, False, True, lda=K + ld[0], ldb=K + ld[1], ldc=N + ld[2]) < TOL


@pytest.mark.parametrize("tb", [False, True])
@pytest.mark.parametrize("shape,ld", [((2048, 1, 1024), (0, 0, 0)), ((1100, 8, 1028), (4, 8, 3)), ((4099, 16, 516), (8, 0, 1)),
                                      ((1300, 5, 2052), (0, 12, 0)), ((70000, 3, 16), (0, 0, 0)), ((4099, 4, 516), (8, 0, 1)),
                                      ((2049, 2, 1300), (4, 8, 0)), ((1025, 3, 4096), (0, 4, 3))])
def test_a_few_columns_against_a_large_a_take_the_streaming_kernel(shape, ld, tb):
    """A matrix-vector product and its relatives (N up to 16): the few-row kernel on the transposed
    problem, A streamed, B as given (K x N, read by the element) or transposed (N x K); exact on
    small integers, within tolerance on random values; M ragged, padded rows."""
    M, N, K = shape
    a, bm, c = wl.sgemm_inputs(71 + N, wl.GemmShape(M, N, K), exact=True, c_zero=False)
    ldb = (K if tb else N) + (ld[1] if tb else ld[1] // 4)
    kw = dict(lda=K + ld[0], ldb=ldb, ldc=N + ld[2])
    if tb:
        check(a, bm, c, False, True, exact=True, **kw)
    else:
        got = run_sgemm(a, bm, c, **kw)
        ref, _ = oracle.sgemm(a, bm, c)
        assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
    # (a short reduction stays on the tile kernels, where the call is its epilogue, unless B's rows
    # are not 16-byte aligned)
    expect_cols = K >= 32 + 12 * N or (not tb and ldb % 4 != 0)
    assert b.last_variant().startswith("sgemm_cols_64x16x64_w4") == expect_cols, b.last_variant()
    a, bm, c = wl.sgemm_inputs(72 + N, wl.GemmShape(M, N, K), c_zero=False)
    if tb:
        assert check(a, bm, c, False, True, **kw) < TOL
    else:
        got = run_sgemm(a, bm, c, **kw)
        ref, absum = oracle.sgemm(a, bm, c)
        assert assert_close(got, ref, absum, what=b.last_variant()) < TOL


@pytest.mark.parametrize("ta,tb", OPS)
@pytest.mark.parametrize("shape,ld", [((4096, 4096, 272), (0, 0, 0)), ((512, 32768, 288), (8, 4, 16))])
@pytest.mark.parametrize("kernel", ["sgemm_dma_128x128x16_w4x2_s2_c0", "sgemm_dma_256x128x16_w4x2_s2_c0"])
def test_eight_wave_tiles_on_transposed_operands_exact(ta, tb, shape, ld, kernel):
    """The eight-wave tiles the library takes when every CU gets the same number of them (128 x 128
    by itself here, 256 x 128 forced), on operands stored transposed, with padded rows: every
    element against the oracle."""
    print("case: sgemm_op eight-wave tiles", ta, tb, shape, ld, kernel, flush=True)
    a, bm, c = wl.sgemm_inputs(81, wl.GemmShape(*shape), exact=True, c_zero=False)
    A, B = stored(a, bm, ta, tb)
    if kernel.startswith("sgemm_dma_256"):
        assert b.set_tuning(b.variant_names().index(kernel), 0) == b.OK
    check(a, bm, c, ta, tb, exact=True, lda=A.shape[1] + ld[0], ldb=B.shape[1] + ld[1], ldc=shape[1] + ld[2])
    assert b.last_variant() == kernel + SUFFIX[(ta, tb)], b.last_variant()
