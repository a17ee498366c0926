"""GPU parity (bit-exact) of igemm_s8s32 against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    b.set_igemm_tuning(-1)
    yield
    b.set_tuning(-1, 0)
    b.set_igemm_tuning(-1)


def run_igemm(A, B, C, lda=None, ldb=None, ldc=None, offset=0):
    M, K = A.shape
    N = B.shape[1]
    lda, ldb, ldc = lda or K, ldb or N, ldc or N

    def place(a, ld, fill):
        buf = np.full(a.shape[0] * ld + offset, fill, a.dtype)
        buf[offset:].reshape(a.shape[0], ld)[:, :a.shape[1]] = a
        return buf

    dA, dB, dC = dev(place(A, lda, 77)), dev(place(B, ldb, 77)), dev(place(C, ldc, 777))
    st = b.igemm_s8s32(M, N, K, dA.data_ptr() + offset, lda, dB.data_ptr() + offset, ldb,
                       dC.data_ptr() + 4 * offset, ldc)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    full = out[offset:].reshape(M, ldc)
    assert np.all(full[:, N:] == 777) and np.all(out[:offset] == 777), "wrote outside C"
    return full[:, :N].copy()


def check(shape, seed, c_zero=False, **kw):
    A, B, C = wl.igemm_inputs(seed, wl.GemmShape(*shape), c_zero=c_zero)
    got = run_igemm(A, B, C, **kw)
    ref = oracle.igemm_s8s32(A, B, C)
    assert np.array_equal(got, ref), f"{shape} {b.last_variant()}: {int((got != ref).sum())} mismatches"


def test_hand_sum_on_gpu():
    A = np.array([[-128, 127], [127, -128]], np.int8)
    B = np.array([[-128, 127], [-128, 127]], np.int8)
    got = run_igemm(A, B, np.zeros((2, 2), np.int32))
    assert np.array_equal(got, np.array([[128, -127], [128, -127]], np.int32))


def test_config_igemm_1024():
    seed, shape = wl.IGEMM_1024
    print("case: igemm 1024^3 seed", seed, flush=True)
    check((shape.M, shape.N, shape.K), seed, c_zero=True)
    print("   variant", b.last_variant(), flush=True)


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 64, 64), (65, 63, 65), (130, 70, 200),
                                   (1, 300, 33), (300, 1, 33), (257, 255, 129), (128, 128, 4096)])
def test_ragged_shapes(shape):
    print("case: igemm", shape, flush=True)
    check(shape, sum(shape))


@pytest.mark.parametrize("split", [1, 2, 5])
def test_split_k_is_bit_exact(split):
    assert b.set_tuning(-1, split) == b.OK
    check((200, 136, 1000), 90 + split)


def test_large_tiles():
    check((2944, 2945, 328), 95)   # rows of B at odd addresses: the register-staged kernel, 128 x 128 tiles
    assert b.last_variant() == "igemm_128x128x64"
    check((2940, 2949, 200), 96)   # a handful of chunks: its 64 x 64 tiles
    assert b.last_variant() == "igemm_64x64x64"
    check((2944, 2944, 328), 95)   # rows of A that are only 4-byte aligned: 128 x 128 tiles on 4-byte loads
    assert b.last_variant().startswith("igemm_dma_edge4_128x128x128"), b.last_variant()


DMA_NAMES = [n for n in b.igemm_variant_names() if n.startswith("igemm_dma_")]


@pytest.mark.parametrize("split", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", [(256, 128, 128), (256, 256, 384), (512, 384, 1024), (768, 128, 640)])
@pytest.mark.parametrize("name", DMA_NAMES)
def test_direct_to_lds_kernels_bit_exact(name, shape, split):
    """Every direct-to-LDS kernel on whole-tile shapes: one chunk, fewer chunks than ring
    stages, several rounds of the ring, slices of unequal length; non-zero C."""
    print("case: igemm dma", name, shape, "split", split, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    assert b.set_tuning(-1, split) == b.OK
    check(shape, 70 + split)
    assert b.last_variant() == name, b.last_variant()


@pytest.mark.parametrize("name", DMA_NAMES)
def test_direct_to_lds_kernels_with_row_padding_and_offsets(name):
    print("case: igemm dma ld", name, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check((256, 256, 256), 75, lda=256 + 32, ldb=256 + 48, ldc=256 + 5, offset=16)
    assert b.last_variant() == name, b.last_variant()
    # rows that are not 16-byte aligned fall back to the register-staged kernels, unless the
    # forced kernel is one of the 4-byte forms and they are 4-byte aligned
    check((256, 256, 256), 76, lda=256 + 8, ldb=256 + 48, ldc=256, offset=0)
    assert b.last_variant() == (name if "_edge4_" in name else "igemm_64x64x64"), b.last_variant()
    check((256, 256, 256), 77, offset=4)
    assert b.last_variant() == (name if "_edge4_" in name else "igemm_64x64x64"), b.last_variant()
    check((256, 256, 256), 77, lda=256 + 9)
    assert not b.last_variant().startswith("igemm_dma"), b.last_variant()
    check((256, 256, 256), 77, offset=2)
    assert not b.last_variant().startswith("igemm_dma"), b.last_variant()


def test_default_choice_takes_the_direct_to_lds_kernels_when_aligned():
    check((1024, 1024, 1024), 78)
    assert b.last_variant().startswith("igemm_dma_"), b.last_variant()
    check((2048, 2048, 256), 79)
    assert b.last_variant().startswith("igemm_dma_"), b.last_variant()
    check((1000, 1024, 1024), 80)     # M not a multiple of the tile: the ragged form of the same kernels
    assert b.last_variant().startswith("igemm_dma_edge_"), b.last_variant()
    check((1000, 1024, 1000), 81)     # rows of A that are only 4-byte aligned: the 4-byte loads
    assert b.last_variant().startswith("igemm_dma_edge4_"), b.last_variant()
    check((1000, 1024, 1001), 81)     # rows of A at odd addresses: the register-staged kernel
    assert not b.last_variant().startswith("igemm_dma_"), b.last_variant()
    check((1000, 1024, 1001), 81, lda=1008)   # K itself may be anything
    assert b.last_variant().startswith("igemm_dma_edge_"), b.last_variant()


def test_extreme_values_through_the_transpose_read():
    # every byte value in every position of a chunk: B[k, n] = ((k * 7 + n * 13) % 256) - 128
    k = np.arange(256)[:, None]
    n = np.arange(128)[None, :]
    B = (((k * 7 + n * 13) % 256) - 128).astype(np.int8)
    A = np.zeros((64, 256), np.int8)
    for i in range(64):
        A[i, (i * 5) % 256] = 1   # row i picks out one row of B
        A[i, (i * 5 + 1) % 256] = -1
    got = run_igemm(A, B, np.zeros((64, 128), np.int32))
    assert b.last_variant().startswith("igemm_dma_"), b.last_variant()
    ref = B[(np.arange(64) * 5) % 256].astype(np.int32) - B[(np.arange(64) * 5 + 1) % 256].astype(np.int32)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("lda,ldb,ldc,offset", [(272, 144, 140, 0), (259, 139, 137, 0),
                                                (272, 144, 140, 1), (272, 144, 140, 16)])
def test_leading_dimensions_and_misaligned_bases(lda, ldb, ldc, offset):
    check((100, 136, 256), 97, lda=lda, ldb=ldb, ldc=ldc, offset=offset)


def test_all_minimum_values():
    A = np.full((64, 1024), -128, np.int8)
    B = np.full((1024, 64), -128, np.int8)
    got = run_igemm(A, B, np.zeros((64, 64), np.int32))
    assert np.all(got == 2**24)


def test_k_zero_leaves_c():
    C = np.arange(12, dtype=np.int32).reshape(3, 4)
    dC = dev(C)
    assert b.igemm_s8s32(3, 4, 0, 0, 1, 0, 4, dC.data_ptr(), 4) == b.OK
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), C)


BIG_NAMES = [n for n in b.igemm_variant_names() if n.startswith("igemm_big_")]
BIG_SHAPES = [(256, 256, 64), (256, 256, 128), (512, 256, 448), (256, 512, 1024), (768, 512, 192)]


@pytest.mark.parametrize("shape", BIG_SHAPES)
@pytest.mark.parametrize("name", BIG_NAMES)
def test_big_tile_kernels_bit_exact(name, shape):
    """The 256 x 256 tile kernels: fewer chunks than ring stages, one more than a ring, many
    rounds of the ring, several tiles in either direction; non-zero C."""
    print("case: igemm big", name, shape, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check(shape, 60)
    assert b.last_variant() == name, b.last_variant()


@pytest.mark.parametrize("name", BIG_NAMES)
def test_big_tile_kernels_with_row_padding_and_offsets(name):
    print("case: igemm big ld", name, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check((256, 512, 320), 61, lda=320 + 32, ldb=512 + 48, ldc=512 + 5, offset=16)
    assert b.last_variant() == name, b.last_variant()
    check((250, 512, 320), 62)   # not whole tiles: another kernel takes it
    assert not b.last_variant().startswith("igemm_big"), b.last_variant()


def test_short_reductions_take_the_eight_wave_tiles_whatever_the_output():
    print("case: igemm default 4096x4096x128", flush=True)
    check((4096, 4096, 128), 63)
    assert b.last_variant().startswith("igemm_dma_64x128x128_w2x4"), b.last_variant()
    check_bt((4096, 4096, 128), 64)
    assert b.last_variant().startswith("igemm_bt_dma_64x128x128_w2x4"), b.last_variant()
    check((4096, 4352, 128), 65)
    assert b.last_variant().startswith("igemm_dma_64x128x128_w2x4"), b.last_variant()


def test_full_size_4096_rows_against_the_oracle():
    """The bench extra's launch (4096^3, 256 tiles of 256 x 256, one per CU): every tile row and
    tile column is hit by the 160 sampled rows, compared bit for bit with the oracle."""
    print("case: igemm 4096^3 sampled rows", flush=True)
    M = N = K = 4096
    A, B, C = wl.igemm_inputs(66, wl.GemmShape(M, N, K), c_zero=False)
    dA, dB, dC = dev(A), dev(B), dev(C)
    b.igemm_s8s32_t(dA, dB, dC)
    torch.cuda.synchronize()
    assert b.last_variant().startswith("igemm_big_"), b.last_variant()
    rows = np.unique(np.concatenate([np.arange(0, M, 256), np.arange(255, M, 256), np.arange(100, M, 32)]))
    got = dC[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref = oracle.igemm_s8s32(np.ascontiguousarray(A[rows]), B, np.ascontiguousarray(C[rows]))
    assert np.array_equal(got, ref), f"{int((got != ref).sum())} mismatches"


def test_big_tile_kernel_extreme_values():
    k = np.arange(128)[:, None]
    n = np.arange(256)[None, :]
    B = (((k * 7 + n * 13) % 256) - 128).astype(np.int8)
    A = np.zeros((256, 128), np.int8)
    for i in range(256):
        A[i, (i * 5) % 128] = 1
        A[i, (i * 5 + 3) % 128] = -1
    assert b.set_igemm_tuning(b.igemm_variant_names().index(BIG_NAMES[0])) == b.OK
    got = run_igemm(A, B, np.zeros((256, 256), np.int32))
    assert b.last_variant() == BIG_NAMES[0], b.last_variant()
    ref = B[(np.arange(256) * 5) % 128].astype(np.int32) - B[(np.arange(256) * 5 + 3) % 128].astype(np.int32)
    assert np.array_equal(got, ref)


# ---- second operand given transposed (N x K, k-contiguous): igemm_s8s32_bt ----

def run_igemm_bt(A, Bt, C, lda=None, ldbt=None, ldc=None, offset=0):
    M, K = A.shape
    N = Bt.shape[0]
    lda, ldbt, ldc = lda or K, ldbt or K, ldc or N

    def place(a, ld, fill):
        buf = np.full(a.shape[0] * ld + offset, fill, a.dtype)
        buf[offset:].reshape(a.shape[0], ld)[:, :a.shape[1]] = a
        return buf

    dA, dB, dC = dev(place(A, lda, 77)), dev(place(Bt, ldbt, 77)), dev(place(C, ldc, 777))
    st = b.igemm_s8s32_bt(M, N, K, dA.data_ptr() + offset, lda, dB.data_ptr() + offset, ldbt,
                          dC.data_ptr() + 4 * offset, ldc)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    full = out[offset:].reshape(M, ldc)
    assert np.all(full[:, N:] == 777) and np.all(out[:offset] == 777), "wrote outside C"
    return full[:, :N].copy()


def check_bt(shape, seed, c_zero=False, **kw):
    A, B, C = wl.igemm_inputs(seed, wl.GemmShape(*shape), c_zero=c_zero)
    Bt = np.ascontiguousarray(B.T)
    got = run_igemm_bt(A, Bt, C, **kw)
    ref = oracle.igemm_s8s32_bt(A, Bt, C)
    assert np.array_equal(got, ref), f"bt {shape} {b.last_variant()}: {int((got != ref).sum())} mismatches"


def test_bt_hand_sum_on_gpu():
    A = np.array([[1, 2, 3], [-4, 5, -6]], np.int8)
    Bt = np.array([[7, -8, 9], [10, 11, -12], [0, 1, 0], [-128, 127, -128]], np.int8)   # 4 x 3
    C = np.array([[1, 0, -1, 5], [0, 2, 0, 0]], np.int32)
    got = run_igemm_bt(A, Bt, C)
    # row 0: 7-16+27=18, 10+22-36=-4, 2, -128+254-384=-258;  row 1: -28-40-54=-122, -40+55+72=87, 5, 512+635+768=1915
    assert np.array_equal(got, np.array([[19, -4, 1, -253], [-122, 89, 5, 1915]], np.int32))


def test_bt_config_igemm_1024():
    seed, shape = wl.IGEMM_1024
    print("case: igemm_bt 1024^3 seed", seed, flush=True)
    check_bt((shape.M, shape.N, shape.K), seed, c_zero=True)
    print("   variant", b.last_variant(), flush=True)
    assert b.last_variant().startswith("igemm_bt_dma_"), b.last_variant()


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (64, 64, 64), (65, 63, 65), (130, 70, 200),
                                   (1, 300, 33), (300, 1, 33), (257, 255, 129), (128, 128, 4096)])
def test_bt_ragged_shapes(shape):
    print("case: igemm_bt", shape, flush=True)
    check_bt(shape, 200 + sum(shape))


@pytest.mark.parametrize("split", [1, 2, 5])
def test_bt_split_k_is_bit_exact(split):
    assert b.set_tuning(-1, split) == b.OK
    check_bt((200, 136, 1000), 290 + split)


def test_bt_large_tiles():
    check_bt((2944, 2944, 329), 295)   # rows at odd addresses: the register-staged kernel
    assert b.last_variant() == "igemm_bt_128x128x64", b.last_variant()
    check_bt((2944, 2944, 328), 295)   # rows that are only 4-byte aligned: 4-byte loads
    assert b.last_variant().startswith("igemm_bt_dma_edge4_128x128x128"), b.last_variant()
    check_bt((2940, 2949, 200), 296)


@pytest.mark.parametrize("split", [0, 1, 2, 3])
@pytest.mark.parametrize("shape", [(256, 128, 128), (256, 256, 384), (512, 384, 1024), (768, 128, 640)])
@pytest.mark.parametrize("name", DMA_NAMES)
def test_bt_direct_to_lds_kernels_bit_exact(name, shape, split):
    print("case: igemm_bt dma", name, shape, "split", split, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    assert b.set_tuning(-1, split) == b.OK
    check_bt(shape, 270 + split)
    assert b.last_variant() == name.replace("igemm_dma_", "igemm_bt_dma_"), b.last_variant()


@pytest.mark.parametrize("name", DMA_NAMES)
def test_bt_direct_to_lds_kernels_with_row_padding_and_offsets(name):
    print("case: igemm_bt dma ld", name, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check_bt((256, 256, 256), 275, lda=256 + 32, ldbt=256 + 48, ldc=256 + 5, offset=16)
    assert b.last_variant() == name.replace("igemm_dma_", "igemm_bt_dma_"), b.last_variant()
    four = name.replace("igemm_dma_", "igemm_bt_dma_") if "_edge4_" in name else "igemm_bt_64x64x64"
    check_bt((256, 256, 256), 276, lda=256 + 16, ldbt=256 + 8, ldc=256, offset=0)
    assert b.last_variant() == four, b.last_variant()
    check_bt((256, 256, 256), 277, offset=4)
    assert b.last_variant() == four, b.last_variant()
    check_bt((256, 256, 256), 277, ldbt=256 + 6)
    assert not b.last_variant().startswith("igemm_bt_dma"), b.last_variant()


@pytest.mark.parametrize("lda,ldbt,ldc,offset", [(272, 288, 140, 0), (259, 261, 137, 0),
                                                 (272, 288, 140, 1), (272, 288, 140, 16)])
def test_bt_leading_dimensions_and_misaligned_bases(lda, ldbt, ldc, offset):
    check_bt((100, 136, 256), 297, lda=lda, ldbt=ldbt, ldc=ldc, offset=offset)


def test_bt_equals_plain_call_on_the_transpose():
    A, B, C = wl.igemm_inputs(298, wl.GemmShape(384, 256, 512), c_zero=False)
    assert np.array_equal(run_igemm_bt(A, np.ascontiguousarray(B.T), C), run_igemm(A, B, C))


def test_bt_after_packing_with_tensor_copy():
    """The pipeline the call exists for: pack B (K x N) k-contiguously with the single-operand
    contraction, then multiply."""
    A, B, C = wl.igemm_inputs(299, wl.GemmShape(256, 384, 640), c_zero=True)
    dA, dB, dC = dev(A), dev(B), dev(C)
    dBt = torch.empty((384, 640), dtype=torch.int8, device="cuda")
    b.tensor_copy_t(dB.t(), dBt)
    b.igemm_s8s32_bt_t(dA, dBt, dC)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), oracle.igemm_s8s32(A, B, C))


@pytest.mark.parametrize("shape", BIG_SHAPES)
@pytest.mark.parametrize("name", BIG_NAMES)
def test_bt_big_tile_kernels_bit_exact(name, shape):
    print("case: igemm_bt big", name, shape, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check_bt(shape, 260)
    assert b.last_variant() == name.replace("igemm_big_", "igemm_bt_big_"), b.last_variant()


@pytest.mark.parametrize("name", BIG_NAMES)
def test_bt_big_tile_kernels_with_row_padding_and_offsets(name):
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check_bt((512, 256, 320), 261, lda=320 + 32, ldbt=320 + 48, ldc=256 + 5, offset=16)
    assert b.last_variant() == name.replace("igemm_big_", "igemm_bt_big_"), b.last_variant()


@pytest.mark.parametrize("shape,expect", [
    ((3072, 3072, 3072), "igemm_big_256x256x64"),   # 144 tiles of 256 x 256: one round on more than half the CUs
    ((3072, 3072, 256), "igemm_dma_64x128x128_w2x4"),  # the same output, a short reduction: small tiles of eight waves
    ((2048, 4096, 2048), "igemm_big_256x128x64"),   # 128 tiles of 256 x 256: halves, one per CU
    ((4096, 4096, 2048), "igemm_big_256x128x64"),   # 256 tiles: halves, two per CU out of step
    ((2048, 2048, 256), "igemm_dma_64x128x128"),    # 128 x 128 tiles would give each CU exactly one
    ((2560, 2560, 2048), "igemm_dma_128x128x128"),  # 400 tiles of 128 x 128
    ((2560, 2560, 256), "igemm_dma_64x128x128_w2x4"),  # the same output, a short reduction
])
def test_built_in_tile_size_for_partial_rounds(shape, expect):
    """The kernel the library picks by itself when the largest tiles do not fill a round of
    the CUs; sampled rows compared bit for bit with the oracle."""
    M, N, K = shape
    print("case: igemm built-in choice", shape, flush=True)
    A, B, C = wl.igemm_inputs(67, wl.GemmShape(M, N, K), c_zero=False)
    dA, dB, dC = dev(A), dev(B), dev(C)
    b.igemm_s8s32_t(dA, dB, dC)
    torch.cuda.synchronize()
    assert b.last_variant().startswith(expect), b.last_variant()
    rows = np.unique(np.concatenate([np.arange(0, M, 256), np.arange(255, M, 256), np.arange(37, M, 101)]))
    got = dC[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref = oracle.igemm_s8s32(np.ascontiguousarray(A[rows]), B, np.ascontiguousarray(C[rows]))
    assert np.array_equal(got, ref), f"{int((got != ref).sum())} mismatches"


# ---- ragged M, N, K on the direct-to-LDS kernels (buffer loads that return zeros past the edges) ----

IEDGE_NAMES = [n for n in b.igemm_variant_names() if "_dma_edge_" in n]


@pytest.mark.parametrize("split", [1, 3])
@pytest.mark.parametrize("name", IEDGE_NAMES)
@pytest.mark.parametrize("shape,ld", [((300, 304, 208), (208, 304, 304)), ((129, 80, 48), (64, 96, 83)),
                                      ((1, 16, 16), (16, 16, 16)), ((64, 128, 128), (128, 128, 128)),
                                      ((200, 144, 1008), (1024, 160, 147)), ((385, 400, 272), (272, 400, 401)),
                                      ((300, 301, 208), (208, 304, 301)), ((129, 77, 48), (64, 80, 83)),
                                      ((70, 1, 32), (32, 16, 1)), ((300, 301, 203), (208, 304, 301)),
                                      ((129, 77, 1), (16, 80, 83)), ((200, 144, 1001), (1024, 160, 147))])
def test_ragged_direct_to_lds_kernels_exact(name, split, shape, ld):
    """M arbitrary, K anything (the row pitch of A a multiple of 16), N a multiple of 16 or (with
    a row pitch that is one) anything, padded
    leading dimensions (padding bytes are 77: a stray read would show), whole and cut reduction."""
    print("case: igemm edge", name, split, shape, ld, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    assert b.set_tuning(-1, split) == b.OK
    check(shape, 71, lda=ld[0], ldb=ld[1], ldc=ld[2])
    assert b.last_variant() == name, b.last_variant()


@pytest.mark.parametrize("name", IEDGE_NAMES)
@pytest.mark.parametrize("shape,ld", [((300, 301, 208), (208, 208, 301)), ((129, 77, 48), (64, 64, 83)),
                                      ((200, 131, 1008), (1024, 1040, 131)), ((1, 1, 16), (16, 16, 1))])
def test_ragged_direct_to_lds_kernels_exact_bt(name, shape, ld):
    """Second operand k-contiguous (N x K): N need not be a multiple of anything."""
    print("case: igemm bt edge", name, shape, ld, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check_bt(shape, 72, lda=ld[0], ldbt=ld[1], ldc=ld[2])
    assert b.last_variant() == name.replace("igemm_dma", "igemm_bt_dma"), b.last_variant()


IEDGE4_NAMES = [n for n in b.igemm_variant_names() if "_dma_edge4_" in n]


@pytest.mark.parametrize("split", [1, 3])
@pytest.mark.parametrize("name", IEDGE4_NAMES)
@pytest.mark.parametrize("shape,ld", [((300, 300, 204), (204, 300, 300)), ((129, 77, 45), (52, 84, 83)),
                                      ((1, 4, 4), (4, 4, 4)), ((64, 128, 128), (128, 128, 128)),
                                      ((200, 140, 1001), (1004, 148, 147)), ((385, 399, 270), (276, 404, 401)),
                                      ((70, 1, 30), (36, 4, 1)), ((3, 5, 7), (8, 8, 5)),
                                      ((1000, 1000, 1000), (1000, 1000, 1000))])
def test_ragged_4_byte_direct_to_lds_kernels_exact(name, split, shape, ld):
    """The 4-byte loads: bases and row pitches multiples of 4 only; M, N, K anything; padding bytes
    are 77 (a stray read would show); whole and cut reduction."""
    print("case: igemm edge4", name, split, shape, ld, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    assert b.set_tuning(-1, split) == b.OK
    check(shape, 74, lda=ld[0], ldb=ld[1], ldc=ld[2], offset=4 if shape[0] == 129 else 0)
    assert b.last_variant() == name, b.last_variant()


@pytest.mark.parametrize("name", IEDGE4_NAMES)
@pytest.mark.parametrize("shape,ld", [((300, 301, 204), (204, 212, 301)), ((129, 77, 44), (52, 60, 83)),
                                      ((200, 131, 1004), (1004, 1012, 131)), ((1, 1, 4), (4, 4, 1)),
                                      ((1000, 1000, 1000), (1000, 1000, 1000))])
def test_ragged_4_byte_direct_to_lds_kernels_exact_bt(name, shape, ld):
    """Second operand k-contiguous (N x K): K a multiple of 4, N anything."""
    print("case: igemm bt edge4", name, shape, ld, flush=True)
    assert b.set_igemm_tuning(b.igemm_variant_names().index(name)) == b.OK
    check_bt(shape, 75, lda=ld[0], ldbt=ld[1], ldc=ld[2])
    assert b.last_variant() == name.replace("igemm_dma", "igemm_bt_dma"), b.last_variant()
    # K not a multiple of 4: both operands would bring bytes from past K
    check_bt((shape[0], shape[1], shape[2] - 1), 75, lda=ld[0], ldbt=ld[1], ldc=ld[2])
    assert "dma" not in b.last_variant(), b.last_variant()


def test_ragged_aligned_shapes_take_the_direct_to_lds_kernels():
    """Built-in choice: 4100 x 4112 x 2064 (N, K multiples of 16) runs on the ragged 128 x 128
    kernel and so does 2200 x 2208 x 528 (a short reduction, every tile resident at once), 3000 x 3008 x 1008
    and 1000 x 1008 x 528 on the 64-row ones; K = 520 (rows of A multiples of 4, not 16) on the
    4-byte loads, K = 521 (rows at odd addresses) on the register-staged kernel.  Sampled rows
    against the oracle."""
    for shape, expect in (((4100, 4112, 2064), "igemm_dma_edge_128x128x128"), ((2200, 2208, 528), "igemm_dma_edge_128x128x128_w2x4"),
                          ((3000, 3008, 1008), "igemm_dma_edge_64x128x128_w2x4"),
                          ((1000, 1008, 528), "igemm_dma_edge_64x128x128"),
                          ((1000, 1008, 520), "igemm_dma_edge4_64x128x128"), ((1000, 1008, 521), "igemm_")):
        M, N, K = shape
        A, B, C = wl.igemm_inputs(73, wl.GemmShape(M, N, K), c_zero=False)
        dA, dB, dC = dev(A), dev(B), dev(C)
        b.igemm_s8s32_t(dA, dB, dC)
        torch.cuda.synchronize()
        assert b.last_variant().startswith(expect), b.last_variant()
        if expect == "igemm_":
            assert "dma" not in b.last_variant(), b.last_variant()
        rows = np.unique(np.concatenate([np.arange(0, M, 128), np.arange(127, M, 128), [M - 1, M - 2], np.arange(37, M, 101)]))
        got = dC[torch.from_numpy(rows).cuda()].cpu().numpy()
        ref = oracle.igemm_s8s32(np.ascontiguousarray(A[rows]), B, np.ascontiguousarray(C[rows]))
        assert np.array_equal(got, ref), f"{shape}: {int((got != ref).sum())} mismatches"
