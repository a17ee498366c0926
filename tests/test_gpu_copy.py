"""GPU parity (bit-exact) of tensor_copy_f32 / tensor_copy_s8 against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev
from paper_2205_00618_amd import binding as b

pytestmark = pytest.mark.gpu


def run_copy(x, dims, strides, offset=0, out_offset=0):
    """x: flat numpy buffer (float32 or int8).  The output buffer has guard elements on both sides."""
    dx = dev(x)
    total = int(np.prod(dims))
    guard = 64
    fill = 99 if x.dtype == np.int8 else 777.0
    buf = torch.full((total + 2 * guard + out_offset,), fill, dtype=dx.dtype, device="cuda")
    fn = b.tensor_copy_f32 if x.dtype == np.float32 else b.tensor_copy_s8
    esz = x.dtype.itemsize
    b.set_stream(None)
    st = fn(*[int(v) for v in dims], *[int(v) for v in strides], dx.data_ptr() + offset * esz,
            buf.data_ptr() + (guard + out_offset) * esz)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert np.all(host[:guard + out_offset] == fill) and np.all(host[guard + out_offset + total:] == fill), "wrote outside out"
    return host[guard + out_offset:guard + out_offset + total].reshape(dims)


def data(dtype, n, seed):
    rng = np.random.default_rng(seed)
    if dtype == np.int8:
        return rng.integers(-128, 128, size=n, dtype=np.int8)
    return rng.standard_normal(n).astype(np.float32)


def check(dtype, dims, strides, offset=0, out_offset=0, expect=None, seed=1):
    dims, strides = list(dims), list(strides)
    need = offset + sum((d - 1) * s for d, s in zip(dims, strides)) + 1
    x = data(dtype, need + 3, seed)
    got = run_copy(x, dims, strides, offset, out_offset)
    ref = oracle.tensor_copy(x, dims, strides, offset)
    assert got.dtype == ref.dtype and np.array_equal(got.view(np.uint8), ref.view(np.uint8)), b.last_variant()
    if expect is not None:
        assert expect in b.last_variant(), b.last_variant()


DTYPES = [np.float32, np.int8]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("perm", [(0, 2, 3, 1), (0, 3, 1, 2), (3, 2, 1, 0), (1, 0, 3, 2), (2, 0, 1, 3), (0, 1, 3, 2)])
@pytest.mark.parametrize("shape", [(2, 3, 70, 65), (3, 130, 5, 64), (1, 64, 64, 64), (2, 9, 8, 7)])
def test_permutations(dtype, shape, perm):
    print("case: copy perm", dtype.__name__, shape, perm, flush=True)
    strides = [shape[1] * shape[2] * shape[3], shape[2] * shape[3], shape[3], 1]
    dims = [shape[p] for p in perm]
    check(dtype, dims, [strides[p] for p in perm])


@pytest.mark.parametrize("dtype", DTYPES)
def test_nchw_nhwc_and_matrix_transpose_take_the_tiled_kernel(dtype):
    # NCHW (2, 24, 20, 36) -> NHWC: out (n, h, w, c), input strides (C*H*W, W, 1, H*W)
    check(dtype, (2, 20, 36, 24), (24 * 20 * 36, 36, 1, 20 * 36), expect="transpose")
    # NHWC -> NCHW
    check(dtype, (2, 24, 20, 36), (20 * 36 * 24, 1, 36 * 24, 24), expect="transpose")
    # 200 x 333 matrix transpose, row stride 340
    check(dtype, (1, 1, 333, 200), (0, 0, 1, 340), expect="transpose")


@pytest.mark.parametrize("dtype,vec", [(np.float32, 4), (np.int8, 16)])
def test_row_copies_vector_and_element(dtype, vec):
    check(dtype, (3, 4, 5, 8 * vec), (4 * 6 * 9 * vec * 8, 6 * 9 * vec * 8, 9 * vec * 8, 1), expect="rows_vec")   # padded rows
    check(dtype, (3, 4, 5, 8 * vec), (4 * 6 * 9 * vec * 8, 6 * 9 * vec * 8, 9 * vec * 8, 1), offset=vec, out_offset=vec,
          expect="rows_vec")
    check(dtype, (3, 4, 5, 8 * vec), (4 * 6 * 9 * vec * 8, 6 * 9 * vec * 8, 9 * vec * 8, 1), offset=1, expect="gather")
    check(dtype, (3, 4, 5, 8 * vec + 1), (4 * 6 * 400, 6 * 400, 400, 1), expect="gather")
    check(dtype, (2, 2, 3, 4 * vec), (0, 6 * 4 * vec + 1, 4 * vec, 1), expect="gather")   # a stride that breaks alignment


@pytest.mark.parametrize("dtype", DTYPES)
def test_broadcast_slices_and_degenerate_extents(dtype):
    check(dtype, (4, 3, 50, 33), (0, 0, 1, 0))                            # O[.., r, c] = I[r]
    check(dtype, (4, 3, 50, 33), (0, 0, 2, 0), expect="gather")          # no unit stride at all
    check(dtype, (2, 3, 1, 64), (0, 0, 0, 1))                            # one row repeated
    check(dtype, (2, 5, 6, 7), (1000, 2 * 70, 10, 3), offset=11)         # strided slice in every index
    check(dtype, (1, 1, 1, 1), (5, 5, 5, 5))
    check(dtype, (1, 1, 100, 1), (0, 0, 3, 0))
    check(dtype, (7, 1, 1, 1), (2, 0, 0, 0))
    check(dtype, (1, 1, 5, 100), (0, 0, 1, 5))                            # transpose too thin for tiles: gather


@pytest.mark.parametrize("offset,out_offset", [(0, 0), (1, 0), (0, 2), (3, 1), (4, 4)])
@pytest.mark.parametrize("dims,strides", [((1, 1, 300, 260), (0, 0, 1, 304)), ((1, 1, 131, 129), (0, 0, 1, 131)),
                                          ((2, 3, 140, 136), (3 * 140 * 136, 136, 1, 3 * 136 * 140 // 3)),
                                          ((3, 130, 2, 132), (130, 1, 3 * 130 * 132, 3 * 130))])
def test_byte_transpose_alignment_cases(dims, strides, offset, out_offset):
    """The byte kernel's dword and byte paths on both sides: bases off by 1..3, extents and
    strides that are not multiples of four, partial tiles."""
    print("case: copy bytes", dims, strides, offset, out_offset, flush=True)
    check(np.int8, dims, strides, offset=offset, out_offset=out_offset, expect="transpose")


@pytest.mark.parametrize("dtype,vec", [(np.float32, 4), (np.int8, 16)])
def test_transposes_with_16_byte_accesses(dtype, vec):
    """Extents, strides and bases that are multiples of 16 bytes take the wide kernels: several
    tiles and ragged last tiles in both directions, each position of the unit-stride index,
    padded rows, a base 16 bytes in; one extent or stride off by one element falls back."""
    name = "vec%d" % vec
    # matrix transposes: out (rows, cols) = in^T, input row stride padded
    check(dtype, (1, 1, 21 * vec, 37 * vec), (0, 0, 1, 23 * vec), expect=name)
    check(dtype, (1, 1, 21 * vec, 37 * vec), (0, 0, 1, 23 * vec), offset=vec, out_offset=vec, expect=name)
    # NCHW -> NHWC and back, unit stride in positions 2 and 1
    C, H, W = 9 * vec, 5, 3 * vec
    check(dtype, (2, H, W, C), (C * H * W, W, 1, H * W), expect=name)
    check(dtype, (2, C, H, W), (H * W * C, 1, W * C, C), expect=name)
    # unit stride in position 0
    check(dtype, (5 * vec, 3, 2, 7 * vec), (1, 5 * vec, 15 * vec, 30 * vec), expect=name)
    # one element off in an extent, a stride or a base: the narrower kernel, same values
    check(dtype, (1, 1, 21 * vec + 1, 37 * vec), (0, 0, 1, 23 * vec), expect="transpose")
    assert name not in b.last_variant()
    check(dtype, (1, 1, 21 * vec, 37 * vec), (0, 0, 1, 23 * vec + 1), expect="transpose")
    assert name not in b.last_variant()
    check(dtype, (1, 1, 21 * vec, 37 * vec), (0, 0, 1, 23 * vec), offset=1, expect="transpose")
    assert name not in b.last_variant()
    check(dtype, (2, H, W, C), (C * H * W + 1, W, 1, H * W), expect="transpose")
    assert name not in b.last_variant()


@pytest.mark.parametrize("dtype", DTYPES)
def test_large_transpose(dtype):
    # the shapes the benchmark times: NCHW -> NHWC of 8 x 64 x 56 x 56 and a 1024 x 768 transpose
    check(dtype, (8, 56, 56, 64), (64 * 56 * 56, 56, 1, 56 * 56), expect="transpose")
    check(dtype, (1, 1, 768, 1024), (0, 0, 1, 768), expect="transpose")


def test_torch_view_helper():
    x = torch.arange(2 * 3 * 4 * 5, dtype=torch.float32, device="cuda").reshape(2, 3, 4, 5)
    b.use_torch_stream()
    out = torch.empty(2, 5, 3, 4, device="cuda")
    b.tensor_copy_t(x.permute(0, 3, 1, 2), out)
    torch.cuda.synchronize()
    assert torch.equal(out, x.permute(0, 3, 1, 2).contiguous())
    m = torch.arange(12, dtype=torch.int8, device="cuda").reshape(3, 4)
    out8 = torch.empty(4, 3, dtype=torch.int8, device="cuda")
    b.tensor_copy_t(m.t(), out8)
    torch.cuda.synchronize()
    assert torch.equal(out8, m.t().contiguous())
    b.set_stream(None)


def test_packed_b_feeds_the_int8_product():
    """The use the paper names for this operation: reorganise an operand's memory for the
    kernel that follows.  B^T (N x K, k-contiguous) is unpacked to K x N and multiplied."""
    rng = np.random.default_rng(5)
    A = rng.integers(-128, 128, size=(128, 256), dtype=np.int8)
    Bt = rng.integers(-128, 128, size=(128, 256), dtype=np.int8)   # N x K
    dBt, dA = dev(Bt), dev(A)
    dB = torch.empty(256, 128, dtype=torch.int8, device="cuda")
    dC = torch.zeros(128, 128, dtype=torch.int32, device="cuda")
    b.set_stream(None)
    assert b.tensor_copy_s8(1, 1, 256, 128, 0, 0, 1, 256, dBt.data_ptr(), dB.data_ptr()) == b.OK
    assert b.igemm_s8s32(128, 128, 256, dA.data_ptr(), 256, dB.data_ptr(), 128, dC.data_ptr(), 128) == b.OK
    torch.cuda.synchronize()
    ref = oracle.igemm_s8s32(A, np.ascontiguousarray(Bt.T), np.zeros((128, 128), np.int32))
    assert np.array_equal(dC.cpu().numpy(), ref)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("channels", [1, 2, 3, 4, 7, 16])
@pytest.mark.parametrize("n,h,w", [(2, 20, 23), (1, 16, 16), (3, 1, 700), (2, 8, 8)])
def test_layout_changes_with_a_short_channel_extent(dtype, channels, n, h, w):
    """NCHW <-> NHWC with 1 to 16 channels (a batch of RGB images): the transpose whose tile is
    256 positions by the whole short extent; one channel is a plain copy, planes of fewer than
    64 positions go element by element."""
    print("case: copy narrow", dtype.__name__, channels, n, h, w, flush=True)
    c = channels
    narrow = "narrow" if c > 1 and h * w >= 64 else None
    # NCHW input, NHWC output
    check(dtype, (n, h, w, c), (c * h * w, w, 1, h * w), expect=narrow, seed=3)
    # NHWC input, NCHW output
    check(dtype, (n, c, h, w), (h * w * c, 1, w * c, c), expect=narrow, seed=4)
    # the same from a padded input (pixels of c + 2 elements) and an offset
    check(dtype, (n, c, h, w), (h * w * (c + 2), 1, w * (c + 2), c + 2), offset=3, out_offset=1, expect=narrow, seed=5)
    # the short index first in the output, the long one with a pitch: (c, n, 1, hw) from (n, hw, c)
    check(dtype, (c, n, 1, h * w), (1, h * w * c, 0, c), expect=narrow, seed=6)


def test_rgb_image_batches_take_16_byte_accesses():
    n, c, h, w = 4, 3, 56, 60
    check(np.float32, (n, h, w, c), (c * h * w, w, 1, h * w), expect="narrow_1024_vec4", seed=7)
    check(np.float32, (n, c, h, w), (h * w * c, 1, w * c, c), expect="narrow_1024_vec4", seed=8)
    check(np.float32, (n, h, w, 4), (4 * h * w, w, 1, h * w), expect="narrow_1024_vec4", seed=9)
    # a plane that is not a multiple of four positions, or a base off 16 bytes: element accesses
    check(np.float32, (n, 57, 59, c), (c * 57 * 59, 59, 1, 57 * 59), expect="narrow_256", seed=10)
    check(np.float32, (n, c, h, w), (h * w * c, 1, w * c, c), offset=1, expect="narrow_256", seed=11)
