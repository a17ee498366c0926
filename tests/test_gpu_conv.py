"""GPU parity of conv2d_nhwc against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, assert_close, dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_conv(x, w, stride, pad):
    N, P, Q, K = oracle.conv_out_shape(x.shape, w.shape, stride, pad)
    dx, dw = dev(x), dev(w)
    guard = 64
    buf = torch.full((N * P * Q * K + 2 * guard,), float("nan"), device="cuda")
    buf[:guard] = 777.0
    buf[-guard:] = 777.0
    out_ptr = buf.data_ptr() + 4 * guard
    H, W, C = x.shape[1:]
    R, S = w.shape[1:3]
    b.set_stream(None)
    st = b.conv2d_nhwc(N, H, W, C, K, R, S, stride, pad, dx.data_ptr(), dw.data_ptr(), out_ptr)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert np.all(host[:guard] == 777.0) and np.all(host[-guard:] == 777.0), "wrote outside out"
    return host[guard:-guard].reshape(N, P, Q, K)


def check(shape: wl.ConvShape, seed, exact=False):
    x, w = wl.conv_inputs(seed, shape, exact=exact)
    got = run_conv(x, w, shape.stride, shape.pad)
    ref, absum = oracle.conv2d_nhwc(x, w, shape.stride, shape.pad)
    assert not np.any(np.isnan(got)), "output elements left unwritten"
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
        return 0.0
    return assert_close(got, ref, absum + 1e-30, what=b.last_variant())


@pytest.fixture(autouse=True)
def _defaults():
    b.set_conv_tuning(-1)
    b.set_conv_split(0)
    b.set_conv_tail(-1)
    yield
    b.set_conv_tuning(-1)
    b.set_conv_split(0)
    b.set_conv_tail(-1)


@pytest.mark.parametrize("variant", range(len(b.conv_variant_names())))
@pytest.mark.parametrize("shape", [
    wl.ConvShape(2, 9, 11, 16, 64, 3, 3, 1, 1),    # chunk-in-tap path (C % 16 == 0)
    wl.ConvShape(2, 9, 11, 32, 70, 3, 3, 2, 1),    # same with stride 2 and a channel tail
    wl.ConvShape(1, 10, 7, 12, 40, 3, 2, 1, 1),    # flat path, 16-byte loads (C % 4 == 0)
    wl.ConvShape(1, 6, 7, 5, 9, 3, 3, 1, 1),       # flat path, element loads
])
def test_every_tile_configuration_exact(variant, shape):
    print("case: conv variant", variant, shape, flush=True)
    assert b.set_conv_tuning(variant) == b.OK
    check(shape, 11, exact=True)


@pytest.mark.parametrize("slices", [2, 3, 5, 1000])
@pytest.mark.parametrize("variant", [i for i, n in enumerate(b.conv_variant_names()) if "_dma_" in n])
@pytest.mark.parametrize("shape", [
    wl.ConvShape(2, 9, 11, 32, 64, 3, 3, 1, 1),    # 9 or 18 chunks, slices of unequal length
    wl.ConvShape(1, 7, 7, 64, 70, 3, 3, 1, 0),     # few pixels, channel tail
    wl.ConvShape(1, 6, 5, 96, 33, 2, 3, 2, 1),     # slice boundaries inside a tap (C = 3 chunks of 32)
])
def test_split_reduction_exact(shape, variant, slices):
    """The reduction cut into slices whose partial sums are added atomically: exact on
    small integers in any order; the first slices start in the middle of the (r, s, c) walk."""
    print("case: conv split", variant, shape, slices, flush=True)
    assert b.set_conv_tuning(variant) == b.OK
    assert b.set_conv_split(slices) == b.OK
    check(shape, 13, exact=True)
    assert b.last_variant().endswith("_splitk"), b.last_variant()


PIECE_VARIANTS = [i for i, n in enumerate(b.conv_variant_names())
                  if "_dma_" in n and "_w2x2_" in n]   # the four-wave direct-to-LDS kernels


@pytest.mark.parametrize("tail", [1, 2, 1000])
@pytest.mark.parametrize("variant", PIECE_VARIANTS)
@pytest.mark.parametrize("shape", [
    wl.ConvShape(3, 9, 11, 32, 64, 3, 3, 1, 1),    # 297 pixels: the last piece row is ragged
    wl.ConvShape(2, 9, 11, 32, 70, 3, 3, 2, 1),    # stride 2, channel tail in the last piece column
    wl.ConvShape(5, 8, 8, 16, 33, 1, 1, 1, 0),     # 1 x 1 filter: two groups of eight, waves without work
    wl.ConvShape(2, 12, 13, 48, 40, 2, 3, 1, 2),   # wide padding, a tap boundary inside a wave's share
    wl.ConvShape(2, 12, 13, 24, 40, 3, 3, 1, 1),   # 24 channels: the per-lane-tap kernels (the others hand over to them)
])
def test_quarter_tile_pieces_exact(shape, variant, tail):
    """The last tile rows computed as 32 x 32 pieces with the reduction split over the waves
    (tail = 1000: the whole output): exact on small integers."""
    print("case: conv pieces", variant, shape, tail, flush=True)
    assert b.set_conv_tuning(variant) == b.OK
    assert b.set_conv_split(1) == b.OK
    assert b.set_conv_tail(tail) == b.OK
    check(shape, 17, exact=True)
    assert b.last_variant().endswith("_pieces"), b.last_variant()


def test_quarter_tile_pieces_are_deterministic_and_within_tolerance():
    shape = wl.ConvShape(4, 20, 20, 64, 64, 3, 3, 1, 1)
    assert b.set_conv_tail(7) == b.OK
    x, w = wl.conv_inputs(18, shape)
    first = run_conv(x, w, shape.stride, shape.pad)
    assert b.last_variant().endswith("_pieces"), b.last_variant()
    ref, absum = oracle.conv2d_nhwc(x, w, shape.stride, shape.pad)
    assert assert_close(first, ref, absum + 1e-30, what=b.last_variant()) < TOL
    for _ in range(3):
        assert np.array_equal(run_conv(x, w, shape.stride, shape.pad), first)


def test_pieces_are_the_built_in_choice_for_a_sparse_last_round():
    # 270 tiles of 64 x 64 on 256 CUs: the 14 tiles of the second round become pieces
    shape = wl.ConvShape(5, 54, 64, 16, 64, 3, 3, 1, 1)
    assert shape.N * shape.P * shape.Q == 270 * 64
    assert check(shape, 19) < TOL
    assert b.last_variant().endswith("_pieces"), b.last_variant()
    assert b.set_conv_tail(0) == b.OK
    assert check(shape, 19) < TOL
    assert not b.last_variant().endswith("_pieces"), b.last_variant()


def test_table1_single_image_shapes_split_by_default():
    # CONV-2..4: few output tiles and a reduction of 36 to 144 chunks
    for i, shape in enumerate(wl.TABLE1_CONV[1:]):
        print("case: conv table-1 default split", shape, flush=True)
        assert check(shape, 30 + i) < TOL
        assert b.last_variant().endswith("_splitk"), b.last_variant()


def test_batched_small_images_split_by_the_fitted_cost():
    # 98 tiles and 72 chunks: slices shorten the fullest CU's work by more than they cost
    shape = wl.ConvShape(16, 14, 14, 128, 128, 3, 3, 1, 1)
    print("case: conv default split", shape, flush=True)
    assert check(shape, 41) < TOL
    assert b.last_variant().endswith("_splitk"), b.last_variant()
    # 196 tiles and 72 chunks: no slice count pays for the extra launches and atomics
    shape = wl.ConvShape(8, 28, 28, 128, 128, 3, 3, 1, 1)
    print("case: conv default whole", shape, flush=True)
    assert check(shape, 42) < TOL
    assert not b.last_variant().endswith("_splitk"), b.last_variant()


C4_VARIANTS = [i for i, n in enumerate(b.conv_variant_names()) if "_dma_c4_" in n]


@pytest.mark.parametrize("slices", [1, 3])
@pytest.mark.parametrize("variant", C4_VARIANTS)
@pytest.mark.parametrize("shape", [
    wl.ConvShape(2, 9, 11, 4, 64, 3, 3, 1, 1),     # four taps per chunk, reduction 36 ends inside a chunk
    wl.ConvShape(1, 23, 21, 4, 40, 7, 7, 2, 3),    # a padded stem: 49 taps, stride 2, wide padding
    wl.ConvShape(2, 10, 7, 12, 70, 3, 2, 1, 1),    # a chunk holds one tap and a third
    wl.ConvShape(3, 8, 9, 24, 33, 3, 3, 1, 1),     # groups of one chunk in two taps
    wl.ConvShape(2, 7, 6, 40, 64, 1, 1, 1, 0),     # 1 x 1 filter: the tap never changes, 2.5 chunks
    wl.ConvShape(1, 9, 9, 72, 130, 3, 3, 2, 0),    # 4.5 chunks per tap
    wl.ConvShape(2, 5, 5, 20, 64, 5, 4, 1, 2),     # padding wider than half the image
    wl.ConvShape(1, 1, 300, 8, 64, 1, 3, 1, 1),    # one image row
])
def test_kernels_for_channel_multiples_of_four_exact(shape, variant, slices):
    """The direct-to-LDS kernels whose lanes follow the tap of their own four channels:
    C % 4 == 0 only, whole reduction and cut into slices; exact on small integers."""
    print("case: conv c4", variant, shape, slices, flush=True)
    assert b.set_conv_tuning(variant) == b.OK
    assert b.set_conv_split(slices) == b.OK
    check(shape, 19, exact=True)
    name = b.conv_variant_names()[variant]
    assert b.last_variant() == (name if slices == 1 else name + "_splitk"), b.last_variant()


C1_VARIANTS = [i for i, n in enumerate(b.conv_variant_names()) if "_dma_c1_" in n]


@pytest.mark.parametrize("slices", [1, 3])
@pytest.mark.parametrize("variant", C1_VARIANTS)
@pytest.mark.parametrize("shape", [
    wl.ConvShape(2, 9, 11, 3, 64, 3, 3, 1, 1),     # five taps and a third per chunk, reduction 27
    wl.ConvShape(1, 23, 21, 3, 40, 7, 7, 2, 3),    # a stem: 49 taps of 3 channels, stride 2, wide padding
    wl.ConvShape(2, 10, 7, 1, 70, 3, 2, 1, 1),     # one channel: a filter row is two elements
    wl.ConvShape(3, 8, 9, 5, 33, 3, 3, 1, 1),      # odd channel count, output channels 33
    wl.ConvShape(2, 7, 6, 13, 64, 1, 1, 1, 0),     # 1 x 1 filter over 13 channels: less than a chunk
    wl.ConvShape(1, 9, 9, 18, 130, 3, 3, 2, 0),    # a tap is a chunk and an eighth
    wl.ConvShape(2, 5, 5, 6, 64, 5, 4, 1, 2),      # padding wider than half the image
    wl.ConvShape(1, 1, 300, 7, 64, 1, 3, 1, 1),    # one image row
    wl.ConvShape(2, 12, 12, 17, 65, 3, 3, 1, 1),   # 153 elements: nine chunks and nine elements
])
def test_kernels_for_any_channel_count_exact(shape, variant, slices):
    """The direct-to-LDS kernels whose lanes follow their own element of the reduction: any C,
    whole reduction and cut into slices; exact on small integers."""
    print("case: conv c1", variant, shape, slices, flush=True)
    assert b.set_conv_tuning(variant) == b.OK
    assert b.set_conv_split(slices) == b.OK
    check(shape, 29, exact=True)
    name = b.conv_variant_names()[variant]
    assert b.last_variant() == (name if slices == 1 or shape.R * shape.S * shape.C <= 16 else name + "_splitk"), b.last_variant()


def test_channel_multiples_of_four_take_the_direct_to_lds_kernels():
    """Built-in choice: 24 channels (not a multiple of 16) run on the per-lane-tap kernel,
    26 channels, 3 channels and a misaligned input on the per-lane-element one."""
    check(wl.ConvShape(4, 28, 28, 24, 64, 3, 3, 1, 1), 23)
    assert b.last_variant().startswith("conv2d_dma_c4_"), b.last_variant()
    check(wl.ConvShape(4, 28, 28, 26, 64, 3, 3, 1, 1), 24)
    assert b.last_variant().startswith("conv2d_dma_c1_"), b.last_variant()
    check(wl.ConvShape(2, 56, 56, 3, 64, 7, 7, 2, 3), 24)
    assert b.last_variant().startswith("conv2d_dma_c1_"), b.last_variant()
    s = wl.ConvShape(2, 14, 14, 24, 64, 3, 3, 1, 1)
    x, w = wl.conv_inputs(25, s, exact=True)
    flat = torch.empty(x.size + 1, device="cuda")
    flat[1:] = torch.from_numpy(x.ravel()).cuda()        # input 4 bytes off a 16-byte boundary
    dw, dout = dev(w), torch.empty(s.N, s.P, s.Q, s.K, device="cuda")
    st = b.conv2d_nhwc(s.N, s.H, s.W, s.C, s.K, s.R, s.S, s.stride, s.pad, flat.data_ptr() + 4, dw.data_ptr(), dout.data_ptr())
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    assert b.last_variant().startswith("conv2d_dma_c1_"), b.last_variant()
    ref, _ = oracle.conv2d_nhwc(x, w, s.stride, s.pad)
    assert np.array_equal(dout.cpu().numpy().astype(np.float64), ref)


def test_output_channels_that_leave_a_wide_tile_column_mostly_empty_take_32_wide_tiles():
    """Built-in choice: 96 and 20 output channels run on the 64 x 32 direct-to-LDS tile (also
    in its per-lane-tap form), 128 and 224 on the 64-wide ones."""
    for shape, expect in ((wl.ConvShape(4, 28, 28, 32, 96, 3, 3, 1, 1), "conv2d_dma_64x32x16"),
                          (wl.ConvShape(4, 28, 28, 24, 20, 3, 3, 1, 1), "conv2d_dma_c4_64x32x16"),
                          (wl.ConvShape(4, 28, 28, 32, 128, 3, 3, 1, 1), "conv2d_dma_64x64x16"),
                          (wl.ConvShape(4, 28, 28, 32, 224, 3, 3, 1, 1), "conv2d_dma_64x64x16")):
        check(shape, 27, exact=True)
        assert b.last_variant().startswith(expect), (shape, b.last_variant())


def test_hand_sum_on_gpu():
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 3, 3, 1)
    w = np.array([1, 2, 3, 4], np.float32).reshape(1, 2, 2, 1)
    got = run_conv(x, w, 1, 1)
    expect = np.array([[4, 11, 18, 9], [18, 37, 47, 21], [36, 67, 77, 33], [14, 23, 26, 9]], np.float32)
    assert np.array_equal(got[0, :, :, 0], expect)
    got = run_conv(x, w, 2, 1)
    assert np.array_equal(got[0, :, :, 0], np.array([[4, 18], [36, 77]], np.float32))


@pytest.mark.parametrize("shape", [
    wl.ConvShape(2, 9, 11, 16, 64, 3, 3, 1, 1),    # vector path, wide kernel
    wl.ConvShape(1, 8, 8, 4, 8, 3, 3, 1, 1),       # small kernel
    wl.ConvShape(2, 7, 9, 3, 5, 3, 3, 1, 1),       # C and K not multiples of 4: element-wise path
    wl.ConvShape(1, 12, 10, 8, 70, 5, 3, 2, 2),    # stride 2, rectangular filter, K tail
    wl.ConvShape(3, 6, 6, 20, 33, 1, 1, 1, 0),     # 1x1
    wl.ConvShape(1, 5, 5, 8, 16, 5, 5, 1, 0),      # filter as large as the image: one output pixel
    wl.ConvShape(1, 10, 10, 6, 12, 2, 4, 3, 1),    # stride 3, even filter
    wl.ConvShape(1, 3, 3, 4, 4, 3, 3, 1, 3),       # padding wider than the filter reach
    wl.ConvShape(1, 0, 4, 4, 4, 3, 3, 1, 2),       # empty image, output is all padding
])
def test_exact_integer_inputs(shape):
    print("case: conv exact", shape, flush=True)
    check(shape, 7, exact=True)


def test_center_delta_filter_copies_input():
    rng = np.random.default_rng(3)
    x = wl.uniform_f32(rng, (2, 13, 9, 16))
    w = np.zeros((16, 3, 3, 16), np.float32)
    for k in range(16):
        w[k, 1, 1, k] = 1.0
    assert np.array_equal(run_conv(x, w, 1, 1), x)


@pytest.mark.parametrize("i", range(4))
def test_table1_conv_shapes(i):
    shape = wl.TABLE1_CONV[i]
    print("case: conv table-1", shape, flush=True)
    assert check(shape, 20 + i) < TOL


def test_config_conv_56():
    seed, shape = wl.CONV_56
    print("case: conv config", shape, "seed", seed, flush=True)
    ratio = check(shape, seed)
    print("   variant", b.last_variant(), "max err/absum", ratio, flush=True)
    assert ratio < TOL


def test_batch_zero_is_a_no_op():
    assert b.conv2d_nhwc(0, 8, 8, 4, 4, 3, 3, 1, 1, 0, 0, 0) == b.OK
