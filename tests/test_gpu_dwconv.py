"""GPU parity of dwconv2d_nhwc / dwconv2d_nhwc_fused against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu

DIRECT_VEC4, DIRECT_SCALAR = 4, 5


def run_dwconv(x, w, stride, pad, bias=None, post=b.POST_NONE, offset=0, fused=True):
    """Runs the library on device copies placed `offset` floats into their buffers; the
    output buffer carries guard words on both sides and NaN where it must be written."""
    N, H, W, C = x.shape
    R, S = w.shape[:2]
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1

    def place(a):
        buf = np.full(a.size + offset, np.nan, np.float32)
        buf[offset:] = a.ravel()
        return dev(buf)

    dx, dw = place(x), place(w)
    db = place(bias) if bias is not None else None
    guard = 64
    buf = torch.full((N * P * Q * C + 2 * guard + offset,), float("nan"), device="cuda")
    buf[:guard + offset] = 777.0
    buf[-guard:] = 777.0
    out_ptr = buf.data_ptr() + 4 * (guard + offset)
    b.set_stream(None)
    if fused:
        st = b.dwconv2d_nhwc_fused(N, H, W, C, R, S, stride, pad, dx.data_ptr() + 4 * offset,
                                   dw.data_ptr() + 4 * offset, out_ptr,
                                   db.data_ptr() + 4 * offset if db is not None else None, post)
    else:
        st = b.dwconv2d_nhwc(N, H, W, C, R, S, stride, pad, dx.data_ptr() + 4 * offset,
                             dw.data_ptr() + 4 * offset, out_ptr)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert np.all(host[:guard + offset] == 777.0) and np.all(host[-guard:] == 777.0), "wrote outside out"
    return host[guard + offset:-guard].reshape(N, P, Q, C)


def check(shape: wl.DwConvShape, seed, exact, with_bias=False, post=b.POST_NONE, offset=0, expect=None):
    x, w, bias = wl.dwconv_inputs(seed, shape, exact=exact)
    bias = bias if with_bias else None
    got = run_dwconv(x, w, shape.stride, shape.pad, bias, post, offset,
                     fused=with_bias or post != b.POST_NONE or seed % 2 == 0)
    ref, absum = oracle.dwconv2d_nhwc(x, w, shape.stride, shape.pad, bias, post)
    assert not np.any(np.isnan(got)), "output elements left unwritten"
    if expect is not None:
        assert b.last_variant().startswith(expect), b.last_variant()
    if exact:
        assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
    else:
        assert_close(got, ref, absum + 1e-30, what=b.last_variant())


@pytest.fixture(autouse=True)
def _defaults():
    b.set_dwconv_tuning(-1, 0)
    b.set_dwconv_tile(0, 0, 0)
    yield
    b.set_dwconv_tuning(-1, 0)
    b.set_dwconv_tile(0, 0, 0)


def variant_index(name):
    return b.dwconv_variant_names().index(name)


FORMS = [(False, b.POST_NONE), (True, b.POST_NONE), (True, b.POST_RELU), (False, b.POST_RELU)]


@pytest.mark.parametrize("with_bias,post", FORMS)
@pytest.mark.parametrize("strip", [0, 1, 2, 3, 5, 7])
@pytest.mark.parametrize("shape,expect", [
    (wl.DwConvShape(2, 13, 11, 8, 3, 3, 1, 1), "dwconv_window_3x3_s1"),
    (wl.DwConvShape(2, 13, 11, 12, 3, 3, 1, 0), "dwconv_window_3x3_s1"),
    (wl.DwConvShape(2, 13, 12, 8, 3, 3, 2, 1), "dwconv_window_3x3_s2"),
    (wl.DwConvShape(1, 14, 9, 4, 3, 3, 2, 0), "dwconv_window_3x3_s2"),
    (wl.DwConvShape(2, 9, 10, 6, 5, 5, 1, 2), "dwconv_window_5x5_s1"),
    (wl.DwConvShape(1, 15, 13, 4, 5, 5, 2, 2), "dwconv_window_5x5_s2"),
    (wl.DwConvShape(1, 11, 12, 2, 5, 5, 2, 0), "dwconv_window_5x5_s2"),
])
def test_window_kernels_exact_for_every_strip_length(shape, expect, strip, with_bias, post):
    print("case: dwconv", shape, "strip", strip, with_bias, post, flush=True)
    assert b.set_dwconv_tuning(variant_index(expect + ("_v4" if "3x3" in expect else "_v2")), strip) == b.OK
    check(shape, 31, True, with_bias, post, expect=expect)


LDS_SHAPES = {
    "3x3_s1": [wl.DwConvShape(2, 13, 11, 8, 3, 3, 1, 1), wl.DwConvShape(1, 9, 30, 24, 3, 3, 1, 0),
               wl.DwConvShape(3, 5, 7, 4, 3, 3, 1, 2)],
    "3x3_s2": [wl.DwConvShape(2, 13, 12, 8, 3, 3, 2, 1), wl.DwConvShape(1, 14, 33, 20, 3, 3, 2, 0)],
    "5x5_s1": [wl.DwConvShape(2, 9, 10, 8, 5, 5, 1, 2), wl.DwConvShape(1, 12, 21, 16, 5, 5, 1, 0)],
    "5x5_s2": [wl.DwConvShape(1, 15, 13, 4, 5, 5, 2, 2), wl.DwConvShape(2, 11, 24, 12, 5, 5, 2, 1)],
    "7x7_s1": [wl.DwConvShape(2, 9, 10, 8, 7, 7, 1, 3), wl.DwConvShape(1, 12, 23, 16, 7, 7, 1, 0),
               wl.DwConvShape(1, 5, 6, 4, 7, 7, 1, 3)],
    "7x7_s2": [wl.DwConvShape(1, 15, 13, 4, 7, 7, 2, 3), wl.DwConvShape(2, 11, 26, 12, 7, 7, 2, 1)],
}


def lds_variants():
    return [n for n in ("dwconv_lds_3x3_s1_tp2", "dwconv_lds_3x3_s1_tp2_regs", "dwconv_lds_3x3_s1_tp4",
                        "dwconv_lds_3x3_s1_tp4_regs", "dwconv_lds_3x3_s2_tp1", "dwconv_lds_3x3_s2_tp1_regs",
                        "dwconv_lds_3x3_s2_tp2", "dwconv_lds_3x3_s2_tp2_regs", "dwconv_lds_5x5_s1_tp1",
                        "dwconv_lds_5x5_s1_tp1_regs", "dwconv_lds_5x5_s2_tp1", "dwconv_lds_5x5_s2_tp1_regs",
                        "dwconv_lds_5x5_s1_tp1_q2", "dwconv_lds_5x5_s1_tp1_q2_regs", "dwconv_lds_3x3_s1_tp2_q2", "dwconv_lds_3x3_s1_tp2_q2_regs", "dwconv_lds_3x3_s2_tp1_q2_regs",
                        "dwconv_lds_7x7_s1_tp1", "dwconv_lds_7x7_s1_tp1_q2", "dwconv_lds_7x7_s1_tp1_q4",
                        "dwconv_lds_7x7_s2_tp1", "dwconv_lds_7x7_s2_tp1_q2")]


@pytest.mark.parametrize("depth", [1, 2])
@pytest.mark.parametrize("band", [0, 1, 3, 4, 100])
@pytest.mark.parametrize("name", lds_variants())
def test_lds_staged_kernels_exact(name, band, depth):
    """Every LDS-staged kernel, bands of several lengths (one step, ragged last step, whole
    image), both prefetch depths, with bias and ReLU; small-integer data, so bit-exact."""
    key = name[len("dwconv_lds_"):len("dwconv_lds_") + 6]
    for shape in LDS_SHAPES[key]:
        print("case: dwconv lds", name, shape, "band", band, "depth", depth, flush=True)
        assert b.set_dwconv_tuning(variant_index(name), band) == b.OK
        assert b.set_dwconv_tile(0, 0, depth) == b.OK
        check(shape, 41, True, True, b.POST_RELU, expect=name)
        check(shape, 43, True, False, b.POST_NONE, expect=name)


@pytest.mark.parametrize("cols,channels", [(1, 0), (2, 4), (3, 8), (5, 0), (7, 12), (0, 4)])
@pytest.mark.parametrize("name", ["dwconv_lds_3x3_s1_tp2", "dwconv_lds_3x3_s2_tp2_regs", "dwconv_lds_5x5_s1_tp1_regs",
                                  "dwconv_lds_5x5_s2_tp1", "dwconv_lds_5x5_s1_tp1_q2", "dwconv_lds_5x5_s1_tp1_q2_regs", "dwconv_lds_3x3_s1_tp2_q2_regs"])
def test_lds_staged_tiles_in_columns_and_channels(name, cols, channels):
    """Column tiles with halo columns, channel tiles, ragged last tiles in both."""
    R = 3 if "3x3" in name else 5
    stride = 1 if "_s1_" in name else 2
    shape = wl.DwConvShape(2, 12, 15, 24, R, R, stride, R // 2)
    if cols:
        cols = min(cols, shape.Q)
    print("case: dwconv lds tiles", name, shape, cols, channels, flush=True)
    assert b.set_dwconv_tuning(variant_index(name), 0) == b.OK
    assert b.set_dwconv_tile(cols, channels, 0) == b.OK
    # a column count the planner cannot produce (not ceil(Q/k)) makes the call fall back; both are checked
    check(shape, 45, True, True, b.POST_RELU)
    check(shape, 46, False, True, b.POST_NONE)


def test_lds_staged_many_items_and_passes():
    """More than 256 (column, channel group) items per tile: several passes per step."""
    shape = wl.DwConvShape(2, 9, 40, 64, 3, 3, 1, 1)
    print("case: dwconv lds passes", shape, flush=True)
    assert b.set_dwconv_tuning(variant_index("dwconv_lds_3x3_s1_tp2"), 0) == b.OK
    check(shape, 47, True, True, b.POST_RELU, expect="dwconv_lds_3x3_s1_tp2")


@pytest.mark.parametrize("with_bias,post", FORMS)
@pytest.mark.parametrize("variant", [DIRECT_VEC4, DIRECT_SCALAR])
@pytest.mark.parametrize("shape", [
    wl.DwConvShape(2, 13, 11, 8, 3, 3, 1, 1),
    wl.DwConvShape(1, 9, 14, 12, 4, 2, 3, 2),     # even filter, stride 3, pad larger than needed
    wl.DwConvShape(2, 7, 7, 4, 7, 7, 1, 3),       # filter as large as the image
    wl.DwConvShape(1, 6, 8, 16, 1, 1, 2, 0),      # 1x1 filter, stride 2
])
def test_direct_kernels_exact(shape, variant, with_bias, post):
    print("case: dwconv direct", shape, variant, with_bias, post, flush=True)
    assert b.set_dwconv_tuning(variant, 0) == b.OK
    check(shape, 32, True, with_bias, post, expect="dwconv_direct")


@pytest.mark.parametrize("shape", [
    wl.DwConvShape(2, 9, 10, 5, 3, 3, 1, 1),      # C not a multiple of 2 or 4
    wl.DwConvShape(1, 9, 10, 3, 5, 5, 2, 2),
    wl.DwConvShape(3, 8, 8, 1, 3, 3, 2, 1),       # a single channel
    wl.DwConvShape(1, 8, 9, 7, 2, 3, 1, 0),
])
def test_odd_channel_counts_take_the_scalar_kernel(shape):
    print("case: dwconv odd C", shape, flush=True)
    check(shape, 33, True, True, b.POST_RELU, expect="dwconv_direct_scalar")
    check(shape, 34, False, expect="dwconv_direct_scalar")


@pytest.mark.parametrize("offset,expect", [(1, "dwconv_direct_scalar"), (2, "dwconv_direct_scalar"),
                                           (4, "dwconv_window_3x3_s1")])
def test_misaligned_tensors_fall_back(offset, expect):
    print("case: dwconv offset", offset, flush=True)
    check(wl.DwConvShape(2, 10, 9, 8, 3, 3, 1, 1), 35, True, True, b.POST_NONE, offset=offset, expect=expect)


def test_misaligned_by_eight_bytes_uses_two_channel_window_kernel():
    print("case: dwconv 5x5 offset 2", flush=True)
    check(wl.DwConvShape(1, 10, 9, 8, 5, 5, 1, 2), 36, True, True, b.POST_RELU, offset=2,
          expect="dwconv_window_5x5_s1_v2")


@pytest.mark.parametrize("index", range(4))
@pytest.mark.parametrize("batch", [1, 3])
def test_table1_shapes_random_data(index, batch):
    shape = wl.table1_dwconv(batch)[index]
    print("case: dwconv table 1", shape, flush=True)
    check(shape, wl.TABLE1_DWCONV_SEED, False, True, b.POST_RELU)
    check(shape, wl.TABLE1_DWCONV_SEED + 1, False)


def test_many_strips_and_blocks_exact():
    # several workgroups per XCD, strips that do not divide P, a ragged last block
    shape = wl.DwConvShape(5, 37, 29, 20, 3, 3, 1, 1)
    print("case: dwconv many blocks", shape, flush=True)
    for strip in (0, 4, 16, 37, 64):
        assert b.set_dwconv_tuning(-1, strip) == b.OK
        check(shape, 37, True, True, b.POST_NONE, expect="dwconv_window_3x3_s1")


def test_bench_shape_sampled_images():
    # the batched workload the benchmark times: first, middle and last image against the oracle
    shape = wl.table1_dwconv(64)[0]
    print("case: dwconv bench shape", shape, flush=True)
    x, w, bias = wl.dwconv_inputs(wl.TABLE1_DWCONV_SEED, shape)
    got = run_dwconv(x, w, shape.stride, shape.pad, bias, b.POST_RELU)
    for n in (0, shape.N // 2, shape.N - 1):
        ref, absum = oracle.dwconv2d_nhwc(x[n:n + 1], w, shape.stride, shape.pad, bias, b.POST_RELU)
        assert_close(got[n:n + 1], ref, absum + 1e-30, what=f"image {n}")


def test_empty_image_with_padding_writes_post_of_bias():
    # H = 0 with pad 1 and a 2x2 filter still has one output row: every tap is padding
    b.set_stream(None)
    bias = dev(np.array([-1.0, 2.0, 3.0, -4.0], np.float32))
    w = dev(np.ones((2, 2, 4), np.float32))
    out = torch.full((1, 1, 4, 4), float("nan"), device="cuda")
    st = b.dwconv2d_nhwc_fused(1, 0, 3, 4, 2, 2, 1, 1, None, w.data_ptr(), out.data_ptr(), bias.data_ptr(),
                               b.POST_RELU)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[0, 0], np.tile([0.0, 2.0, 3.0, 0.0], (4, 1)))
