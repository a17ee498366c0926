"""GPU parity of the fused pre/post-operation entry points against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, assert_close, dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu

FORMS = [(b.PRE_ACCUMULATE, b.POST_NONE), (b.PRE_ACCUMULATE, b.POST_RELU), (b.PRE_ZERO, b.POST_NONE),
         (b.PRE_ZERO, b.POST_RELU), (b.PRE_BIAS, b.POST_NONE), (b.PRE_BIAS, b.POST_RELU)]


@pytest.fixture(autouse=True)
def _defaults():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    b.set_conv_tuning(-1)
    b.set_conv_split(0)
    yield
    b.set_tuning(-1, 0)
    b.set_conv_tuning(-1)
    b.set_conv_split(0)


def run_fused(A, B, C, bias, pre, post):
    dA, dB, dC, dbias = dev(A), dev(B), dev(C), dev(bias)
    b.sgemm_fused_t(dA, dB, dC, dbias if pre == b.PRE_BIAS else None, pre, post)
    torch.cuda.synchronize()
    return dC.cpu().numpy()


def test_hand_sum_on_gpu():
    A = np.array([[1, 2], [3, 4]], np.float32)
    B = np.array([[5, 6], [7, 8]], np.float32)
    C = np.full((2, 2), 100, np.float32)
    got = run_fused(A, B, C, np.array([-20, -45], np.float32), b.PRE_BIAS, b.POST_RELU)
    assert np.array_equal(got, np.array([[0, 0], [23, 5]], np.float32))


@pytest.mark.parametrize("pre,post", FORMS)
@pytest.mark.parametrize("variant", range(len(b.variant_names())))
@pytest.mark.parametrize("shape", [(256, 256, 96), (200, 150, 75)])
def test_every_form_every_kernel_exact(variant, shape, pre, post):
    # small-integer data: bit-exact for any summation order; an aligned shape (all kernels)
    # and a ragged one (the aligned-only kernels hand over to the generic kernel)
    print("case: fused", shape, "variant", variant, "pre", pre, "post", post, flush=True)
    assert b.set_tuning(variant, 0) == b.OK
    A, B, C = wl.sgemm_inputs(5, wl.GemmShape(*shape), exact=True, c_zero=False)
    bias = wl.small_int_f32(np.random.default_rng(6), (shape[1],), 50)
    got = run_fused(A, B, C, bias, pre, post)
    ref, _ = oracle.sgemm_fused(A, B, C, bias, pre, post)
    assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
    if post == b.POST_RELU:
        assert (got == 0).any() and (got > 0).any()


@pytest.mark.parametrize("pre,post", FORMS)
def test_random_values_within_tolerance(pre, post):
    A, B, C = wl.sgemm_inputs(7, wl.GemmShape(512, 384, 320), c_zero=False)
    bias = wl.uniform_f32(np.random.default_rng(8), (384,))
    got = run_fused(A, B, C, bias, pre, post)
    ref, absum = oracle.sgemm_fused(A, B, C, bias, pre, post)
    assert assert_close(got, ref, absum, what=b.last_variant()) < TOL


def test_fused_form_over_several_launches_exact():
    """1536 tiles of 128 x 128 run as launches of 1024 and 512 tiles: the bias and the ReLU
    apply in every one of them."""
    shape = (6144, 4096, 64)
    A, B, C = wl.sgemm_inputs(7, wl.GemmShape(*shape), exact=True, c_zero=False)
    bias = wl.small_int_f32(np.random.default_rng(8), (shape[1],), 50)
    # (with so short a reduction the built-in choice is the buffer-load form of the tile, one launch)
    assert b.set_tuning(b.variant_names().index("sgemm_dma_128x128x16_w2x2_s2_c0"), 0) == b.OK
    got = run_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert b.last_variant() == "sgemm_dma_128x128x16_w2x2_s2_c0", b.last_variant()
    ref, _ = oracle.sgemm_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert np.array_equal(got.astype(np.float64), ref)
    assert (got == 0).any() and (got > 0).any()


@pytest.mark.parametrize("pre,post", FORMS[1:])
@pytest.mark.parametrize("shape,ld", [((256, 256, 2048), (0, 0, 0)), ((64, 1024, 4096), (0, 0, 0)),
                                      ((100, 130, 3001), (3, 2, 7)), ((32, 32, 16384), (0, 0, 0)),
                                      ((8, 2048, 2048), (0, 0, 0)),      # a few rows: the kernel that streams B
                                      ((64, 256, 1024), (0, 0, 0))])     # four tiles: the register-staged kernel
def test_few_tiles_and_a_long_reduction_run_as_pre_then_cut_product_then_post(shape, ld, pre, post):
    """A small output with a long reduction (a fully connected layer at a small batch): pre(C) is
    written out, the plain product adds its slices onto it, post runs in place.  Exact on small
    integers; padded rows keep their padding."""
    M, N, K = shape
    A, B, C = wl.sgemm_inputs(9, wl.GemmShape(*shape), exact=True, c_zero=False)
    bias = wl.small_int_f32(np.random.default_rng(10), (N,), 50)
    lda, ldb, ldc = K + ld[0], N + ld[1], N + ld[2]
    bufA = np.full((M, lda), 77, np.float32); bufA[:, :K] = A
    bufB = np.full((K, ldb), 77, np.float32); bufB[:, :N] = B
    bufC = np.full((M, ldc), 777, np.float32); bufC[:, :N] = C
    dA, dB, dC, dbias = dev(bufA), dev(bufB), dev(bufC), dev(bias)
    st = b.sgemm_fused(M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb, dC.data_ptr(), ldc,
                       dbias.data_ptr() if pre == b.PRE_BIAS else None, pre, post)
    assert st == b.OK, b.strerror(st)
    torch.cuda.synchronize()
    assert b.last_split() > 1, (b.last_variant(), b.last_split())
    out = dC.cpu().numpy()
    assert np.all(out[:, N:] == 777), "wrote into the padding of C"
    ref, _ = oracle.sgemm_fused(A, B, C, bias, pre, post)
    assert np.array_equal(out[:, :N].astype(np.float64), ref), b.last_variant()


def test_a_caller_who_keeps_reductions_whole_gets_one_kernel_when_fused():
    shape = wl.GemmShape(256, 256, 2048)
    A, B, C = wl.sgemm_inputs(9, shape, exact=True, c_zero=False)
    bias = wl.small_int_f32(np.random.default_rng(10), (256,), 50)
    assert b.set_tuning(-1, 1) == b.OK
    got = run_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert b.last_split() == 1
    ref, _ = oracle.sgemm_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert np.array_equal(got.astype(np.float64), ref)
    # random data, whole reductions: two calls give the same bits
    A, B, C = wl.sgemm_inputs(11, shape, c_zero=False)
    one = run_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    two = run_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert np.array_equal(one, two)


def test_fused_cut_within_tolerance_on_random_values():
    shape = wl.GemmShape(64, 1024, 4096)
    A, B, C = wl.sgemm_inputs(12, shape, c_zero=False)
    bias = wl.uniform_f32(np.random.default_rng(13), (1024,))
    got = run_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert b.last_split() > 1
    ref, absum = oracle.sgemm_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    assert assert_close(got, ref, absum, what=b.last_variant()) < TOL


def test_k_zero_applies_pre_and_post():
    C = np.array([[-1, 2, 7], [3, -4, -9]], np.float32)
    dC = dev(C)
    assert b.sgemm_fused(2, 3, 0, 0, 1, 0, 3, dC.data_ptr(), 3, None, b.PRE_ACCUMULATE, b.POST_RELU) == b.OK
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), np.maximum(C, 0))
    dbias = dev(np.array([5, -6, 7], np.float32))
    assert b.sgemm_fused(2, 3, 0, 0, 1, 0, 3, dC.data_ptr(), 3, dbias.data_ptr(), b.PRE_BIAS, b.POST_NONE) == b.OK
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy(), np.array([[5, -6, 7], [5, -6, 7]], np.float32))


def test_argument_errors():
    assert b.sgemm_fused(4, 4, 4, 16, 4, 16, 4, 16, 4, None, 3, 0) == b.ERR_OP
    assert b.sgemm_fused(4, 4, 4, 16, 4, 16, 4, 16, 4, None, 0, 2) == b.ERR_OP
    assert b.sgemm_fused(4, 4, 4, 16, 4, 16, 4, 16, 4, None, b.PRE_BIAS, 0) == b.ERR_NULL
    assert b.conv2d_nhwc_fused(1, 4, 4, 4, 4, 3, 3, 1, 1, 16, 16, 16, None, 7) == b.ERR_OP


@pytest.mark.parametrize("slices", [1, 4])
@pytest.mark.parametrize("variant", range(len(b.conv_variant_names())))
@pytest.mark.parametrize("with_bias,post", [(True, b.POST_RELU), (True, b.POST_NONE), (False, b.POST_RELU)])
def test_conv_fused_exact(variant, with_bias, post, slices):
    # slices = 4: the direct-to-LDS kernels (4..8) cut the reduction; bias then enters as the
    # output's initial value and ReLU runs after the last partial sum
    print("case: conv fused variant", variant, with_bias, post, slices, flush=True)
    assert b.set_conv_tuning(variant) == b.OK
    assert b.set_conv_split(slices) == b.OK
    shape = wl.ConvShape(2, 9, 11, 32, 70, 3, 3, 1, 1)
    x, w = wl.conv_inputs(12, shape, exact=True)
    bias = wl.small_int_f32(np.random.default_rng(13), (shape.K,), 60) if with_bias else None
    dx, dw = dev(x), dev(w)
    dbias = dev(bias) if with_bias else None
    dout = torch.full((shape.N, shape.P, shape.Q, shape.K), float("nan"), device="cuda")
    b.conv2d_nhwc_t(dx, dw, dout, shape.stride, shape.pad, dbias, post)
    torch.cuda.synchronize()
    ref, _ = oracle.conv2d_nhwc(x, w, shape.stride, shape.pad, bias=bias, post=post)
    got = dout.cpu().numpy()
    assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
    if post == b.POST_RELU:
        assert (got == 0).any() and (got > 0).any()


@pytest.mark.parametrize("with_bias,post", [(True, b.POST_RELU), (True, b.POST_NONE), (False, b.POST_RELU)])
def test_conv_fused_quarter_tile_pieces_exact(with_bias, post):
    print("case: conv fused pieces", with_bias, post, flush=True)
    assert b.set_conv_split(1) == b.OK
    assert b.set_conv_tail(2) == b.OK
    try:
        shape = wl.ConvShape(3, 9, 11, 32, 70, 3, 3, 1, 1)
        x, w = wl.conv_inputs(15, shape, exact=True)
        bias = wl.small_int_f32(np.random.default_rng(16), (shape.K,), 60) if with_bias else None
        dx, dw = dev(x), dev(w)
        dbias = dev(bias) if with_bias else None
        dout = torch.full((shape.N, shape.P, shape.Q, shape.K), float("nan"), device="cuda")
        b.conv2d_nhwc_t(dx, dw, dout, shape.stride, shape.pad, dbias, post)
        torch.cuda.synchronize()
        assert b.last_variant().endswith("_pieces"), b.last_variant()
        ref, _ = oracle.conv2d_nhwc(x, w, shape.stride, shape.pad, bias=bias, post=post)
        assert np.array_equal(dout.cpu().numpy().astype(np.float64), ref), b.last_variant()
    finally:
        b.set_conv_split(0)
        b.set_conv_tail(-1)


def test_conv_fused_workload_shape_within_tolerance():
    seed, shape = wl.CONV_56
    x, w = wl.conv_inputs(seed, shape)
    bias = wl.uniform_f32(np.random.default_rng(14), (shape.K,))
    dx, dw, dbias = dev(x), dev(w), dev(bias)
    dout = torch.empty((shape.N, shape.P, shape.Q, shape.K), device="cuda")
    b.conv2d_nhwc_t(dx, dw, dout, shape.stride, shape.pad, dbias, b.POST_RELU)
    torch.cuda.synchronize()
    ref, absum = oracle.conv2d_nhwc(x, w, shape.stride, shape.pad, bias=bias, post=b.POST_RELU)
    assert assert_close(dout.cpu().numpy(), ref, absum + 1e-30, what=b.last_variant()) < TOL


@pytest.mark.parametrize("pre,post", FORMS)
@pytest.mark.parametrize("kernel", ["sgemm_dma_128x128x16_w4x2_s2_c0", "sgemm_dma_256x128x16_w4x2_s2_c0"])
def test_fused_forms_on_the_eight_wave_tiles_exact(pre, post, kernel):
    """The kernels the library takes for 4096 x 4096 outputs (128 x 128 tiles on eight waves by
    itself at this K, 256 x 128 forced), under every epilogue form, every element against the oracle."""
    print("case: fused eight-wave tile", kernel, "pre", pre, "post", post, flush=True)
    shape = (4096, 4096, 272)
    A, B, C = wl.sgemm_inputs(9, wl.GemmShape(*shape), exact=True, c_zero=False)
    bias = wl.small_int_f32(np.random.default_rng(10), (shape[1],), 50)
    if kernel.startswith("sgemm_dma_256"):
        assert b.set_tuning(b.variant_names().index(kernel), 0) == b.OK
    got = run_fused(A, B, C, bias, pre, post)
    assert b.last_variant() == kernel, b.last_variant()
    ref, _ = oracle.sgemm_fused(A, B, C, bias, pre, post)
    assert np.array_equal(got.astype(np.float64), ref)
