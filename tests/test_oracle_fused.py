"""Pins for the oracle's fused pre/post-operation forms: hand sums and reduction to the
already pinned plain oracles (post = max(., 0) of the plain result, pre = a change of C_in)."""
import numpy as np
import pytest

import oracle
from golden_io import read_cases
from paper_2205_00618_amd import workloads as wl


@pytest.mark.parametrize("name", ["bias_relu", "bias_only", "overwrite", "accumulate_relu"])
def test_sgemm_fused_hand_sums(name):
    c = read_cases("fused_hand.txt")[name]
    val, absum = oracle.sgemm_fused(c["A"].astype(np.float32), c["B"].astype(np.float32),
                                    c["Cin"].astype(np.float32), c["bias"].astype(np.float32).ravel(),
                                    c["pre"], c["post"])
    assert np.array_equal(val, c["expect"])
    assert np.all(absum >= np.abs(val))


def test_conv_fused_hand_sum():
    c = read_cases("fused_hand.txt")["conv_bias_relu"]
    val, _ = oracle.conv2d_nhwc(c["x"].astype(np.float32), c["w"].astype(np.float32), c["stride"], c["pad"],
                                bias=c["bias"].astype(np.float32).ravel(), post=c["post"])
    assert np.array_equal(val, c["expect"])


def test_sgemm_fused_reduces_to_plain_oracle():
    rng = np.random.default_rng(3)
    A, B, C = wl.uniform_f32(rng, (19, 37)), wl.uniform_f32(rng, (37, 23)), wl.uniform_f32(rng, (19, 23))
    bias = wl.uniform_f32(rng, (23,))
    plain, plain_abs = oracle.sgemm(A, B, C)
    v, a = oracle.sgemm_fused(A, B, C, None, oracle.PRE_ACCUMULATE, oracle.POST_NONE)
    assert np.array_equal(v, plain) and np.array_equal(a, plain_abs)
    v, _ = oracle.sgemm_fused(A, B, C, None, oracle.PRE_ACCUMULATE, oracle.POST_RELU)
    assert np.array_equal(v, np.maximum(plain, 0.0)) and (v == 0).any() and (v > 0).any()
    # pre = zero / bias is the plain product started from another C_in
    zero, zero_abs = oracle.sgemm(A, B, np.zeros_like(C))
    v, a = oracle.sgemm_fused(A, B, C, None, oracle.PRE_ZERO, oracle.POST_NONE)
    assert np.array_equal(v, zero) and np.array_equal(a, zero_abs)
    tiled = np.ascontiguousarray(np.broadcast_to(bias, C.shape))
    with_bias, bias_abs = oracle.sgemm(A, B, tiled)
    v, a = oracle.sgemm_fused(A, B, C, bias, oracle.PRE_BIAS, oracle.POST_NONE)
    assert np.array_equal(v, with_bias) and np.array_equal(a, bias_abs)
    v, _ = oracle.sgemm_fused(A, B, C, bias, oracle.PRE_BIAS, oracle.POST_RELU)
    assert np.array_equal(v, np.maximum(with_bias, 0.0))
    # bias runs along columns (j), not rows
    assert np.allclose(v[:, 0].min(), np.maximum(with_bias[:, 0], 0).min())


def test_conv_fused_reduces_to_plain_oracle():
    rng = np.random.default_rng(4)
    x, w = wl.uniform_f32(rng, (2, 6, 5, 3)), wl.uniform_f32(rng, (4, 3, 3, 3))
    bias = wl.uniform_f32(rng, (4,))
    plain, plain_abs = oracle.conv2d_nhwc(x, w, 1, 1)
    v, a = oracle.conv2d_nhwc(x, w, 1, 1, bias=bias)
    assert np.allclose(v, plain + bias.astype(np.float64), rtol=0, atol=1e-15)
    assert np.allclose(a, plain_abs + np.abs(bias).astype(np.float64), rtol=0, atol=1e-15)
    v, _ = oracle.conv2d_nhwc(x, w, 1, 1, bias=bias, post=oracle.POST_RELU)
    assert np.allclose(v, np.maximum(plain + bias.astype(np.float64), 0), rtol=0, atol=1e-15)
    v, _ = oracle.conv2d_nhwc(x, w, 1, 1, post=oracle.POST_RELU)
    assert np.array_equal(v, np.maximum(plain, 0.0))


def test_k_zero_applies_pre_and_post():
    C = np.array([[-1, 2], [3, -4]], np.float32)
    v, _ = oracle.sgemm_fused(np.zeros((2, 0), np.float32), np.zeros((0, 2), np.float32), C, None,
                              oracle.PRE_ACCUMULATE, oracle.POST_RELU)
    assert np.array_equal(v, np.array([[0, 2], [3, 0]], np.float64))
    v, _ = oracle.sgemm_fused(np.zeros((2, 0), np.float32), np.zeros((0, 2), np.float32), C,
                              np.array([5, -6], np.float32), oracle.PRE_BIAS, oracle.POST_NONE)
    assert np.array_equal(v, np.array([[5, -6], [5, -6]], np.float64))
