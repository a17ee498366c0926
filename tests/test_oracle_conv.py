"""Pins for the convolution oracle: hand sums, structure (delta filter, tap counting,
shifts), reduction to the GEMM oracle, and a library correlation."""
import numpy as np
import pytest
from scipy.signal import correlate2d

import oracle
from golden_io import read_cases
from paper_2205_00618_amd import workloads as wl


@pytest.mark.parametrize("name", ["valid_2x2", "pad1_2x2", "pad1_stride2", "channels_1x1",
                                  "width_filter_batch2"])
def test_conv_hand_sums(name):
    c = read_cases("conv_hand.txt")[name]
    val, absum = oracle.conv2d_nhwc(c["x"].astype(np.float32), c["w"].astype(np.float32),
                                    c["stride"], c["pad"])
    assert val.shape == c["expect"].shape
    assert np.array_equal(val, c["expect"])
    assert np.all(absum >= np.abs(val))


def test_conv_center_delta_filter_is_identity():
    rng = np.random.default_rng(2)
    x = wl.uniform_f32(rng, (2, 6, 7, 5))
    w = np.zeros((5, 3, 3, 5), np.float32)
    for k in range(5):
        w[k, 1, 1, k] = 1.0
    val, _ = oracle.conv2d_nhwc(x, w, 1, 1)
    assert np.array_equal(val, x.astype(np.float64))


def test_conv_all_ones_counts_in_range_taps():
    C = 3
    x = np.ones((1, 5, 6, C), np.float32)
    w = np.ones((2, 3, 3, C), np.float32)
    val, absum = oracle.conv2d_nhwc(x, w, 1, 1)
    assert val.shape == (1, 5, 6, 2)
    rows = np.array([2, 3, 3, 3, 2])
    cols = np.array([2, 3, 3, 3, 3, 2])
    expect = (C * np.outer(rows, cols))[None, :, :, None] * np.ones((1, 1, 1, 2))
    assert np.array_equal(val, expect) and np.array_equal(absum, expect)
    assert val[0, 0, 0, 0] == 4 * C and val[0, 0, 2, 0] == 6 * C and val[0, 2, 2, 0] == 9 * C


def test_conv_shift_filters_pin_tap_direction():
    # a one-hot tap at (r,s) reads the input displaced by (r-pad, s-pad)
    rng = np.random.default_rng(4)
    x = wl.uniform_f32(rng, (1, 6, 6, 1))
    for r in range(3):
        for s in range(3):
            w = np.zeros((1, 3, 3, 1), np.float32)
            w[0, r, s, 0] = 1.0
            val, _ = oracle.conv2d_nhwc(x, w, 1, 1)
            expect = np.zeros((6, 6))
            for p in range(6):
                for q in range(6):
                    h, c = p + r - 1, q + s - 1
                    if 0 <= h < 6 and 0 <= c < 6:
                        expect[p, q] = x[0, h, c, 0]
            assert np.array_equal(val[0, :, :, 0], expect), (r, s)


def test_conv_1x1_equals_gemm_oracle_and_back():
    rng = np.random.default_rng(6)
    x = wl.uniform_f32(rng, (2, 4, 5, 7))
    w = wl.uniform_f32(rng, (3, 1, 1, 7))
    val, absum = oracle.conv2d_nhwc(x, w, 1, 0)
    A = x.reshape(-1, 7)
    B = np.ascontiguousarray(w.reshape(3, 7).T)
    g, ga = oracle.sgemm(A, B, np.zeros((A.shape[0], 3), np.float32))
    assert np.array_equal(val.reshape(-1, 3), g) and np.array_equal(absum.reshape(-1, 3), ga)
    # a GEMM is a convolution over 1x1 images
    A = wl.uniform_f32(rng, (9, 11))
    B = wl.uniform_f32(rng, (11, 4))
    g, _ = oracle.sgemm(A, B, np.zeros((9, 4), np.float32))
    c, _ = oracle.conv2d_nhwc(A.reshape(9, 1, 1, 11), np.ascontiguousarray(B.T).reshape(4, 1, 1, 11), 1, 0)
    assert np.array_equal(c.reshape(9, 4), g)


@pytest.mark.parametrize("stride,pad,R,S", [(1, 1, 3, 3), (1, 0, 3, 3), (2, 1, 3, 3), (1, 2, 5, 3),
                                            (2, 0, 2, 4), (3, 2, 3, 3)])
def test_conv_matches_scipy_correlation(stride, pad, R, S):
    rng = np.random.default_rng(8)
    N, H, W, C, K = 2, 9, 10, 3, 4
    x = wl.uniform_f32(rng, (N, H, W, C))
    w = wl.uniform_f32(rng, (K, R, S, C))
    val, _ = oracle.conv2d_nhwc(x, w, stride, pad)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    assert val.shape == (N, P, Q, K)
    xp = np.pad(x.astype(np.float64), ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    for n in range(N):
        for k in range(K):
            full = sum(correlate2d(xp[n, :, :, c], w[k, :, :, c].astype(np.float64), mode="valid")
                       for c in range(C))
            ref = full[::stride, ::stride][:P, :Q]
            assert np.max(np.abs(val[n, :, :, k] - ref)) < 1e-12


def test_conv_brute_force_python_loops():
    rng = np.random.default_rng(10)
    N, H, W, C, K, R, S, stride, pad = 1, 4, 5, 2, 2, 3, 2, 2, 1
    x = wl.small_int_f32(rng, (N, H, W, C), 3)
    w = wl.small_int_f32(rng, (K, R, S, C), 3)
    val, absum = oracle.conv2d_nhwc(x, w, stride, pad)
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    for p in range(P):
        for q in range(Q):
            for k in range(K):
                tot = mag = 0
                for r in range(R):
                    for s in range(S):
                        h, c0 = p * stride - pad + r, q * stride - pad + s
                        if 0 <= h < H and 0 <= c0 < W:
                            for c in range(C):
                                tot += int(x[0, h, c0, c]) * int(w[k, r, s, c])
                                mag += abs(int(x[0, h, c0, c]) * int(w[k, r, s, c]))
                assert val[0, p, q, k] == tot and absum[0, p, q, k] == mag


def test_conv_linearity_in_filter_and_batch_independence():
    rng = np.random.default_rng(12)
    x = wl.small_int_f32(rng, (3, 5, 5, 2), 4)
    w1 = wl.small_int_f32(rng, (2, 3, 3, 2), 4)
    w2 = wl.small_int_f32(rng, (2, 3, 3, 2), 4)
    f = lambda a, b: oracle.conv2d_nhwc(a, b, 1, 1)[0]
    assert np.array_equal(f(x, w1 + w2), f(x, w1) + f(x, w2))
    assert np.array_equal(f(x, w1)[1], f(x[1:2], w1)[0])
