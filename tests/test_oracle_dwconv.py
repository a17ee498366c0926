"""Pins for the depth-wise convolution oracle: hand sums, reduction to the (separately
pinned) full convolution oracle with a channel-diagonal filter, a library correlation per
channel, and structural checks (channel independence, delta filter, tap counting)."""
import numpy as np
import pytest
from scipy.signal import correlate2d

import oracle
from golden_io import read_cases
from paper_2205_00618_amd import workloads as wl


@pytest.mark.parametrize("name", ["two_channels_valid", "two_channels_pad1_stride2",
                                  "two_channels_bias_relu"])
def test_dwconv_hand_sums(name):
    c = read_cases("dwconv_hand.txt")[name]
    val, absum = oracle.dwconv2d_nhwc(c["x"].astype(np.float32), c["w"].astype(np.float32),
                                      c["stride"], c["pad"], c["bias"].astype(np.float32), c["post"])
    assert val.shape == c["expect"].shape
    assert np.array_equal(val, c["expect"])
    assert np.all(absum >= np.abs(val))


@pytest.mark.parametrize("shape,R,S,stride,pad", [((2, 7, 6, 5), 3, 3, 1, 1), ((1, 9, 8, 4), 3, 3, 2, 1),
                                                 ((1, 8, 8, 3), 5, 5, 1, 2), ((2, 6, 7, 2), 2, 3, 2, 0)])
def test_dwconv_equals_full_convolution_with_channel_diagonal_filter(shape, R, S, stride, pad):
    rng = np.random.default_rng(11)
    x = wl.small_int_f32(rng, shape, 4)
    C = shape[3]
    w = wl.small_int_f32(rng, (R, S, C), 4)
    full = np.zeros((C, R, S, C), np.float32)
    for c in range(C):
        full[c, :, :, c] = w[:, :, c]
    val, absum = oracle.dwconv2d_nhwc(x, w, stride, pad)
    ref, ref_abs = oracle.conv2d_nhwc(x, full, stride, pad)
    assert np.array_equal(val, ref)
    assert np.array_equal(absum, ref_abs)


def test_dwconv_matches_library_correlation_per_channel():
    rng = np.random.default_rng(12)
    x = wl.uniform_f32(rng, (2, 9, 11, 3))
    w = wl.uniform_f32(rng, (3, 5, 3))
    val, absum = oracle.dwconv2d_nhwc(x, w, 1, 0)
    for n in range(2):
        for c in range(3):
            ref = correlate2d(x[n, :, :, c].astype(np.float64), w[:, :, c].astype(np.float64), mode="valid")
            assert np.allclose(val[n, :, :, c], ref, rtol=0, atol=1e-12)
    assert np.all(np.abs(val) <= absum + 1e-15)


def test_dwconv_channels_do_not_mix():
    rng = np.random.default_rng(13)
    x = wl.uniform_f32(rng, (1, 6, 6, 4))
    w = wl.uniform_f32(rng, (3, 3, 4))
    base, _ = oracle.dwconv2d_nhwc(x, w, 1, 1)
    x2 = x.copy()
    x2[..., 2] += 1.0
    w2 = w.copy()
    w2[..., 1] *= 2.0
    moved_x, _ = oracle.dwconv2d_nhwc(x2, w, 1, 1)
    moved_w, _ = oracle.dwconv2d_nhwc(x, w2, 1, 1)
    for c in range(4):
        assert np.array_equal(moved_x[..., c], base[..., c]) == (c != 2)
        assert np.array_equal(moved_w[..., c], base[..., c]) == (c != 1)


def test_dwconv_center_delta_is_identity_and_ones_count_taps():
    rng = np.random.default_rng(14)
    x = wl.uniform_f32(rng, (2, 5, 6, 3))
    w = np.zeros((3, 3, 3), np.float32)
    w[1, 1, :] = 1.0
    val, _ = oracle.dwconv2d_nhwc(x, w, 1, 1)
    assert np.array_equal(val, x.astype(np.float64))
    ones, _ = oracle.dwconv2d_nhwc(np.ones((1, 5, 6, 2), np.float32), np.ones((3, 3, 2), np.float32), 1, 1)
    rows = np.array([2, 3, 3, 3, 2])
    cols = np.array([2, 3, 3, 3, 3, 2])
    assert np.array_equal(ones[0, :, :, 0], np.outer(rows, cols))
    assert np.array_equal(ones[0, :, :, 1], np.outer(rows, cols))


def test_dwconv_one_hot_tap_shifts_the_image():
    x = np.arange(2 * 5 * 5, dtype=np.float32).reshape(1, 5, 5, 2)
    w = np.zeros((3, 3, 2), np.float32)
    w[0, 2, 0] = 1.0   # channel 0 reads the pixel one up, one right
    w[2, 1, 1] = 1.0   # channel 1 reads the pixel one down
    val, _ = oracle.dwconv2d_nhwc(x, w, 1, 1)
    assert np.array_equal(val[0, 1:, :-1, 0], x[0, :-1, 1:, 0])
    assert np.all(val[0, 0, :, 0] == 0) and np.all(val[0, :, -1, 0] == 0)
    assert np.array_equal(val[0, :-1, :, 1], x[0, 1:, :, 1])
    assert np.all(val[0, -1, :, 1] == 0)


def test_dwconv_rejects_bad_arguments():
    x = np.zeros((1, 2, 2, 1), np.float32)
    with pytest.raises(RuntimeError):
        oracle.dwconv2d_nhwc(x, np.zeros((3, 3, 1), np.float32), 1, 0)   # filter larger than image
    with pytest.raises(ValueError):
        oracle.dwconv2d_nhwc(x, np.zeros((1, 1, 2), np.float32), 1, 0)   # channel mismatch
