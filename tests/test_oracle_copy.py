"""Pins for the single-operand (strided copy) oracle: hand cases and numpy's own
transposition, broadcasting and slicing."""
import numpy as np
import pytest

import oracle
from golden_io import read_cases


@pytest.mark.parametrize("name", ["transpose_2x3", "broadcast_rows", "sub_block", "nchw_to_nhwc"])
@pytest.mark.parametrize("dtype", [np.float32, np.int8])
def test_copy_hand_cases(name, dtype):
    c = read_cases("copy_hand.txt")[name]
    got = oracle.tensor_copy(c["x"].astype(dtype), c["d"].astype(np.int64), c["s"].astype(np.int64),
                             c.get("offset", 0))
    assert got.dtype == dtype and np.array_equal(got, c["expect"].astype(dtype))


@pytest.mark.parametrize("perm", [(0, 1, 2, 3), (0, 2, 3, 1), (0, 3, 1, 2), (3, 2, 1, 0), (1, 0, 3, 2), (2, 0, 1, 3)])
def test_copy_equals_numpy_transpose(perm):
    rng = np.random.default_rng(21)
    x = rng.integers(-100, 100, size=(3, 4, 5, 6)).astype(np.float32)
    strides = np.array(x.strides) // 4
    want = np.ascontiguousarray(np.transpose(x, perm))
    got = oracle.tensor_copy(x, want.shape, strides[list(perm)])
    assert np.array_equal(got, want)


def test_copy_equals_numpy_broadcast_and_slice():
    rng = np.random.default_rng(22)
    v = rng.integers(-128, 128, size=(7,), dtype=np.int8)
    assert np.array_equal(oracle.tensor_copy(v, (2, 3, 7, 4), (0, 0, 1, 0)),
                          np.ascontiguousarray(np.broadcast_to(v[None, None, :, None], (2, 3, 7, 4))))
    x = rng.integers(-128, 128, size=(4, 5, 6, 7), dtype=np.int8)
    want = np.ascontiguousarray(x[1:3, ::2, 2:5, 1::3])
    strides = np.array(x.strides)
    got = oracle.tensor_copy(x, want.shape, strides * [1, 2, 1, 3], offset=int((strides * [1, 0, 2, 1]).sum()))
    assert np.array_equal(got, want)


def test_copy_empty_and_errors():
    x = np.zeros(4, np.float32)
    assert oracle.tensor_copy(x, (0, 1, 1, 1), (0, 0, 0, 1)).shape == (0, 1, 1, 1)
    with pytest.raises(ValueError):
        oracle.tensor_copy(x, (1, 1, 1, 5), (0, 0, 0, 1))      # reads past the end
    with pytest.raises(RuntimeError):
        oracle.tensor_copy(x, (1, 1, 1, 2), (0, 0, 0, -1))     # negative stride
    with pytest.raises(ValueError):
        oracle.tensor_copy(x.astype(np.float64), (1, 1, 1, 2), (0, 0, 0, 1))
