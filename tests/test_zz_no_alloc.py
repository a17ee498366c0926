"""The entry point that allocates nothing, sgemm_static, against sgemm_ws with a caller's
workspace of the same size: same kernels, so the results must be bit-identical; and both
against the CPU oracle.  Two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, assert_close, dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu

STATIC_BYTES = 65536 + (8 << 20)


def both(shape, seed, exact):
    M, N, K = shape
    A, B, C = wl.sgemm_inputs(seed, wl.GemmShape(M, N, K), exact=exact, c_zero=False)
    dA, dB = dev(A), dev(B)
    ws = torch.zeros(STATIC_BYTES // 4, dtype=torch.float32, device="cuda")
    c_ws, c_st = dev(C), dev(C)
    assert b.sgemm_ws(M, N, K, dA.data_ptr(), K, dB.data_ptr(), N, c_ws.data_ptr(), N, ws.data_ptr(), STATIC_BYTES) == b.OK
    split_ws, name_ws = b.last_split(), b.last_variant()
    assert b.sgemm_static(M, N, K, dA.data_ptr(), K, dB.data_ptr(), N, c_st.data_ptr(), N) == b.OK
    assert (b.last_split(), b.last_variant()) == (split_ws, name_ws)
    torch.cuda.synchronize()
    got_ws, got_st = c_ws.cpu().numpy(), c_st.cpu().numpy()
    assert np.array_equal(got_ws, got_st), f"sgemm_static differs from sgemm_ws ({name_ws}, {split_ws} slices)"
    ref, absum = oracle.sgemm(A, B, C)
    if exact:
        assert np.array_equal(got_st.astype(np.float64), ref)
    else:
        assert assert_close(got_st, ref, absum, what=name_ws) < TOL
    return split_ws


def test_two_calls_in_a_row_the_second_smaller():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    print("case: sgemm_static 256x256x8192 then 130x70x2050", flush=True)
    assert both((256, 256, 8192), 71, exact=False) > 1     # cut: the partial sums meet in the library's array
    assert both((130, 70, 2050), 72, exact=True) > 1       # smaller, ragged, rows off 16 bytes
    # and once more the first shape: the array is as the second call left it
    assert both((256, 256, 8192), 73, exact=True) > 1


def test_uncut_and_refused_calls():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    assert both((1024, 1024, 1024), 74, exact=False) == 1   # nothing to meet: the array is not touched
    # forced: 300 tiles of 64 x 64 in 8 slices would need 37.5 MiB of partial tiles
    P = 4096
    b.set_tuning(15, 8)
    try:
        assert b.sgemm_static(1280, 960, 4096, P, 4096, P, 960, P, 960) == b.ERR_TOO_LARGE
    finally:
        b.set_tuning(-1, 0)
    assert b.sgemm_static(4, 4, 4, P, 3, P, 4, P, 4) == b.ERR_LD
    assert b.sgemm_static(0, 4, 4, 0, 4, 0, 4, 0, 4) == b.OK
