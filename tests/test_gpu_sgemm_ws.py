"""GPU parity of sgemm_ws (partial sums of a cut reduction meet in a caller-provided workspace
and are added in a fixed order) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, assert_close, dev, run_sgemm
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu

COUNTER_BYTES = 65536
EDGE = [i for i, n in enumerate(b.variant_names()) if "_dma_edge" in n]


@pytest.fixture(autouse=True)
def _defaults():
    b.set_stream(None)
    b.set_tuning(-1, 0)
    yield
    b.set_tuning(-1, 0)


def workspace(nbytes, poison=True):
    """Zero counters, the partial-tile area poisoned with NaN (it may hold anything)."""
    ws = torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda")
    if poison:
        ws[COUNTER_BYTES // 4:] = float("nan")
    return ws


def counters_are_zero(ws):
    return bool(torch.all(ws[:COUNTER_BYTES // 4].view(torch.int32) == 0).item())


@pytest.mark.parametrize("variant", EDGE)
@pytest.mark.parametrize("split", [2, 3, 7])
@pytest.mark.parametrize("shape,ld", [((300, 292, 204), (204, 292, 292)), ((129, 67, 1000), (1000, 68, 71)),
                                      ((64, 64, 512), (512, 64, 64)), ((200, 131, 1000), (1004, 132, 131)),
                                      ((257, 255, 960), (960, 256, 255))])
def test_every_buffer_load_kernel_meets_in_the_workspace_exact(variant, split, shape, ld):
    print("case: ws variant", variant, "split", split, shape, ld, flush=True)
    assert b.set_tuning(variant, split) == b.OK
    A, B, C = wl.sgemm_inputs(61, wl.GemmShape(*shape), exact=True, c_zero=False)
    ws = workspace(COUNTER_BYTES + (8 << 20))
    got = run_sgemm(A, B, C, lda=ld[0], ldb=ld[1], ldc=ld[2], workspace=ws)
    ref, _ = oracle.sgemm(A, B, C)
    assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
    assert b.last_variant() == b.variant_names()[variant]
    assert b.last_split() > 1
    assert counters_are_zero(ws)
    # a second call on the same workspace, as left by the first
    got2 = run_sgemm(A, B, C, lda=ld[0], ldb=ld[1], ldc=ld[2], workspace=ws)
    assert np.array_equal(got2, got) and counters_are_zero(ws)


@pytest.mark.parametrize("shape", [(256, 256, 8192), (1000, 1000, 1000), (4097, 129, 511), (512, 512, 512),
                                   (100, 100, 5000), (1536, 1536, 1024), (64, 64, 64)])
def test_built_in_choice_is_right_and_reproducible(shape):
    print("case: ws built-in", shape, flush=True)
    A, B, C = wl.sgemm_inputs(62, wl.GemmShape(*shape), c_zero=False)
    # exactly what the library asks for (at least the counters, so that the call has a workspace)
    ws = workspace(max(b.sgemm_ws_bytes(*shape), COUNTER_BYTES + 256))
    got = run_sgemm(A, B, C, workspace=ws)
    ref, absum = oracle.sgemm(A, B, C)
    assert assert_close(got, ref, absum, what=b.last_variant()) < TOL
    print("   ", b.last_variant(), "split", b.last_split(), flush=True)
    for _ in range(3):
        again = run_sgemm(A, B, C, workspace=ws)
        assert np.array_equal(again, got), "two runs differ"
    assert counters_are_zero(ws)


def test_tail_of_an_incomplete_round_meets_in_the_workspace():
    # 2304 x 2304: 324 tiles of 128 x 128, 68 left over after one round of 256 compute units
    shape = (2304, 2304, 1024)
    A, B, C = wl.sgemm_inputs(63, wl.GemmShape(*shape), exact=True, c_zero=False)
    ws = workspace(b.sgemm_ws_bytes(*shape))
    got = run_sgemm(A, B, C, workspace=ws)
    ref, _ = oracle.sgemm(A, B, C)
    assert np.array_equal(got.astype(np.float64), ref), b.last_variant()
    print("   ", b.last_variant(), "split", b.last_split(), flush=True)
    assert counters_are_zero(ws)


@pytest.mark.parametrize("nbytes", [0, COUNTER_BYTES, COUNTER_BYTES + 64 * 64 * 4, COUNTER_BYTES + 40 * 64 * 64 * 4])
def test_a_small_workspace_limits_the_slices_not_the_result(nbytes):
    shape = (256, 256, 2048)   # 16 tiles of 64 x 64: wants many slices
    b.set_tuning(8, 0)
    A, B, C = wl.sgemm_inputs(64, wl.GemmShape(*shape), exact=True, c_zero=False)
    ws = workspace(max(nbytes, 256)) if nbytes else None
    if ws is None:
        dA, dB, dC = dev(A), dev(B), dev(C)
        assert b.sgemm_ws(256, 256, 2048, dA.data_ptr(), 2048, dB.data_ptr(), 256, dC.data_ptr(), 256, None, 0) == b.OK
        torch.cuda.synchronize()
        got = dC.cpu().numpy()
    else:
        got = run_sgemm(A, B, C, workspace=ws[:nbytes // 4])
    ref, _ = oracle.sgemm(A, B, C)
    assert np.array_equal(got.astype(np.float64), ref)
    assert b.last_split() * 16 * 64 * 64 * 4 <= max(nbytes - COUNTER_BYTES, 16 * 64 * 64 * 4)


def test_without_edge_kernels_nothing_is_cut():
    # a forced register-staged kernel cannot meet in the workspace: the reduction stays whole
    b.set_tuning(1, 4)
    A, B, C = wl.sgemm_inputs(65, wl.GemmShape(100, 90, 500), exact=True, c_zero=False)
    ws = workspace(COUNTER_BYTES + (8 << 20))
    got = run_sgemm(A, B, C, workspace=ws)
    assert np.array_equal(got.astype(np.float64), oracle.sgemm(A, B, C)[0])
    assert b.last_split() == 1


def test_validation():
    P = 4096
    assert b.sgemm_ws(4, 4, 4, P, 4, P, 4, P, 4, P + 8, 1 << 20) == b.ERR_DIM   # workspace not 256-byte aligned
    assert b.sgemm_ws(4, 4, 4, P, 4, P, 4, P, 4, P, -1) == b.ERR_DIM
    assert b.sgemm_ws(4, 4, 4, P, 3, P, 4, P, 4, P, 0) == b.ERR_LD
    assert b.sgemm_ws(0, 4, 4, 0, 4, 0, 4, 0, 4, 0, 0) == b.OK
    assert b.sgemm_ws_bytes(0, 4, 4) == 0 and b.sgemm_ws_bytes(256, 256, 8192) >= COUNTER_BYTES + 2 * 16 * 64 * 64 * 4
