"""The entry points under HIP graph capture: a call allocates nothing, waits for nothing and
clears nothing with a memset, so a sequence of calls can be recorded once and replayed.  Each
graph is replayed several times with eager work and synchronisations between the replays, and
every replay is checked against the oracle (small integers: bit-exact in any summation order)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _default_stream():
    yield
    b.set_stream(None)


def capture(record):
    """Runs `record` once eagerly on a side stream (lazy set-up happens outside the capture),
    then records it into a graph on that stream."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        b.use_torch_stream()
        record()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        b.use_torch_stream()
        record()
    b.set_stream(None)
    return graph


def replay_and_check(graph, reset, check, replays=3):
    scratch = torch.zeros(1 << 20, device="cuda")
    for r in range(replays):
        reset()
        graph.replay()
        torch.cuda.synchronize()
        check(r)
        scratch.add_(1.0)          # eager work between the replays
        torch.cuda.synchronize()


def test_small_sgemm_calls_replay():
    """Eight dependent 64^3 products, the launch-bound regime a graph is for."""
    shape = wl.GemmShape(64, 64, 64)
    A, B, C = wl.sgemm_inputs(101, shape, exact=True)
    dA, dB, dC = dev(A), dev(B), dev(C)
    ref, _ = oracle.sgemm(A, B, C)

    graph = capture(lambda: [b.sgemm_t(dA, dB, dC) for _ in range(8)])
    replay_and_check(graph, lambda: dC.zero_(),
                     lambda r: np.testing.assert_array_equal(dC.cpu().numpy().astype(np.float64), 8 * ref))


def test_split_reduction_paths_replay():
    """A split-K sgemm (atomics into C), a conv2d whose reduction is split (initial-value
    kernel, atomics, no memset) and an igemm in one graph."""
    gs = wl.GemmShape(256, 256, 2048)
    A, B, C = wl.sgemm_inputs(102, gs, exact=True)
    A, B = np.sign(A), np.sign(B)                       # entries in {-1, 0, 1}: sums stay exact
    dA, dB, dC = dev(A), dev(B), dev(C)
    ref_g, _ = oracle.sgemm(A, B, C)
    cs = wl.ConvShape(1, 14, 14, 256, 64, 3, 3, 1, 0)
    x, w = wl.conv_inputs(103, cs, exact=True)
    dx, dw = dev(x), dev(w)
    dout = torch.empty(cs.N, cs.P, cs.Q, cs.K, device="cuda")
    ref_c, _ = oracle.conv2d_nhwc(x, w, cs.stride, cs.pad)
    isz = wl.GemmShape(128, 256, 512)
    iA, iB, iC = wl.igemm_inputs(104, isz)
    diA, diB, diC = dev(iA), dev(iB), dev(iC)
    ref_i = oracle.igemm_s8s32(iA, iB, iC)
    seen = {}

    def record():
        b.sgemm_t(dA, dB, dC)
        seen["sgemm"] = b.last_variant()
        b.conv2d_nhwc_t(dx, dw, dout, cs.stride, cs.pad)
        seen["conv"] = b.last_variant()
        b.igemm_s8s32_t(diA, diB, diC)

    graph = capture(record)
    assert seen["conv"].endswith("_splitk"), seen

    def reset():
        dC.zero_()
        dout.fill_(-7.0)
        diC.zero_()

    def check(r):
        np.testing.assert_array_equal(dC.cpu().numpy().astype(np.float64), ref_g)
        np.testing.assert_array_equal(dout.cpu().numpy().astype(np.float64), ref_c)
        np.testing.assert_array_equal(diC.cpu().numpy(), ref_i)

    replay_and_check(graph, reset, check)


def test_fused_layer_at_a_small_batch_replays():
    """A fully connected layer with bias and ReLU at a small batch: pre(C), the cut product and
    post as three kernels; a few-row product on weights stored output-major; a matrix-vector
    product.  All in one graph."""
    fs = wl.GemmShape(64, 256, 2048)
    A, B, C = wl.sgemm_inputs(111, fs, exact=True, c_zero=False)
    A, B = np.sign(A), np.sign(B)
    bias = wl.small_int_f32(np.random.default_rng(112), (fs.N,), 50)
    dA, dB, dC, dbias = dev(A), dev(B), dev(C), dev(bias)
    ref_f, _ = oracle.sgemm_fused(A, B, C, bias, b.PRE_BIAS, b.POST_RELU)
    rs = wl.GemmShape(8, 1024, 1024)
    rA, rB, rC = wl.sgemm_inputs(113, rs, exact=True)
    rBt = np.ascontiguousarray(rB.T)
    drA, drBt, drC = dev(rA), dev(rBt), dev(rC)
    ref_r, _ = oracle.sgemm(rA, rB, rC)
    vs = wl.GemmShape(2048, 1, 1024)
    vA, vB, vC = wl.sgemm_inputs(114, vs, exact=True)
    dvA, dvB, dvC = dev(vA), dev(vB), dev(vC)
    ref_v, _ = oracle.sgemm(vA, vB, vC)
    seen = {}

    def record():
        b.sgemm_fused_t(dA, dB, dC, dbias, b.PRE_BIAS, b.POST_RELU)
        seen["fused"] = b.last_split()
        b.sgemm_op_t(False, True, drA, drBt, drC)
        seen["rows"] = b.last_variant()
        b.sgemm_t(dvA, dvB, dvC)
        seen["cols"] = b.last_variant()

    graph = capture(record)
    assert seen["fused"] > 1 and seen["rows"].startswith("sgemm_rows") and seen["cols"].startswith("sgemm_cols"), seen

    def reset():
        dC.copy_(torch.from_numpy(C))
        drC.zero_()
        dvC.zero_()

    def check(r):
        np.testing.assert_array_equal(dC.cpu().numpy().astype(np.float64), ref_f)
        np.testing.assert_array_equal(drC.cpu().numpy().astype(np.float64), ref_r)
        np.testing.assert_array_equal(dvC.cpu().numpy().astype(np.float64), ref_v)

    replay_and_check(graph, reset, check)


def test_depthwise_and_layout_calls_replay():
    """NCHW -> NHWC, then the LDS-staged depth-wise kernel with bias and ReLU on the result."""
    ds = wl.DwConvShape(64, 28, 28, 64, 3, 3, 1, 1)
    x, w, bias = wl.dwconv_inputs(105, ds, exact=True)
    x_nchw = np.ascontiguousarray(x.transpose(0, 3, 1, 2))
    dxc, dw, dbias = dev(x_nchw), dev(w), dev(bias)
    dx = torch.empty(ds.N, ds.H, ds.W, ds.C, device="cuda")
    dout = torch.empty(ds.N, ds.P, ds.Q, ds.C, device="cuda")
    ref, _ = oracle.dwconv2d_nhwc(x, w, ds.stride, ds.pad, bias=bias, post=oracle.POST_RELU)
    seen = {}

    def record():
        b.tensor_copy_t(dxc.permute(0, 2, 3, 1), dx)
        b.dwconv2d_nhwc_t(dx, dw, dout, ds.stride, ds.pad, bias=dbias, post=b.POST_RELU)
        seen["dwconv"] = b.last_variant()

    graph = capture(record)
    assert "_lds_" in seen["dwconv"], seen

    def reset():
        dx.fill_(-3.0)
        dout.fill_(-7.0)

    def check(r):
        np.testing.assert_array_equal(dx.cpu().numpy(), x)
        np.testing.assert_array_equal(dout.cpu().numpy().astype(np.float64), ref)

    replay_and_check(graph, reset, check)
