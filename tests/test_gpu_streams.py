"""Stream and thread behaviour of the C ABI: calls enqueue on the stream set for the calling
thread, state is per thread, and nothing synchronises behind the caller's back."""
import threading

import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, dev
from paper_2205_00618_amd import binding as b
from paper_2205_00618_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_calls_follow_a_non_default_stream():
    A, B, C = wl.sgemm_inputs(50, wl.GemmShape(300, 200, 150), c_zero=False)
    ref, absum = oracle.sgemm(A, B, C)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        b.use_torch_stream()
        dA, dB, dC = dev(A), dev(B), dev(C)          # uploads ordered on `stream`
        b.sgemm_t(dA, dB, dC)
        x, w, bias = wl.dwconv_inputs(51, wl.DwConvShape(2, 12, 12, 8, 3, 3, 1, 1))
        dx, dw, dbias = dev(x), dev(w), dev(bias)
        dout = torch.empty(2, 12, 12, 8, device="cuda")
        b.dwconv2d_nhwc_t(dx, dw, dout, 1, 1, dbias, b.POST_RELU)
    stream.synchronize()
    b.set_stream(None)
    assert_close(dC.cpu().numpy(), ref, absum, what="sgemm on a side stream")
    dref, dabs = oracle.dwconv2d_nhwc(x, w, 1, 1, bias, oracle.POST_RELU)
    assert_close(dout.cpu().numpy(), dref, dabs + 1e-30, what="dwconv on a side stream")


def test_dependent_calls_on_one_stream_run_in_order():
    # C2 = (A.B).B2 through two calls without a synchronisation in between
    rng = np.random.default_rng(52)
    A = wl.small_int_f32(rng, (128, 64), 3)
    B = wl.small_int_f32(rng, (64, 96), 3)
    B2 = wl.small_int_f32(rng, (96, 80), 3)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        b.use_torch_stream()
        dA, dB, dB2 = dev(A), dev(B), dev(B2)
        dC1 = torch.zeros(128, 96, device="cuda")
        dC2 = torch.zeros(128, 80, device="cuda")
        for _ in range(3):   # the second call of each pair reads what the first one wrote
            dC1.zero_()
            dC2.zero_()
            b.sgemm_t(dA, dB, dC1)
            b.sgemm_t(dC1, dB2, dC2)
    stream.synchronize()
    b.set_stream(None)
    want = (A.astype(np.float64) @ B.astype(np.float64)) @ B2.astype(np.float64)
    assert np.array_equal(dC2.cpu().numpy().astype(np.float64), want)


def test_tuning_and_stream_are_per_thread():
    A, B, C = wl.sgemm_inputs(53, wl.GemmShape(256, 256, 256), exact=True)
    ref, _ = oracle.sgemm(A, B, C)
    results = {}

    def worker(name, variant):
        torch.cuda.set_device(0)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            b.use_torch_stream()
            assert b.set_tuning(variant, 0) == b.OK
            dA, dB, dC = dev(A), dev(B), dev(C)
            for _ in range(20):
                dC.zero_()
                b.sgemm_t(dA, dB, dC)
            results[name] = (b.last_variant(), None)
        stream.synchronize()
        results[name] = (results[name][0], dC.cpu().numpy())

    names = b.variant_names()
    threads = [threading.Thread(target=worker, args=(f"t{i}", i)) for i in (0, 1, 2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for i in (0, 1, 2):
        variant, out = results[f"t{i}"]
        assert variant == names[i], (variant, names[i])     # each thread kept its own override
        assert np.array_equal(out.astype(np.float64), ref)
    assert b.last_variant() not in ("",)                     # this thread's state is untouched by the workers
    b.set_tuning(-1, 0)
    b.set_stream(None)
