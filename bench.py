#!/usr/bin/env python3
"""Benchmark: fp32 SGEMM C += A.B at M=N=K=4096 on one MI355X, as TFLOP/s and as a
fraction of the fp32 matrix peak; the other workloads and the CPU oracle are timed beside it.

One "step" is one `sgemm` call on the seeded 4096^3 workload with A, B and C resident in
HBM.  Prints ONE JSON line on stdout (everything else goes to stderr).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_TFLOPS = 157.3   # 256 CUs x 2.4 GHz x 256 flop/clk/CU (v_mfma_f32_32x32x2_f32)
PEAK_INT8_TOPS = 5033.0    # 256 CUs x 2.4 GHz x 8192 op/clk/CU (v_mfma_i32_32x32x32_i8)


PEAK_HBM_TBS = 8.0         # HBM3E

# (kernel variant, digest of the sgemm kernel sources) -> bytes per 4096^3 launch:
# (FETCH_SIZE x 1.99965 + WRITE_SIZE) KiB.  The digest ties the figure to the kernel it was
# measured on: once any of those sources changes, `traffic` is reported as null.
SGEMM_KERNEL_SOURCES = ("sgemm_dma.hpp", "tile_f32.hpp", "sgemm_variants.hpp", "sgemm_gfx950.hip")  # the kernel, its instantiations, the launcher (tile walk)
MEASURED_TRAFFIC = {("sgemm_dma_256x128x16_w4x2_s2_c0", "ae8df5860a03003e"): 653727 * 1024}


def sgemm_kernel_digest() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in SGEMM_KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2205_00618_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def timed(fn, steps, warmup, torch):
    """Wall clock around exactly `steps` calls (synchronised on both sides) plus the
    stream-event time of the same region.  Returns (wall_ms_per_step, event_ms_per_step)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def warm_clocks(fn, torch, min_ms):
    """Back-to-back calls for at least min_ms of wall time: the shader clock ramps up over the
    first tens of milliseconds of load, and a short timed region that starts from idle clocks
    measures the ramp instead of the kernel.  Returns the time spent, in ms."""
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < min_ms:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3


def timed_in_graph(fn, torch, binding, calls=64, replays=20):
    """ms per call when `calls` calls are recorded in one HIP graph and the graph is replayed."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        binding.use_torch_stream()
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        binding.use_torch_stream()
        for _ in range(calls):
            fn()
    binding.use_torch_stream()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * calls)


def timed_steady(fn, torch, min_ms=40.0):
    """For the short side workloads: the clocks drop while the GPU idles between small
    launches, so warm up for min_ms of back-to-back calls, then time at least as long."""
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 0
    while (time.perf_counter() - t0) * 1e3 < min_ms:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        n += 20
    steps = max(20, n)
    return timed(fn, steps, 0, torch)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-extras", action="store_true", help="time only the headline workload")
    ap.add_argument("--cpu-seconds", type=float, default=30.0, help="upper bound on the oracle's time")
    ap.add_argument("--clock-warmup-ms", type=float, default=300.0,
                    help="back-to-back headline calls before the counted warm-up, so that the timed "
                         "region does not start from idle clocks whatever --steps and --warmup are")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one elementwise kernel that reads 256 MiB and writes 256 MiB, "
                         "outside the timed region, as the known-size reference for HBM counters")
    ap.add_argument("--variant", type=int, default=-1, help="force an sgemm tile configuration")
    ap.add_argument("--split-k", type=int, default=0)
    ap.add_argument("--tile-walk", type=int, default=0,
                    help="tile rows per band of the walk over C's tiles (0: the library's choice)")
    ap.add_argument("--conv-variant", type=int, default=-1, help="force a conv2d tile configuration")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this library runs on one GPU; --gpus must be 1 (the contractions shard "
            "without exchange by rows of C or by batch, which is not built here)")
        return 2

    import numpy as np
    import torch

    from paper_2205_00618_amd import binding, workloads as wl
    if not os.path.exists(binding.LIB_PATH):
        from paper_2205_00618_amd import build as lib_build
        lib_build.build(verbose=False)
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    torch.cuda.set_device(0)
    binding.use_torch_stream()
    assert binding.set_tuning(args.variant, args.split_k) == binding.OK
    assert binding.set_tile_walk(args.tile_walk) == binding.OK

    seed, shape = wl.SGEMM_4096
    A, B, C = wl.sgemm_inputs(seed, shape)
    dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dC = torch.zeros(shape.M, shape.N, device="cuda")
    flop = 2.0 * shape.M * shape.N * shape.K

    if args.calibration_copy:
        src = torch.ones(64 * 1024 * 1024, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)  # one kernel: 256 MiB read, 256 MiB written
        torch.cuda.synchronize()
        del src, dst

    clock_warmup_ms = warm_clocks(lambda: binding.sgemm_t(dA, dB, dC), torch, args.clock_warmup_ms)
    wall_ms, ev_ms = timed(lambda: binding.sgemm_t(dA, dB, dC), args.steps, args.warmup, torch)
    variant = binding.last_variant()
    tflops = flop / (wall_ms * 1e-3) / 1e12
    achieved = flop / (ev_ms * 1e-3) / 1e12
    log(f"sgemm 4096^3 [{variant}]: {wall_ms:.4f} ms/step wall, {ev_ms:.4f} ms/step events, "
        f"{tflops:.2f} TFLOP/s = {100 * tflops / PEAK_FP32_TFLOPS:.1f}% of {PEAK_FP32_TFLOPS}")

    # one checked launch from a fresh C (the timed launches kept accumulating)
    dC.zero_()
    binding.sgemm_t(dA, dB, dC)
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    parity = False  # set by the cpu-baseline leg, the only place the oracle is used

    # what the matrix pipes sustain on registers alone, beside the datasheet peaks
    words = torch.empty(8 * 1024 + 16, dtype=torch.int64, device="cuda")
    mfma_only = {}
    for key, int8, rnd in (("f32_random", False, True), ("f32_constant", False, False),
                           ("i8_random", True, True), ("i8_constant", True, False)):
        ops, hz = binding.mfma_rate(int8, rnd, words.data_ptr(), words.numel())
        mfma_only[key] = {"rate": round(ops / 1e12, 2), "unit": "TOP/s" if int8 else "TFLOP/s",
                          "shader_clock_ghz": round(hz / 1e9, 3)}
    mfma_only["datasheet"] = {"f32": PEAK_FP32_TFLOPS, "i8": PEAK_INT8_TOPS}
    log(f"matrix instructions on registers alone: {mfma_only}")
    del words

    extras = {}
    if not args.no_extras:
        binding.set_tuning(-1, 0)
        binding.set_tile_walk(0)
        # "ms": the plain call (partial sums of a cut reduction meet in atomic adds); "ms_ws": sgemm_ws,
        # where they meet in a workspace and are added in a fixed order (deterministic)
        ws = torch.zeros((65536 + (16 << 20)) // 4, device="cuda")
        for s, a, b_, c in wl.sgemm_ragged_inputs():
            da, db, dc = (torch.from_numpy(t).cuda() for t in (a, b_, c))
            w_ms, _ = timed_steady(lambda: binding.sgemm_t(da, db, dc), torch)
            f = 2.0 * s.M * s.N * s.K
            entry = {"ms": round(w_ms, 5), "tflops": round(f / w_ms / 1e9, 3),
                     "frac_of_peak": round(f / w_ms / 1e9 / PEAK_FP32_TFLOPS, 4),
                     "variant": binding.last_variant(), "slices": binding.last_split()}
            w_ms, _ = timed_steady(lambda: binding.sgemm_ws_t(da, db, dc, ws), torch)
            entry.update({"ms_ws": round(w_ms, 5), "tflops_ws": round(f / w_ms / 1e9, 3),
                          "variant_ws": binding.last_variant(), "slices_ws": binding.last_split()})
            extras[f"sgemm_{s.M}x{s.N}x{s.K}"] = entry
        del ws
        # the 4096^3 product on operands stored transposed (sgemm_op): the same rings fed through
        # the operand's index map, no extra pass over HBM
        for ta, tb in ((True, False), (False, True), (True, True)):
            w_ms, _ = timed_steady(lambda: binding.sgemm_op_t(ta, tb, dA, dB, dC), torch)   # square: any layout reading is valid
            extras[f"sgemm_op_{'t' if ta else 'n'}{'t' if tb else 'n'}_4096x4096x4096"] = {
                "ms": round(w_ms, 5), "tflops": round(flop / w_ms / 1e9, 3),
                "frac_of_peak": round(flop / w_ms / 1e9 / PEAK_FP32_TFLOPS, 4), "variant": binding.last_variant()}
        # the same 4096^3 product as one fully connected layer: bias as pre-, ReLU as post-operation
        dbias = torch.from_numpy(wl.uniform_f32(np.random.default_rng(5), (shape.N,))).cuda()
        w_ms, _ = timed_steady(lambda: binding.sgemm_fused_t(dA, dB, dC, dbias, binding.PRE_BIAS,
                                                             binding.POST_RELU), torch)
        extras["sgemm_fused_bias_relu_4096x4096x4096"] = {
            "ms": round(w_ms, 5), "tflops": round(flop / w_ms / 1e9, 3),
            "frac_of_peak": round(flop / w_ms / 1e9 / PEAK_FP32_TFLOPS, 4), "variant": binding.last_variant()}
        s0seed, s0 = wl.SGEMM_SMALL
        a, b_, c = (torch.from_numpy(t).cuda() for t in wl.sgemm_inputs(s0seed, s0))
        w_ms, _ = timed_steady(lambda: binding.sgemm_t(a, b_, c), torch)
        extras["sgemm_64x64x64"] = {"ms": round(w_ms, 5), "tflops": round(2.0 * 64**3 / w_ms / 1e9, 5),
                                    "variant": binding.last_variant()}
        binding.set_conv_tuning(args.conv_variant)
        cseed, cs = wl.CONV_56
        x, w = wl.conv_inputs(cseed, cs)
        dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        dout = torch.empty(cs.N, cs.P, cs.Q, cs.K, device="cuda")
        w_ms, _ = timed_steady(lambda: binding.conv2d_nhwc_t(dx, dw, dout, cs.stride, cs.pad), torch)
        f = 2.0 * cs.N * cs.P * cs.Q * cs.K * cs.R * cs.S * cs.C
        extras["conv2d_n32_56x56_c64_k64_3x3"] = {
            "ms": round(w_ms, 5), "tflops": round(f / w_ms / 1e9, 3),
            "frac_of_peak": round(f / w_ms / 1e9 / PEAK_FP32_TFLOPS, 4), "variant": binding.last_variant()}
        iseed, ish = wl.IGEMM_1024
        a8, b8, c32 = (torch.from_numpy(t).cuda() for t in wl.igemm_inputs(iseed, ish))
        c32.zero_()
        w_ms, _ = timed_steady(lambda: binding.igemm_s8s32_t(a8, b8, c32), torch, min_ms=10.0)
        f = 2.0 * ish.M * ish.N * ish.K
        extras["igemm_1024x1024x1024"] = {
            "ms": round(w_ms, 5), "tops": round(f / w_ms / 1e9, 3),
            "frac_of_peak": round(f / w_ms / 1e9 / PEAK_INT8_TOPS, 5), "variant": binding.last_variant()}
        # Table 1 of the evaluation: MM-64..512 and CONV-1..4 as listed (single image, hence
        # launch-bound on this machine), DWCONV-1..4 at batch 1 and at batch 256, where the
        # operation is HBM-bound; the batched runs rotate over several buffer sets so that the
        # Infinity Cache does not serve them
        # "ms" is one call per launch from the host; "ms_in_graph" the same call as one of 64
        # recorded in a HIP graph and replayed (the calls allocate nothing and wait for nothing,
        # so they can be captured), i.e. without the host's launch cost between dependent calls
        for s in wl.TABLE1_MM:
            a, b_, c = (torch.from_numpy(t).cuda() for t in wl.sgemm_inputs(6, s))
            w_ms, _ = timed_steady(lambda: binding.sgemm_t(a, b_, c), torch, min_ms=10.0)
            g_ms = timed_in_graph(lambda: binding.sgemm_t(a, b_, c), torch, binding)
            extras[f"table1_mm_{s.M}"] = {"ms": round(w_ms, 5), "ms_in_graph": round(g_ms, 5),
                                          "tflops": round(2.0 * s.M**3 / w_ms / 1e9, 4),
                                          "tflops_in_graph": round(2.0 * s.M**3 / g_ms / 1e9, 4),
                                          "variant": binding.last_variant()}
        for i, cs1 in enumerate(wl.TABLE1_CONV):
            x1, w1 = (torch.from_numpy(t).cuda() for t in wl.conv_inputs(7 + i, cs1))
            o1 = torch.empty(cs1.N, cs1.P, cs1.Q, cs1.K, device="cuda")
            w_ms, _ = timed_steady(lambda: binding.conv2d_nhwc_t(x1, w1, o1, cs1.stride, cs1.pad), torch, min_ms=10.0)
            g_ms = timed_in_graph(lambda: binding.conv2d_nhwc_t(x1, w1, o1, cs1.stride, cs1.pad), torch, binding)
            f = 2.0 * cs1.N * cs1.P * cs1.Q * cs1.K * cs1.R * cs1.S * cs1.C
            extras[f"table1_conv_{i + 1}"] = {"ms": round(w_ms, 5), "ms_in_graph": round(g_ms, 5),
                                              "tflops": round(f / w_ms / 1e9, 3),
                                              "tflops_in_graph": round(f / g_ms / 1e9, 3),
                                              "variant": binding.last_variant()}
        for batch in (1, 256):
            for i, ds in enumerate(wl.table1_dwconv(batch)):
                nset = max(1, min(8, int(2e9 // ds.bytes)))
                g = torch.Generator(device="cuda").manual_seed(wl.TABLE1_DWCONV_SEED)
                sets = [(torch.rand(ds.N, ds.H, ds.W, ds.C, device="cuda", generator=g),
                         torch.empty(ds.N, ds.P, ds.Q, ds.C, device="cuda")) for _ in range(nset)]
                _, wf, bf = wl.dwconv_inputs(wl.TABLE1_DWCONV_SEED, wl.DwConvShape(1, 1, 1, ds.C, ds.R, ds.S, 1, ds.pad))
                dwf, dbf = torch.from_numpy(wf).cuda(), torch.from_numpy(bf).cuda()
                turn = [0]

                def run_dw():
                    xin, xout = sets[turn[0] % nset]
                    turn[0] += 1
                    binding.dwconv2d_nhwc_t(xin, dwf, xout, ds.stride, ds.pad, dbf, binding.POST_RELU)

                w_ms, _ = timed_steady(run_dw, torch, min_ms=10.0 if batch == 1 else 40.0)
                tbs = ds.bytes / w_ms / 1e9
                extras[f"table1_dwconv_{i + 1}_batch{batch}"] = {
                    "ms": round(w_ms, 5), "tb_per_s": round(tbs, 3), "frac_of_hbm_peak": round(tbs / PEAK_HBM_TBS, 4),
                    "bytes": ds.bytes, "variant": binding.last_variant()}
                del sets
        # single-operand contraction (Section 5.2): layout changes as strided copies, HBM-bound
        copies = [("tensor_copy_nchw_to_nhwc_256x64x56x56_f32", torch.rand(256, 64, 56, 56, device="cuda").permute(0, 2, 3, 1)),
                  ("tensor_copy_transpose_8192x8192_f32", torch.rand(8192, 8192, device="cuda").t()),
                  ("tensor_copy_transpose_16384x16384_s8",
                   torch.randint(-128, 128, (16384, 16384), dtype=torch.int8, device="cuda").t()),
                  ("tensor_copy_rows_8192x8192_ld8200_f32", torch.rand(8192, 8200, device="cuda")[:, :8192])]
        for name, view in copies:
            dst = torch.empty(view.shape, dtype=view.dtype, device="cuda")
            w_ms, _ = timed_steady(lambda: binding.tensor_copy_t(view, dst), torch)
            moved = 2 * dst.numel() * dst.element_size()
            extras[name] = {"ms": round(w_ms, 5), "tb_per_s": round(moved / w_ms / 1e9, 3),
                            "frac_of_hbm_peak": round(moved / w_ms / 1e9 / PEAK_HBM_TBS, 4), "bytes": moved,
                            "variant": binding.last_variant()}
            del dst, view
        del copies
        # the int8 product at a size where it is not launch-bound
        big = wl.GemmShape(4096, 4096, 4096)
        a8, b8, c32 = (torch.from_numpy(t).cuda() for t in wl.igemm_inputs(iseed, big))
        w_ms, _ = timed_steady(lambda: binding.igemm_s8s32_t(a8, b8, c32), torch)   # sums wrap, harmless for timing
        f = 2.0 * big.M * big.N * big.K
        extras["igemm_4096x4096x4096"] = {
            "ms": round(w_ms, 5), "tops": round(f / w_ms / 1e9, 3),
            "frac_of_peak": round(f / w_ms / 1e9 / PEAK_INT8_TOPS, 5), "variant": binding.last_variant()}
        del a8, b8, c32
        # shapes off the aligned, many-tile path: a few rows against a large B (bound by reading
        # B once: rate in bytes of B), a channel count that is a multiple of 4 only, ragged int8
        few = wl.GemmShape(8, 4096, 4096)
        a, b_, c = (torch.from_numpy(t).cuda() for t in wl.sgemm_inputs(6, few))
        copies_b = [b_] + [b_.clone() for _ in range(4)]   # 335 MB in rotation: more than the Infinity Cache holds
        turn = [0]

        def few_rows():
            turn[0] = (turn[0] + 1) % len(copies_b)
            binding.sgemm_t(a, copies_b[turn[0]], c)
        w_ms, _ = timed_steady(few_rows, torch)
        del copies_b
        extras["sgemm_8x4096x4096"] = {"ms": round(w_ms, 5), "tb_per_s": round(4.0 * few.N * few.K / w_ms / 1e9, 3),
                                       "frac_of_hbm_peak": round(4.0 * few.N * few.K / w_ms / 1e9 / PEAK_HBM_TBS, 4),
                                       "variant": binding.last_variant()}
        c60 = wl.ConvShape(32, 56, 56, 60, 64, 3, 3, 1, 1)
        x, w = wl.conv_inputs(7, c60)
        dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
        dout = torch.empty(c60.N, c60.P, c60.Q, c60.K, device="cuda")
        w_ms, _ = timed_steady(lambda: binding.conv2d_nhwc_t(dx, dw, dout, c60.stride, c60.pad), torch)
        f = 2.0 * c60.N * c60.P * c60.Q * c60.K * c60.R * c60.S * c60.C
        extras["conv2d_n32_56x56_c60_k64_3x3"] = {
            "ms": round(w_ms, 5), "tflops": round(f / w_ms / 1e9, 3),
            "frac_of_peak": round(f / w_ms / 1e9 / PEAK_FP32_TFLOPS, 4), "variant": binding.last_variant()}
        rag = wl.GemmShape(4000, 4000, 4000)
        a8, b8, c32 = (torch.from_numpy(t).cuda() for t in wl.igemm_inputs(8, rag))
        w_ms, _ = timed_steady(lambda: binding.igemm_s8s32_t(a8, b8, c32), torch)
        f = 2.0 * rag.M * rag.N * rag.K
        extras["igemm_4000x4000x4000"] = {
            "ms": round(w_ms, 5), "tops": round(f / w_ms / 1e9, 3),
            "frac_of_peak": round(f / w_ms / 1e9 / PEAK_INT8_TOPS, 5), "variant": binding.last_variant()}
        del a8, b8, c32
        # int8 operands whose rows are only 4-byte aligned (dense 1000 x 1000): the 4-byte direct-to-LDS loads
        r4 = wl.GemmShape(1000, 1000, 1000)
        a8, b8, c32 = (torch.from_numpy(t).cuda() for t in wl.igemm_inputs(9, r4))
        w_ms, _ = timed_steady(lambda: binding.igemm_s8s32_t(a8, b8, c32), torch, min_ms=10.0)
        extras["igemm_1000x1000x1000"] = {"ms": round(w_ms, 5), "tops": round(2.0e9 / w_ms / 1e9, 3),
                                          "variant": binding.last_variant()}
        del a8, b8, c32
        # a fully connected layer with bias and ReLU at a small batch (the MLP of Section 3's listing):
        # weights K x N, and stored output-major (N x K) through sgemm_op
        fc = wl.GemmShape(64, 1024, 4096)
        a, b_, c = (torch.from_numpy(t).cuda() for t in wl.sgemm_inputs(10, fc))
        fbias = torch.from_numpy(wl.uniform_f32(np.random.default_rng(11), (fc.N,))).cuda()
        w_ms, _ = timed_steady(lambda: binding.sgemm_fused_t(a, b_, c, fbias, binding.PRE_BIAS, binding.POST_RELU),
                               torch, min_ms=10.0)
        extras["sgemm_fused_bias_relu_64x1024x4096"] = {
            "ms": round(w_ms, 5), "tflops": round(2.0 * fc.M * fc.N * fc.K / w_ms / 1e9, 3),
            "variant": binding.last_variant(), "slices": binding.last_split()}
        fc8 = wl.GemmShape(8, 4096, 4096)
        a, b_, c = (torch.from_numpy(t).cuda() for t in wl.sgemm_inputs(12, fc8))
        bt_ = b_.t().contiguous()
        w_ms, _ = timed_steady(lambda: binding.sgemm_op_t(False, True, a, bt_, c), torch, min_ms=10.0)
        extras["sgemm_op_nt_8x4096x4096"] = {
            "ms": round(w_ms, 5), "tb_per_s": round(4.0 * fc8.N * fc8.K / w_ms / 1e9, 3),
            "frac_of_hbm_peak": round(4.0 * fc8.N * fc8.K / w_ms / 1e9 / PEAK_HBM_TBS, 4), "variant": binding.last_variant()}
        # a matrix-vector product
        mv = wl.GemmShape(4096, 1, 4096)
        a, b_, c = (torch.from_numpy(t).cuda() for t in wl.sgemm_inputs(13, mv))
        w_ms, _ = timed_steady(lambda: binding.sgemm_t(a, b_, c), torch, min_ms=10.0)
        extras["sgemm_4096x1x4096"] = {
            "ms": round(w_ms, 5), "tb_per_s": round(4.0 * mv.M * mv.K / w_ms / 1e9, 3),
            "frac_of_hbm_peak": round(4.0 * mv.M * mv.K / w_ms / 1e9 / PEAK_HBM_TBS, 4), "variant": binding.last_variant()}
        # an RGB stem: the layout change NCHW -> NHWC of the image batch, then 7 x 7, stride 2, 3 -> 64 channels
        img = torch.rand(32, 3, 224, 224, device="cuda")
        nhwc = torch.empty(32, 224, 224, 3, device="cuda")
        w_ms, _ = timed_steady(lambda: binding.tensor_copy_t(img.permute(0, 2, 3, 1), nhwc), torch, min_ms=10.0)
        extras["tensor_copy_nchw_to_nhwc_32x3x224x224_f32"] = {
            "ms": round(w_ms, 5), "tb_per_s": round(2.0 * img.numel() * 4 / w_ms / 1e9, 3),
            "frac_of_hbm_peak": round(2.0 * img.numel() * 4 / w_ms / 1e9 / PEAK_HBM_TBS, 4), "variant": binding.last_variant()}
        stem = wl.ConvShape(32, 224, 224, 3, 64, 7, 7, 2, 3)
        wst = torch.from_numpy(wl.conv_inputs(14, wl.ConvShape(1, 7, 7, 3, 64, 7, 7, 1, 0))[1]).cuda()
        ost = torch.empty(stem.N, stem.P, stem.Q, stem.K, device="cuda")
        w_ms, _ = timed_steady(lambda: binding.conv2d_nhwc_t(nhwc, wst, ost, stem.stride, stem.pad), torch)
        f = 2.0 * stem.N * stem.P * stem.Q * stem.K * stem.R * stem.S * stem.C
        extras["conv2d_n32_224x224_c3_k64_7x7_s2"] = {
            "ms": round(w_ms, 5), "tflops": round(f / w_ms / 1e9, 3),
            "frac_of_peak": round(f / w_ms / 1e9 / PEAK_FP32_TFLOPS, 4), "variant": binding.last_variant()}
        del img, nhwc, ost
        for k, v in extras.items():
            log(f"  {k}: {v}")

    cpu_baseline = None
    if not args.no_cpu_baseline:
        # The oracle, as it stands, on the same workload: a first slab of rows gives its rate,
        # then as many more rows as --cpu-seconds allows -- all of them on a host with 16 cores.
        import oracle
        cores = oracle.num_threads()
        rows = max(cores, 8)
        t0 = time.perf_counter()
        ref, absum = oracle.sgemm(A[:rows], B, C[:rows])
        dt = time.perf_counter() - t0
        err = np.abs(got[:rows].astype(np.float64) - ref)
        ok = bool(np.all(err <= 1e-5 * absum))
        more = int(min(shape.M - rows, rows * max(args.cpu_seconds - dt, 0) / max(dt, 1e-9)))
        if more < shape.M - rows:
            more -= more % cores
        total_rows, total_dt = rows, dt
        if more > 0:
            t0 = time.perf_counter()
            ref2, absum2 = oracle.sgemm(A[rows:rows + more], B, C[rows:rows + more])
            total_dt += time.perf_counter() - t0
            err2 = np.abs(got[rows:rows + more].astype(np.float64) - ref2)
            ok = ok and bool(np.all(err2 <= 1e-5 * absum2))
            total_rows += more
        cpu_tflops = 2.0 * total_rows * shape.N * shape.K / total_dt / 1e12
        cpu_baseline = {"value": round(cpu_tflops, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                        "sample": f"first {total_rows} of {shape.M} rows of C of the same 4096^3 workload "
                                  f"({total_dt:.1f} s); GPU result on those rows within tolerance: {ok}"}
        parity = f"every element of {total_rows} of {shape.M} rows"
        log(f"oracle: {total_rows} rows in {total_dt:.2f} s on {cores} threads = {cpu_tflops * 1e3:.2f} GFLOP/s; "
            f"parity on the slab: {ok}")
        if not ok:
            log("bench.py: GPU result disagrees with the oracle")
            return 4

    # HBM-side bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs; valid only for
    # the kernel and library version they were taken on.
    traffic = MEASURED_TRAFFIC.get((variant, sgemm_kernel_digest()))

    line = {
        "metric": "SGEMM fp32 TFLOP/s at M=N=K=4096 (% of MI355X fp32 matrix peak)",
        "value": round(tflops, 3), "unit": "TFLOP/s", "pct_of_peak": round(100 * tflops / PEAK_FP32_TFLOPS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 5),
        "clock_warmup_ms": round(clock_warmup_ms, 1), "parity_checked": parity,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "sgemm M=N=K=4096 row-major lda=ldb=ldc=4096, A,B ~ U[-1,1] seed 1, C zeros",
                   "variant": variant},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_FP32_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_TFLOPS, 4), "traffic": traffic},
        "cpu_baseline": cpu_baseline,
        "mfma_only": mfma_only,
        "extras": extras,
    }
    print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
