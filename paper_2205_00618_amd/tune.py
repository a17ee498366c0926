"""Scripted tuning over the kernel templates' parameters (Section 6.3, "Scripted Tuning").

The paper's script sweeps schedules in three steps and keeps the best of each for the
next: (1) tile and register-block sizes, (2) the order of compute, (3) staging / packing.
The schedules of this library are fixed kernel templates, so the same three steps walk
the knobs the C ABI exposes for sweeps:

  step 1  tile configuration: workgroup tile x wave tile (``lsmi_set_tuning`` /
          ``lsmi_set_conv_tuning`` / ``lsmi_set_dwconv_tuning`` variant index), restricted
          to one staging family;
  step 2  order of compute: how the reduction (sgemm split-K, conv reduction slices) or
          the row walk (dwconv rows per lane / per workgroup) is cut across workgroups;
  step 3  staging: the other staging families (register-staged, direct-to-LDS rings of
          several depths, LDS-staged tiles) around the best tile of step 1.

Every candidate is reported with the three statistics the paper's interface shows for a
schedule: total operations, arithmetic intensity (operations per byte of the operands
read and written once) and the achieved rate.  A candidate counts only if it computes the
same thing: before it is timed it runs once on operands of small integers (every partial
sum exact in fp32, so any summation order gives the same bits) and its result must equal,
bit for bit, the result of the library's own choice on the same operands; a candidate
that differs is reported as WRONG and never wins.

    python -m paper_2205_00618_amd.tune sgemm 1000 1000 1000
    python -m paper_2205_00618_amd.tune sgemm 1000 1000 1000 --workspace   # sgemm_ws: slices meet in a workspace
    python -m paper_2205_00618_amd.tune igemm 4096 4096 4096
    python -m paper_2205_00618_amd.tune conv 1 28 28 128 256 3 3 1 0
    python -m paper_2205_00618_amd.tune dwconv 256 28 28 88 3 3 1 1
    python -m paper_2205_00618_amd.tune sgemm 256 256 8192 --builtin 2000  # only the library's choice, 2000 calls
    python -m paper_2205_00618_amd.tune table                              # the choice against forced kernels
    python -m paper_2205_00618_amd.tune table --grid 1024,2048,4096 128,2048  # the same on round shapes

Needs the built library and a GPU; the last line printed is the best configuration as JSON.
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Tuple


@dataclass(frozen=True)
class Stats:
    """Operation count, bytes moved when every operand is read or written once, and the
    ratio of the two (the roofline abscissa)."""
    ops: float
    bytes: float

    @property
    def intensity(self) -> float:
        return self.ops / self.bytes if self.bytes else float("inf")


def sgemm_stats(M: int, N: int, K: int, elem_in: int = 4, elem_out: int = 4) -> Stats:
    return Stats(2.0 * M * N * K, float(elem_in * (M * K + K * N) + 2 * elem_out * M * N))


def conv_stats(N, H, W, C, K, R, S, stride, pad) -> Stats:
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    return Stats(2.0 * N * P * Q * K * R * S * C, 4.0 * (N * H * W * C + K * R * S * C + N * P * Q * K))


def dwconv_stats(N, H, W, C, R, S, stride, pad) -> Stats:
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    return Stats(2.0 * N * P * Q * C * R * S, 4.0 * (N * H * W * C + R * S * C + N * P * Q * C))


def staging_family(name: str) -> str:
    """Which way a kernel variant brings its operands on chip."""
    if "_rows_" in name:
        return "global to registers"
    if "_dma_edge" in name:
        return "direct-to-LDS (ragged)"
    if "_dma_" in name:
        return "direct-to-LDS"
    if "_lds_" in name:
        return "LDS-staged"
    if "_window_" in name:
        return "register window"
    if "_direct_" in name:
        return "direct"
    return "register-staged"


@dataclass
class Candidate:
    step: int
    label: str
    apply: Callable[[], None]
    us: float = float("nan")
    ran: str = ""
    ok: bool = True  # computed the same bits as the library's own choice on small-integer operands


class Sweep:
    """Times candidates of one operation; a candidate the library maps to another kernel
    (because it does not fit the shape) is recorded under the kernel that actually ran."""

    def __init__(self, stats: Stats, run: Callable[[], None], reset: Callable[[], None], torch, binding,
                 min_ms: float = 20.0, exact: Optional[Callable[[], object]] = None):
        """exact: runs the operation once on small-integer operands under the current settings
        and returns the output tensor; the library's own choice gives the expected bits."""
        self.stats, self.run, self.reset = stats, run, reset
        self.torch, self.binding, self.min_ms = torch, binding, min_ms
        self.rows: List[Candidate] = []
        self.exact, self.expected = exact, None
        if exact is not None:
            reset()
            self.expected = exact().clone()
            torch.cuda.synchronize()

    def time_us(self) -> float:
        torch = self.torch
        self.run()
        torch.cuda.synchronize()
        t0, n = time.perf_counter(), 0
        while (time.perf_counter() - t0) * 1e3 < self.min_ms:  # steady clocks
            for _ in range(10):
                self.run()
            torch.cuda.synchronize()
            n += 10
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(max(n, 10)):
            self.run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / max(n, 10)

    def measure(self, cand: Candidate) -> Candidate:
        self.reset()
        cand.apply()
        if self.exact is not None:
            got = self.exact()
            self.torch.cuda.synchronize()
            cand.ok = bool(self.torch.equal(got, self.expected))
        cand.us = self.time_us()
        cand.ran = self.binding.last_variant()
        self.rows.append(cand)
        rate = self.stats.ops / cand.us / 1e3
        print(f"  step {cand.step}  {cand.label:<44s} {cand.ran:<40s} {cand.us:9.2f} us  {rate:10.1f} Gop/s"
              f"{'' if cand.ok else '  WRONG RESULT'}", file=sys.stderr, flush=True)
        return cand

    def best(self, step: Optional[int] = None) -> Candidate:
        rows = [r for r in self.rows if r.ok and (step is None or r.step == step)]
        return min(rows, key=lambda r: r.us)


def report(op: str, shape, sweep: Sweep, peak: float, unit: str) -> Dict:
    s, b = sweep.stats, sweep.best()
    rate = s.ops / b.us / 1e6  # operations per microsecond / 1e6 = tera-operations per second
    out = {"op": op, "shape": list(shape), "operations": s.ops, "bytes": s.bytes,
           "arithmetic_intensity": round(s.intensity, 3), "best": {"label": b.label, "kernel": b.ran,
           "us": round(b.us, 3), "rate": round(rate, 4), "unit": unit, "frac_of_peak": round(rate / peak, 4)},
           "candidates": len(sweep.rows), "verified": sweep.exact is not None,
           "wrong": [r.label for r in sweep.rows if not r.ok]}
    own = [r for r in sweep.rows if r.step == 0 and r.ok]  # the library's own choice, timed first
    if own:
        out["built_in"] = {"kernel": own[0].ran, "us": round(own[0].us, 3), "over_best": round(own[0].us / b.us, 3)}
    print(json.dumps(out), flush=True)
    return out


def small_integers(torch, shape, bound=8, dtype=None):
    return torch.randint(-bound, bound + 1, shape, device="cuda").to(dtype or torch.float32)


def tune_sgemm(M: int, N: int, K: int, workspace: bool = False) -> Dict:
    import torch
    from . import binding as b
    b.use_torch_stream()
    A = torch.rand(M, K, device="cuda") * 2 - 1
    B = torch.rand(K, N, device="cuda") * 2 - 1
    C = torch.zeros(M, N, device="cuda")
    ws = torch.zeros((65536 + (16 << 20)) // 4, device="cuda") if workspace else None
    call = (lambda a, bb, c: b.sgemm_ws_t(a, bb, c, ws)) if workspace else b.sgemm_t
    Ai, Bi, Ci = small_integers(torch, (M, K)), small_integers(torch, (K, N)), torch.empty(M, N, device="cuda")

    def exact():
        Ci.zero_()
        call(Ai, Bi, Ci)
        return Ci

    def reset():
        b.set_tuning(-1, 0)
        b.set_tile_walk(0)

    sweep = Sweep(sgemm_stats(M, N, K), lambda: call(A, B, C), reset, torch, b, exact=exact)
    names = b.variant_names()
    sweep.measure(Candidate(0, "built-in choice", lambda: None))
    # step 1: tiles of the register-staged family (they take every shape)
    for i, n in enumerate(names):
        if staging_family(n) == "register-staged":
            sweep.measure(Candidate(1, f"tile {n}", lambda i=i: b.set_tuning(i, 1)))
    tile = names.index(sweep.best(1).ran) if sweep.best(1).ran in names else 0
    # step 2: where the reduction is cut
    for split in (2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64):
        if K // split >= 16:
            sweep.measure(Candidate(2, f"tile {names[tile]} split-K {split}", lambda s=split: b.set_tuning(tile, s)))
    # ... and the order in which the tiles are walked (tile rows per band), for outputs of many tiles
    if (M // 128) * (N // 128) >= 512:
        for rows in (1, 2, 4, 16, 32):
            def pick(rows=rows):
                b.set_tuning(-1, 0)
                b.set_tile_walk(rows)
            sweep.measure(Candidate(2, f"built-in kernel, bands of {rows} tile rows", pick))
        b.set_tile_walk(0)
    # step 3: the direct-to-LDS families (ring depth, tile), unsplit and with the best split
    best_split = 1
    b2 = sweep.best(2) if any(r.step == 2 for r in sweep.rows) else None
    if b2 is not None and b2.us < sweep.best(1).us:
        best_split = int(b2.label.rsplit(" ", 1)[1])
    for i, n in enumerate(names):
        if "_rows_" in n and M > 64:
            continue    # the few-row kernels re-read B once per 16 rows: not a candidate for a tall output
        if staging_family(n) != "register-staged":
            sweep.measure(Candidate(3, f"staging {n}", lambda i=i: b.set_tuning(i, 1)))
            if best_split > 1 and "edge" in n:
                sweep.measure(Candidate(3, f"staging {n} split-K {best_split}",
                                        lambda i=i: b.set_tuning(i, best_split)))
            if "edge" in n or "_rows_" in n:  # the library's own cut: uniform, or only the last round's tiles
                c = sweep.measure(Candidate(3, f"staging {n} built-in cut", lambda i=i: b.set_tuning(i, 0)))
                if c.ran == n:
                    sweep.rows.pop()  # it chose no cut: the unsplit row above already says so
    b.set_tuning(-1, 0)
    return report("sgemm_ws" if workspace else "sgemm", (M, N, K), sweep, 157.3, "TFLOP/s")


def tune_igemm(M: int, N: int, K: int) -> Dict:
    """The signed 8-bit product: (1) tiles of one staging family, (2) the cut of the reduction
    for the tiles that take one, (3) the other staging families and ring depths."""
    import torch
    from . import binding as b
    b.use_torch_stream()
    A = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
    B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device="cuda")
    C = torch.zeros(M, N, dtype=torch.int32, device="cuda")
    Ci = torch.empty(M, N, dtype=torch.int32, device="cuda")

    def exact():  # integer sums are exact in any order: the timed operands serve
        Ci.zero_()
        b.igemm_s8s32_t(A, B, Ci)
        return Ci

    def reset():
        b.set_igemm_tuning(-1)
        b.set_tuning(-1, 0)

    sweep = Sweep(sgemm_stats(M, N, K, elem_in=1), lambda: b.igemm_s8s32_t(A, B, C), reset, torch, b, exact=exact)
    names = b.igemm_variant_names()
    sweep.measure(Candidate(0, "built-in choice", lambda: None))
    direct = [i for i, n in enumerate(names) if "_dma_" in n or "_big_" in n]
    for i in direct:  # step 1: tiles of the direct-to-LDS family with the shallowest ring of each tile
        if names[i].endswith("_s2") or "_big_" in names[i] or "_edge_" in names[i]:
            sweep.measure(Candidate(1, f"tile {names[i]}", lambda i=i: b.set_igemm_tuning(i)))
    ran1 = sweep.best(1).ran if any(r.step == 1 for r in sweep.rows) else ""
    tile = names.index(ran1) if ran1 in names else direct[0]
    for split in (2, 3, 4, 6, 8, 16):  # step 2: the reduction cut over workgroups (integer atomics: still exact)
        if K // split >= 256:
            def pick(split=split):
                b.set_igemm_tuning(tile)
                b.set_tuning(-1, split)
            sweep.measure(Candidate(2, f"tile {names[tile]} split-K {split}", pick))
    for i, n in enumerate(names):  # step 3: deeper rings of the same family, and the register-staged kernels
        if i not in direct or not (n.endswith("_s2") or "_big_" in n or "_edge_" in n):
            sweep.measure(Candidate(3, f"staging {n}", lambda i=i: b.set_igemm_tuning(i)))
    reset()
    return report("igemm_s8s32", (M, N, K), sweep, 5033.0 / 1e0, "TOP/s")


def tune_conv(N, H, W, C, K, R, S, stride, pad) -> Dict:
    import torch
    from . import binding as b
    b.use_torch_stream()
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    x = torch.rand(N, H, W, C, device="cuda")
    w = torch.randn(K, R, S, C, device="cuda") * 0.1
    out = torch.empty(N, P, Q, K, device="cuda")

    def reset():
        b.set_conv_tuning(-1)
        b.set_conv_split(0)
        b.set_conv_tail(-1)

    xi, wi, oi = small_integers(torch, (N, H, W, C), 4), small_integers(torch, (K, R, S, C), 4), torch.empty_like(out)

    def exact():
        oi.fill_(float("nan"))
        b.conv2d_nhwc_t(xi, wi, oi, stride, pad)
        return oi

    sweep = Sweep(conv_stats(N, H, W, C, K, R, S, stride, pad),
                  lambda: b.conv2d_nhwc_t(x, w, out, stride, pad), reset, torch, b, exact=exact)
    names = b.conv_variant_names()
    sweep.measure(Candidate(0, "built-in choice", lambda: None))
    for i, n in enumerate(names):  # step 1: register-staged tiles
        if staging_family(n) == "register-staged":
            sweep.measure(Candidate(1, f"tile {n}", lambda i=i: b.set_conv_tuning(i)))
    staged = [i for i, n in enumerate(names) if staging_family(n) != "register-staged"]
    for i in staged:  # step 3 before step 2: only the direct-to-LDS kernels can cut the reduction
        def pick(i=i):
            b.set_conv_tuning(i)
            b.set_conv_split(1)
        sweep.measure(Candidate(3, f"staging {names[i]}", pick))
    s3 = [r for r in sweep.rows if r.step == 3 and r.ran in names and names.index(r.ran) in staged]
    if s3:
        tile = names.index(min(s3, key=lambda r: r.us).ran)
        chunks = R * S * C // (32 if "x32_" in names[tile] else 16)
        for slices in (2, 3, 4, 6, 9, 12, 18, 24, 36):
            if chunks // slices >= 2:
                def pick(slices=slices):
                    b.set_conv_tuning(tile)
                    b.set_conv_split(slices)
                sweep.measure(Candidate(2, f"staging {names[tile]} slices {slices}", pick))
        # the other cut: the last, partly filled round of tiles as quarter-tile pieces or whole
        for i in staged:
            if "_w2x2_" not in names[i] or "_c4_" in names[i] or "_c1_" in names[i]:  # (the per-lane-tap kernels: whole tiles only)
                continue
            bm = int(names[i].split("_dma_")[1].split("x")[0])
            rem = ((N * P * Q + bm - 1) // bm * ((K + 63) // 64)) % 256
            if rem == 0:
                continue
            rows = (rem + (K + 63) // 64 - 1) // ((K + 63) // 64)
            for tail, label in ((0, "whole tiles"), (rows, f"{rows} tile rows as pieces")):
                def pick(i=i, tail=tail):
                    b.set_conv_tuning(i)
                    b.set_conv_split(1)
                    b.set_conv_tail(tail)
                sweep.measure(Candidate(2, f"staging {names[i]} {label}", pick))
    reset()
    return report("conv2d_nhwc", (N, H, W, C, K, R, S, stride, pad), sweep, 157.3, "TFLOP/s")


def tune_dwconv(N, H, W, C, R, S, stride, pad) -> Dict:
    import torch
    from . import binding as b
    b.use_torch_stream()
    P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    stats = dwconv_stats(N, H, W, C, R, S, stride, pad)
    nset = max(1, min(8, int(2e9 // stats.bytes)))  # rotate buffers: keep the Infinity Cache out
    sets = [(torch.rand(N, H, W, C, device="cuda"), torch.empty(N, P, Q, C, device="cuda")) for _ in range(nset)]
    w = torch.randn(R, S, C, device="cuda") * 0.1
    turn = [0]

    def run():
        xin, xout = sets[turn[0] % nset]
        turn[0] += 1
        b.dwconv2d_nhwc_t(xin, w, xout, stride, pad)

    def reset():
        b.set_dwconv_tuning(-1, 0)
        b.set_dwconv_tile(0, 0, 0)

    xi, wi = small_integers(torch, (N, H, W, C), 4), small_integers(torch, (R, S, C), 4)
    oi = torch.empty(N, P, Q, C, device="cuda")

    def exact():
        oi.fill_(float("nan"))
        b.dwconv2d_nhwc_t(xi, wi, oi, stride, pad)
        return oi

    sweep = Sweep(stats, run, reset, torch, b, exact=exact)
    names = b.dwconv_variant_names()
    sweep.measure(Candidate(0, "built-in choice", lambda: None))
    seen = set()
    for i, n in enumerate(names):  # step 1: lane shape of the kernels that keep their data in registers
        if staging_family(n) in ("register window", "direct"):
            c = sweep.measure(Candidate(1, f"kernel {n}", lambda i=i: b.set_dwconv_tuning(i, 0)))
            seen.add(c.ran)
    best1 = sweep.best(1).ran
    if staging_family(best1) == "register window":  # step 2: rows a lane walks
        i1 = names.index(best1)
        for strip in (2, 3, 4, 6, 8, 12, 16, 24, 32):
            if strip <= P:
                sweep.measure(Candidate(2, f"kernel {best1} rows/lane {strip}",
                                        lambda strip=strip: b.set_dwconv_tuning(i1, strip)))
    for i, n in enumerate(names):  # step 3: LDS staging, with its own row walk and prefetch depth
        if staging_family(n) != "LDS-staged":
            continue
        for depth in (2, 1):
            def pick(i=i, depth=depth):
                b.set_dwconv_tuning(i, 0)
                b.set_dwconv_tile(0, 0, depth)
            c = sweep.measure(Candidate(3, f"staging {n} depth {depth}", pick))
            if c.ran != n:
                sweep.rows.pop()  # does not fit this filter / stride
                break
    reset()
    # HBM-bound: the roof at this intensity is 8 TB/s x operations per byte
    return report("dwconv2d_nhwc", (N, H, W, C, R, S, stride, pad), sweep, 8.0 * stats.intensity,
                  "TFLOP/s (peak = HBM roof at this intensity)")


def builtin_only(op: str, dims, calls: int, workspace: bool = False) -> Dict:
    """Times only the library's own choice: `calls` calls back to back after a warm-up by time.
    The command for profiling one workload with rocprofv3 (kernel trace or counters)."""
    import torch
    from . import binding as b
    b.use_torch_stream()
    if op in ("sgemm", "igemm"):
        M, N, K = dims
        if op == "sgemm":
            A, B = torch.rand(M, K, device="cuda") * 2 - 1, torch.rand(K, N, device="cuda") * 2 - 1
            C = torch.zeros(M, N, device="cuda")
            ws = torch.zeros((65536 + (16 << 20)) // 4, device="cuda") if workspace else None
            run = (lambda: b.sgemm_ws_t(A, B, C, ws)) if workspace else (lambda: b.sgemm_t(A, B, C))
            stats, unit = sgemm_stats(M, N, K), "TFLOP/s"
        else:
            A = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
            B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device="cuda")
            C = torch.zeros(M, N, dtype=torch.int32, device="cuda")
            run = lambda: b.igemm_s8s32_t(A, B, C)
            stats, unit = sgemm_stats(M, N, K, elem_in=1), "TOP/s"
    elif op == "conv":
        N, H, W, C_, K, R, S, stride, pad = dims
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        x, w = torch.rand(N, H, W, C_, device="cuda"), torch.randn(K, R, S, C_, device="cuda") * 0.1
        out = torch.empty(N, P, Q, K, device="cuda")
        run = lambda: b.conv2d_nhwc_t(x, w, out, stride, pad)
        stats, unit = conv_stats(*dims), "TFLOP/s"
    elif op == "dwconv":
        N, H, W, C_, R, S, stride, pad = dims
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        stats, unit = dwconv_stats(*dims), "TFLOP/s"
        nset = max(1, min(8, int(2e9 // stats.bytes)))  # rotate buffers: keep the Infinity Cache out
        sets = [(torch.rand(N, H, W, C_, device="cuda"), torch.empty(N, P, Q, C_, device="cuda")) for _ in range(nset)]
        w = torch.randn(R, S, C_, device="cuda") * 0.1
        turn = [0]

        def run():
            xin, xout = sets[turn[0] % nset]
            turn[0] += 1
            b.dwconv2d_nhwc_t(xin, w, xout, stride, pad)
    else:
        raise ValueError("--builtin serves sgemm, igemm, conv and dwconv")
    sweep = Sweep(stats, run, lambda: None, torch, b, min_ms=40.0)
    sweep.time_us()  # warm-up by time
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(calls):
        run()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / calls
    out = {"op": op + ("_ws" if workspace else ""), "shape": list(dims), "kernel": b.last_variant(),
           "slices": b.last_split() if op == "sgemm" else None, "calls": calls, "us": round(us, 3),
           "rate": round(stats.ops / us / 1e6, 4), "unit": unit, "operations": stats.ops, "bytes": stats.bytes}
    print(json.dumps(out), flush=True)
    return out


# Shapes of the table: whole rounds and incomplete rounds of 128 x 128 and 64 x 64 tiles, ragged
# and unaligned extents, small outputs with long reductions, short reductions, few rows.
TABLE_SHAPES = [(4096, 4096, 4096), (4096, 4096, 256), (1000, 1000, 1000), (256, 256, 8192), (4097, 129, 511),
                (1024, 1024, 1024), (1536, 1536, 1536), (2048, 2048, 2048), (3072, 3072, 3072), (4000, 4000, 4000),
                (2304, 2304, 2304), (3000, 3000, 304), (1024, 1024, 128), (4096, 2048, 256), (4000, 4000, 64),
                (512, 512, 512), (768, 768, 3072), (2000, 100, 1000), (384, 384, 4096), (640, 640, 1280),
                (1800, 1800, 1800), (3500, 1000, 2000), (2001, 2001, 2001), (8, 4096, 4096), (8192, 4096, 4096)]


def choice_table(shapes=None, min_ms: float = 10.0, out=sys.stdout, layout: str = "nn") -> List[Dict]:
    """The library's own choice against every kernel variant forced in turn (whole reduction,
    the library's cut, and a few uniform cuts for small outputs): one row per shape.
    layout: "nn" (sgemm) or "nt", "tn", "tt" (sgemm_op on operands stored transposed)."""
    import torch
    from . import binding as b
    b.use_torch_stream()
    names = b.variant_names()
    ta, tb = layout[0] == "t", layout[1] == "t"
    suffix = "" if layout == "nn" else "_" + layout
    rows = []
    print("| M x N x K | built-in kernel (slices) | built-in us | best forced | best forced us | built-in / best |",
          file=out)
    print("|---|---|---|---|---|---|", file=out)
    for M, N, K in shapes or TABLE_SHAPES:
        A = torch.rand((K, M) if ta else (M, K), device="cuda") * 2 - 1
        B = torch.rand((N, K) if tb else (K, N), device="cuda") * 2 - 1
        C = torch.zeros(M, N, device="cuda")
        call = (lambda: b.sgemm_t(A, B, C)) if layout == "nn" else (lambda: b.sgemm_op_t(ta, tb, A, B, C))
        sweep = Sweep(sgemm_stats(M, N, K), call, lambda: b.set_tuning(-1, 0), torch, b, min_ms=min_ms)
        b.set_tuning(-1, 0)
        base = min(sweep.time_us() for _ in range(3))
        base_name, base_split = b.last_variant(), b.last_split()
        best_us, best_label = float("inf"), ""
        small = (M + 63) // 64 * ((N + 63) // 64) < 512
        for i, n in enumerate(names):
            if ("_rows_" in n and M > 32) or ("_cols_" in n and N > 16):
                continue
            for split in ([1, 0] + ([2, 4, 8, 16] if small and "edge" in n else [])):
                if split > 1 and K // split < 64:
                    continue
                b.set_tuning(i, split)
                us = sweep.time_us()
                if b.last_variant() not in (n + suffix, n + "_tail" + suffix):
                    break  # the kernel does not take this shape
                if us < best_us:
                    best_us, best_label = us, f"{b.last_variant()} ({b.last_split()})"
        b.set_tuning(-1, 0)
        rows.append({"shape": (M, N, K), "builtin": base_name, "builtin_us": base, "best": best_label,
                     "best_us": best_us, "ratio": base / best_us})
        print(f"| {M} x {N} x {K} | {base_name} ({base_split}) | {base:.1f} | {best_label} | {best_us:.1f} | "
              f"{base / best_us:.3f} |", file=out, flush=True)
        del A, B, C
    return rows


def random_shapes(seed: int, count: int) -> List[Tuple[int, int, int]]:
    """Seeded (M, N, K) with extents log-uniform in 32 .. 8192 (K from 64), a fifth each multiples of
    128, of 64, of 1 (unaligned rows) and two fifths of 4; at most 2.5e11 multiply-adds and 6e7 outputs."""
    import math
    import random
    rnd = random.Random(seed)

    def extent(lo, hi, align):
        v = int(math.exp(rnd.uniform(math.log(lo), math.log(hi))))
        return max(align, v // align * align)

    shapes = []
    while len(shapes) < count:
        a = rnd.choice([128, 64, 4, 4, 1])
        M, N, K = extent(32, 8192, a), extent(32, 8192, a), extent(64, 8192, 4 if a != 1 else 1)
        if M * N * K <= 2.5e11 and M * N <= 6e7:
            shapes.append((M, N, K))
    return shapes


def random_skinny_shapes(seed: int, count: int) -> List[Tuple[int, int, int]]:
    """Seeded (M, N, K) with one side of C of 1 .. 32 (rows or columns, half each; the columns a
    multiple of 4 half the time), the other side log-uniform in 256 .. 200000 and K in 16 .. 8192,
    both multiples of 4; the large operand between 2e5 and 1.2e8 elements."""
    import math
    import random
    rnd = random.Random(seed)

    def extent(lo, hi, align=1):
        v = int(math.exp(rnd.uniform(math.log(lo), math.log(hi))))
        return max(align, v // align * align)

    shapes = []
    while len(shapes) < count:
        small, big, K = extent(1, 33), extent(256, 200000, 4), extent(16, 8192, 4)
        if not 2e5 <= big * K <= 1.2e8:
            continue
        if rnd.random() < 0.5:
            shapes.append((small, big, K))
        else:
            shapes.append((big, small if rnd.random() < 0.5 else max(4, small // 4 * 4), K))
    return shapes


def random_igemm_shapes(seed: int, count: int) -> List[Tuple[int, int, int]]:
    """Seeded (M, N, K) for the int8 product: extents log-uniform in 32 .. 8192 (K from 64), aligned to
    256, 128, 64, 16 (twice as often), 4 (twice as often) or not at all (then N is a multiple of 16 and
    K one half the time); at most 5e11 multiply-adds and 6e7 outputs."""
    import math
    import random
    rnd = random.Random(seed)

    def extent(lo, hi, align):
        v = int(math.exp(rnd.uniform(math.log(lo), math.log(hi))))
        return max(align, v // align * align)

    shapes = []
    while len(shapes) < count:
        a = rnd.choice([256, 128, 64, 16, 16, 4, 4, 1])
        M, N = extent(32, 8192, a), extent(32, 8192, a if a > 1 else 16)
        K = extent(64, 8192, min(a, 16) if a > 1 else rnd.choice([16, 1]))
        if M * N * K <= 5e11 and M * N <= 6e7:
            shapes.append((M, N, K))
    return shapes


def random_conv_shapes(seed: int, count: int) -> List[Tuple[int, ...]]:
    """Seeded layer shapes (N, H, W, C, K, R, S, stride, pad): batch 1 .. 64, square images of 7 .. 112,
    16 .. 512 channels (24, 40, 3 and 30 among the inputs), filters 1 x 1, 3 x 3 (three times as often) and
    5 x 5 with pad R / 2, stride 1 (twice as often) or 2; 2e7 .. 4e10 flop."""
    import random
    rnd = random.Random(seed)
    shapes = []
    while len(shapes) < count:
        N, HW = rnd.choice([1, 4, 8, 16, 32, 64]), rnd.choice([7, 14, 28, 56, 112])
        C = rnd.choice([16, 32, 48, 64, 96, 128, 192, 256, 512, 24, 40, 3, 30])
        K, R, stride = rnd.choice([16, 32, 64, 96, 128, 256, 512]), rnd.choice([1, 3, 3, 3, 5]), rnd.choice([1, 1, 2])
        pad = R // 2
        P = (HW + 2 * pad - R) // stride + 1
        flops = 2.0 * N * P * P * K * R * R * C
        if 2e7 <= flops <= 4e10 and N * HW * HW * C * 4 <= 5e8:
            shapes.append((N, HW, HW, C, K, R, R, stride, pad))
    return shapes


def _timed_us(torch, run, min_ms):
    run()
    torch.cuda.synchronize()
    t0, n = time.perf_counter(), 0
    while (time.perf_counter() - t0) * 1e3 < min_ms:
        for _ in range(10):
            run()
        torch.cuda.synchronize()
        n += 10
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n):
        run()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def igemm_choice_table(shapes, min_ms: float = 4.0) -> List[Dict]:
    """igemm_s8s32: the library's own choice against every kernel variant forced in turn with the
    reduction cut by the library (0), whole (1), in 2 and in 4."""
    import torch
    from . import binding as b
    b.use_torch_stream()
    names = b.igemm_variant_names()
    rows = []
    for M, N, K in shapes:
        A = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
        B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device="cuda")
        C = torch.zeros(M, N, dtype=torch.int32, device="cuda")
        run = lambda: b.igemm_s8s32_t(A, B, C)
        b.set_igemm_tuning(-1)
        b.set_tuning(-1, 0)
        base = min(_timed_us(torch, run, min_ms) for _ in range(2))
        base_name = b.last_variant()
        best_us, best_label = float("inf"), ""
        for i, n in enumerate(names):
            for split in (0, 1, 2, 4):
                b.set_igemm_tuning(i)
                b.set_tuning(-1, split)
                run()
                if b.last_variant() != n:
                    break  # the kernel does not take this shape
                us = _timed_us(torch, run, min_ms)
                if us < best_us:
                    best_us, best_label = us, f"{n} (cut {split})"
        b.set_igemm_tuning(-1)
        b.set_tuning(-1, 0)
        rows.append({"shape": (M, N, K), "builtin": base_name, "builtin_us": base, "best": best_label,
                     "best_us": best_us, "ratio": base / best_us})
        del A, B, C
    return rows


def conv_choice_table(shapes, min_ms: float = 4.0) -> List[Dict]:
    """conv2d_nhwc: the library's own choice against every kernel variant forced in turn, its last
    round of tiles as the library plans it (-1) or whole (0), its reduction cut by the library (0)
    or whole (1)."""
    import torch
    from . import binding as b
    b.use_torch_stream()
    names = b.conv_variant_names()
    rows = []
    for shape in shapes:
        N, H, W, C, K, R, S, stride, pad = shape
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        x = torch.rand(N, H, W, C, device="cuda")
        w = torch.randn(K, R, S, C, device="cuda") * 0.1
        out = torch.empty(N, P, Q, K, device="cuda")
        run = lambda: b.conv2d_nhwc_t(x, w, out, stride, pad)

        def settings(variant, tail, split):
            b.set_conv_tuning(variant)
            b.set_conv_tail(tail)
            b.set_conv_split(split)

        settings(-1, -1, 0)
        base = min(_timed_us(torch, run, min_ms) for _ in range(2))
        base_name = b.last_variant()
        best_us, best_label = float("inf"), ""
        for i in range(len(names)):
            for tail in (-1, 0):
                for split in (0, 1):
                    settings(i, tail, split)
                    us = _timed_us(torch, run, min_ms)
                    if us < best_us:
                        best_us, best_label = us, f"{b.last_variant()} (tail {tail}, cut {split})"
        settings(-1, -1, 0)
        rows.append({"shape": shape, "builtin": base_name, "builtin_us": base, "best": best_label,
                     "best_us": best_us, "ratio": base / best_us})
        del x, w, out
    return rows


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="op", required=True)
    p = sub.add_parser("sgemm")
    p.add_argument("dims", type=int, nargs=3, metavar=("M", "N", "K"))
    p.add_argument("--workspace", action="store_true", help="sweep sgemm_ws: slices meet in a workspace")
    p = sub.add_parser("igemm")
    p.add_argument("dims", type=int, nargs=3, metavar=("M", "N", "K"))
    p = sub.add_parser("table")
    p.add_argument("--random", type=int, nargs=2, metavar=("SEED", "COUNT"),
                   help="seeded random shapes instead of the fixed list, worst ratio first")
    p.add_argument("--of", dest="audited", choices=["sgemm", "igemm", "conv"], default="sgemm",
                   help="the operation whose choice is audited (igemm and conv: with --random only)")
    p.add_argument("--skinny", action="store_true", help="sgemm with --random: shapes with one side of C of 1 .. 32")
    p.add_argument("--grid", nargs=2, metavar=("EXTENTS", "REDUCTIONS"),
                   help="sgemm: every (M, N) from the comma-separated EXTENTS with every K from REDUCTIONS "
                        "(round shapes, whose tiles divide evenly among the CUs), worst ratio first")
    p.add_argument("--layout", choices=["nn", "nt", "tn", "tt"], default="nn",
                   help="sgemm with --random: operands stored transposed (sgemm_op)")
    p = sub.add_parser("conv")
    p.add_argument("dims", type=int, nargs=9, metavar=("N", "H", "W", "C", "K", "R", "S", "stride", "pad"))
    p = sub.add_parser("dwconv")
    p.add_argument("dims", type=int, nargs=8, metavar=("N", "H", "W", "C", "R", "S", "stride", "pad"))
    for name, q in sub.choices.items():
        if name != "table":
            q.add_argument("--builtin", type=int, default=0, metavar="CALLS",
                           help="time only the library's own choice, CALLS calls back to back")
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("tune: no GPU visible", file=sys.stderr)
        return 3
    if args.op == "table" and args.grid and not args.random:
        import io
        extents = [int(v) for v in args.grid[0].split(",")]
        shapes = [(m, n, k) for m in extents for n in extents for k in (int(v) for v in args.grid[1].split(","))
                  if 2.0 * m * n * k <= 3e11]
        if args.audited == "igemm":
            rows = igemm_choice_table(shapes)
        else:
            rows = choice_table(shapes, min_ms=4.0, out=io.StringIO(), layout=args.layout)
        print("| built-in / best | shape | built-in us, kernel | best forced us, kernel (settings) |")
        print("|---|---|---|---|")
        for r in sorted(rows, key=lambda r: -r["ratio"]):
            print(f"| {r['ratio']:.3f} | {' x '.join(str(v) for v in r['shape'])} | {r['builtin_us']:.1f} "
                  f"{r['builtin']} | {r['best_us']:.1f} {r['best']} |")
    elif args.op == "table" and args.random:
        import io
        if args.audited == "conv":
            rows = conv_choice_table(random_conv_shapes(*args.random))
        elif args.audited == "igemm":
            rows = igemm_choice_table(random_igemm_shapes(*args.random))
        else:
            shapes = random_skinny_shapes(*args.random) if args.skinny else random_shapes(*args.random)
            rows = choice_table(shapes, min_ms=4.0, out=io.StringIO(), layout=args.layout)
        print("| built-in / best | shape | built-in us, kernel | best forced us, kernel (settings) |")
        print("|---|---|---|---|")
        for r in sorted(rows, key=lambda r: -r["ratio"]):
            print(f"| {r['ratio']:.3f} | {' x '.join(str(v) for v in r['shape'])} | {r['builtin_us']:.1f} "
                  f"{r['builtin']} | {r['best_us']:.1f} {r['best']} |")
    elif args.op == "table":
        choice_table()
    elif args.builtin > 0:
        builtin_only(args.op, args.dims, args.builtin, getattr(args, "workspace", False))
    elif args.op == "sgemm":
        tune_sgemm(*args.dims, workspace=args.workspace)
    else:
        {"igemm": tune_igemm, "conv": tune_conv, "dwconv": tune_dwconv}[args.op](*args.dims)
    return 0


if __name__ == "__main__":
    sys.exit(main())
