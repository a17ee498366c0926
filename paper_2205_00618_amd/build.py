"""Build liblsmi.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblsmi.so")
SOURCES = ["api.cpp", "sgemm_gfx950.hip", "sgemm_nt_gfx950.hip", "sgemm_tn_gfx950.hip", "sgemm_tt_gfx950.hip", "conv2d_gfx950.hip", "igemm_gfx950.hip", "dwconv2d_gfx950.hip", "copy_gfx950.hip", "diag_gfx950.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops is switched off for the device pass: the compiler then never fuses
# pairs of fp32 operations into packed instructions (the host pass does not know the
# feature and says so; that warning is harmless).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-Rpass-analysis=kernel-resource-usage"]  # per-kernel register and scratch report


def spilling_kernels(compiler_output: str):
    """(kernel, bytes per lane) for every kernel the resource report shows using scratch
    memory: a kernel of this library that spills registers is a performance bug."""
    bad, name = [], None
    for line in compiler_output.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[-Rpass")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[-Rpass")[0])
            if size:
                bad.append((name, size))
    return bad


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, "-x", "hip", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    spills = spilling_kernels(res.stdout)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "-Rpass-analysis=kernel-resource-usage" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if spills:
        raise RuntimeError(f"{src}: kernels spill registers to scratch memory: {spills}")
    if verbose and out.strip():
        print(out, flush=True)
    return obj


def build(verbose: bool = False, extra_flags=()) -> str:
    global FLAGS
    if extra_flags:
        FLAGS = FLAGS + list(extra_flags)
    with ThreadPoolExecutor(max_workers=6) as pool:
        objs = list(pool.map(lambda s: _compile(s, verbose), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
