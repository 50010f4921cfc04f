"""Builds librollattn.so (gfx950) from csrc/ with hipcc, in-tree, and libbench_peaks.so (bench.py's peak microbenchmarks)."""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librollattn.so")
PEAKS_LIB = os.path.join(HERE, "libbench_peaks.so")      # the benchmark's two peak microbenchmarks, not part of the library
SOURCES = ["api.cpp", "plan.hip", "attn_f32.hip", "decode_mfma.hip", "combine.hip", "append_mfma.hip", "kv_write.hip", "shared_prefix.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


# Kernels that wait for their asynchronous loads by count: a register spill to scratch memory would use the same
# counter behind the compiler's back, so their build fails if the compiler reports any scratch.
NO_SCRATCH = {"append_mfma.hip"}


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, src + ".o")
    check = ["-Rpass-analysis=kernel-resource-usage"] if src in NO_SCRATCH else []
    cmd = ["hipcc", *FLAGS, *extra, *check, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if check and r.returncode == 0:
        sizes = [int(m) for m in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", r.stderr)]
        if not sizes or any(sizes):
            raise RuntimeError(f"{src}: a kernel uses scratch memory (bytes per lane: {sizes}); its counted waits assume none")
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "remark:" not in l)
    if r.returncode:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(extra_flags=(), verbose=False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stderr)
    # the benchmark's microbenchmarks (streaming read, MFMA loop): an object and a library of their own
    peaks_obj = _compile("bench_peaks.hip", list(extra_flags))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PEAKS_LIB, peaks_obj], capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB, "and", PEAKS_LIB)
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:], verbose=True)
