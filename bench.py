#!/usr/bin/env python3
"""Benchmark of librollattn on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME] [--no-cpu]

A step is one pass of the whole attention path over one synthetic batch that is already
resident in HBM: the device-side plan, the main kernel and (decode) the split-K merge.  The
headline workload is the mid-size bf16 decode batch (the slowest of the decode workloads
relative to its roofline); the long-tail decode, the observation-append batch, the mixed FP8
rollout step, the KV-recomputation prefill (append with an empty prefix over whole histories),
the KV write of the append chunks (bf16 and FP8 pools) and the decode step of grouped rollouts
that share an 8k prompt (with the prompt read once per group, and plain decode on the same
aliased tables for comparison) are timed after it and reported in the same JSON line under
"workloads".  Every figure is throughput on ALGORITHMIC bytes / flops (K and V of each KV head
once per call, live page-table entries, page scales, Q in, O out; 4*Hq*D flops per attended
pair), never on what the kernels happen to move.

Timing.  `ms_per_step` is wall time over exactly --steps steps between two device
synchronisations.  A second pass of the same number of steps brackets every call with events on
the call's stream and lets the library bracket its main kernel: the per-leg kernel and
whole-call figures (mean, median, minimum) all come from that one pass.  Fractions are given
against the nominal peaks (HBM 8 TB/s, dense bf16 MFMA 2.5 PFLOP/s) and against what two
microbenchmarks of libbench_peaks.so reach on this GPU in this run (a streaming read of 4 GiB
and a register-resident MFMA loop).  Legs that run the MFMA append kernel also report the shader clock that kernel
got ("append_kernel_clock_mhz": cycles over ticks of the constant 100 MHz counter, summed inside its tiles by the
library while profiling is on) and their fraction of the peak at that clock: the part runs these kernels at its
power limit, well below the 2.4 GHz that the nominal peak assumes.

The "roofline" object is for the main kernel of the headline workload.  "cpu_baseline" is the
float64 oracle, untuned, on the host cores of the same box, on the same bytes;
"cpu_baseline_append" is the same for a bounded sample of the append workload.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "decode-attn achieved HBM GB/s (% of peak) + append TFLOP/s, ragged paged KV"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
NOMINAL_CLOCK_MHZ = 2400.0      # the clock that peak is quoted at
HEADLINE = 2
# HBM bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by its
# reading on a copy of known size).  They cannot be taken inside this program; profiles/hbm_traffic.json keeps
# them together with the hashes of the kernel sources they were taken with, and a figure is reported only while
# those sources are unchanged.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
CSRC = os.path.join(ROOT, "paper_2512_22560_amd", "csrc")
MAIN_KERNEL_SOURCES = {"decode": ["decode_mfma.hip", "rollattn_internal.h"], "append": ["append_mfma.hip", "rollattn_internal.h"]}


def source_hash(files):
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def counter_traffic(workload_name, kind):
    """HBM bytes per launch of this workload's main kernel from the committed counter readings, or None when there
    are none or the kernel's sources have changed since they were taken."""
    try:
        with open(TRAFFIC_FILE) as fh:
            table = json.load(fh)
    except (OSError, ValueError):
        return None
    entry = table.get(f"{workload_name}:{kind}")
    if not entry or kind not in MAIN_KERNEL_SOURCES:
        return None
    if entry.get("source_hash") != source_hash(MAIN_KERNEL_SOURCES[kind]):
        return None
    return int(entry["fetch_bytes"]) + int(entry["write_bytes"])


def _parts(batch, c, W):
    """(kind, sub-batch) legs of one step of configuration c."""
    if c in (2, 3):
        return [("decode", batch)]
    if c in (4, "recompute"):
        return [("append", batch)]
    if c == "kv_write_c4":
        return [("kv_write", batch)]
    if c in ("shared_prompt", "shared_prompt_plain"):
        n_groups = batch.workload.batch // W.SHARED_PROMPT_GROUP
        aliased = W.alias_shared_prefix(batch, W.SHARED_PROMPT_GROUP, np.full(n_groups, W.SHARED_PROMPT_TOKENS))
        return [("decode_shared" if c == "shared_prompt" else "decode_aliased", aliased)]
    if c == "kv_write_c5":
        return [("kv_write", batch.select(batch.append_rows()))]
    if c == "c5_one_call":
        return [("step", batch)]                     # the mixed batch as it is: the library tells the two kinds apart
    return [("decode", batch.select(batch.decode_rows())), ("append", batch.select(batch.append_rows()))]


class Leg:
    """One entry point on one sub-batch, with preallocated output and workspace."""

    def __init__(self, kind, bb, B, W, n_pools=1):
        import torch
        self.kind, self.bb, self.B = kind, bb, B
        self.group_size = W.SHARED_PROMPT_GROUP
        w = bb.workload
        self.w = w
        self.work = W.algorithmic_work(w, bb.ctx_lens_host, bb.q_lens_host)
        desc = B.make_desc(bb.q, bb.k_pages, bb.page_table, sm_scale=w.sm_scale, k_scale=bb.k_scale, v_scale=bb.v_scale)
        self.ws = B.alloc_workspace(desc, bb.total_q, bb.q.device)
        self.out = torch.empty_like(bb.q)
        self.max_q = int(max(1, bb.q_lens_host.max(initial=1)))
        if kind == "decode_shared":
            n_groups = w.batch // W.SHARED_PROMPT_GROUP
            self.shared_lens = torch.full((n_groups,), W.SHARED_PROMPT_TOKENS, dtype=torch.int32, device=bb.q.device)
            self.ws = torch.empty(int(B.lib().rollattn_shared_workspace_bytes(ctypes.byref(desc), W.SHARED_PROMPT_GROUP)),
                                  dtype=torch.uint8, device=bb.q.device)
        if kind == "step":
            self.ws = torch.empty(int(B.lib().rollattn_step_workspace_bytes(ctypes.byref(desc), bb.total_q)),
                                  dtype=torch.uint8, device=bb.q.device)
        if kind in ("decode_shared", "decode_aliased"):
            # bytes that have to move when every physical page is read once: the prompts per group, the rest per trajectory
            kvb = {"f32": 4, "bf16": 2, "fp8_e4m3": 1}[w.kv_dtype]
            n_groups = w.batch // W.SHARED_PROMPT_GROUP
            uniq = n_groups * W.SHARED_PROMPT_TOKENS + int((bb.ctx_lens_host - W.SHARED_PROMPT_TOKENS).sum())
            pages = n_groups * (W.SHARED_PROMPT_TOKENS // 16) + int(((bb.ctx_lens_host - W.SHARED_PROMPT_TOKENS + 15) // 16).sum())
            self.work = {"bytes": int(2 * w.num_kv_heads * w.head_dim * kvb * uniq + pages * (4 + (8 if kvb == 1 else 0))
                                      + 2 * bb.total_q * w.num_q_heads * w.head_dim * 2), "flops": 0}
        if kind == "kv_write":
            # new K / V rows for the chunk region of the cache; unit-scale values as everywhere else
            g = torch.Generator(device=bb.q.device).manual_seed(w.seed)
            shape = (bb.total_q, w.num_kv_heads, w.head_dim)
            self.k_new = torch.randn(shape, generator=g, device=bb.q.device, dtype=torch.float32).to(bb.q.dtype)
            self.v_new = torch.randn(shape, generator=g, device=bb.q.device, dtype=torch.float32).to(bb.q.dtype)
            kvb = {"f32": 4, "bf16": 2, "fp8_e4m3": 1}[w.kv_dtype]
            srcb = {"f32": 4, "bf16": 2}[w.q_dtype]
            first = bb.ctx_lens_host - bb.q_lens_host
            pages = np.where(bb.q_lens_host > 0, (bb.ctx_lens_host + 15) // 16 - first // 16, 0).sum()
            rows = int(bb.q_lens_host.sum()) * w.num_kv_heads * w.head_dim
            # rows read once and written once per pool, one table entry per touched page, FP8: its two scales read and written
            self.work = {"bytes": int(2 * rows * (srcb + kvb) + 4 * pages + (16 * pages if w.kv_dtype == "fp8_e4m3" else 0)), "flops": 0}
        # Rotating copies of the pools keep the 256 MB last-level cache from serving a small KV set.
        self.pools = [(bb.k_pages, bb.v_pages)]
        for _ in range(n_pools - 1):
            self.pools.append((bb.k_pages.clone(), bb.v_pages.clone()))
        self.i = 0

    def step(self):
        bb, w, B = self.bb, self.w, self.B
        k, v = self.pools[self.i % len(self.pools)]
        self.i += 1
        if self.kind == "decode_shared":
            B.attn_decode_shared(bb.q, k, v, bb.page_table, bb.ctx_lens, group_size=self.group_size,
                                 shared_lens=self.shared_lens, sm_scale=w.sm_scale, k_scale=bb.k_scale, v_scale=bb.v_scale,
                                 out=self.out, workspace=self.ws)
        elif self.kind == "kv_write":
            B.kv_write(self.k_new, self.v_new, bb.q_lens, bb.q_offsets, k, v, bb.page_table, bb.ctx_lens, max_q_len=self.max_q,
                       k_scale=bb.k_scale, v_scale=bb.v_scale)
        elif self.kind == "step":
            B.attn_step(bb.q, bb.q_lens, bb.q_offsets, k, v, bb.page_table, bb.ctx_lens, sm_scale=w.sm_scale,
                        max_q_len=self.max_q, k_scale=bb.k_scale, v_scale=bb.v_scale, out=self.out, workspace=self.ws)
        elif self.kind in ("decode", "decode_aliased"):
            B.attn_decode(bb.q, k, v, bb.page_table, bb.ctx_lens, sm_scale=w.sm_scale, k_scale=bb.k_scale,
                          v_scale=bb.v_scale, out=self.out, workspace=self.ws)
        else:
            B.attn_append(bb.q, bb.q_lens, bb.q_offsets, k, v, bb.page_table, bb.ctx_lens, sm_scale=w.sm_scale,
                          max_q_len=self.max_q, k_scale=bb.k_scale, v_scale=bb.v_scale, out=self.out,
                          workspace=self.ws)


def time_legs(legs, steps, warmup, B):
    """ms per step (wall, over exactly `steps` steps), the same through a HIP graph, then one more pass of `steps`
    steps in which every call is bracketed by events on its stream and the library brackets its main kernel:
    per leg (kernel ms per call [steps], whole-call ms per call [steps])."""
    import torch
    for _ in range(warmup):
        for leg in legs:
            leg.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for leg in legs:
            leg.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    # the same step captured once in a HIP graph and replayed (every entry point plans on the device and
    # neither allocates nor synchronises): one graph holds as many steps as there are rotating pools
    per_graph = max(len(leg.pools) for leg in legs)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for leg in legs:
                leg.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for leg in legs:
            leg.i = 0
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(per_graph):
                for leg in legs:
                    leg.step()
        torch.cuda.synchronize()
        replays = max(1, steps // per_graph)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / (replays * per_graph) * 1e3
        del graph
    except Exception as e:      # reported, never fatal: the eager figures above are the contract
        print(f"bench.py: graph replay skipped: {e}", file=sys.stderr)
    # the profiled pass: kernel and whole-call durations of the same calls
    B.profile_enable(True)
    B.profile_read()
    marks = [[] for _ in legs]
    for _ in range(steps):
        for li, leg in enumerate(legs):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            leg.step()
            b.record()
            marks[li].append((a, b))
    torch.cuda.synchronize()
    kernel_all = B.profile_read()
    append_clock = B.profile_append_clock()     # MHz over this pass's MFMA append launches, 0.0 without any
    B.profile_enable(False)
    per_step = sum(2 if leg.kind in ("decode_shared", "step") else 1 for leg in legs)   # main kernels per step, in launch order
    kernel_all = np.asarray(kernel_all[: len(kernel_all) // per_step * per_step]).reshape(-1, per_step)
    out, col = [], 0
    for li, leg in enumerate(legs):
        n = 2 if leg.kind in ("decode_shared", "step") else 1   # two main kernels per call (shared and private half; chunks and decode rows): their sum
        kms = kernel_all[:, col:col + n].sum(axis=1)
        col += n
        call = np.asarray([a.elapsed_time(b) for a, b in marks[li]])
        out.append((kms, call))
    return ms_per_step, out, graph_ms, append_clock


def _stats(x):
    return {"avg": float(np.mean(x)), "median": float(np.median(x)), "min": float(np.min(x))}


def leg_report(leg, kms, call_ms, peaks, step_ms=None):
    """step_ms: wall time per step of a workload with this one leg (then the whole-call figure is taken from it:
    the events around a call cost a few microseconds themselves, which matters for the short decode calls)."""
    k, c = _stats(kms), _stats(call_ms)
    work = leg.work
    hbm = leg.kind in ("decode", "kv_write", "decode_shared", "decode_aliased")
    amount = work["bytes"] if hbm else work["flops"]
    unit, peak, scale = ("GB/s", HBM_PEAK_GBS, 1e6) if hbm else ("TFLOP/s", MFMA_BF16_PEAK_TFLOPS, 1e9)
    ach = amount / k["avg"] / scale
    rep = {"kind": leg.kind, "bound": "hbm" if hbm else "mfma",
           "kernel_ms_avg": k["avg"], "kernel_ms_median": k["median"], "kernel_ms_min": k["min"],
           "call_ms_avg": c["avg"], "call_ms_median": c["median"], "call_ms_min": c["min"],
           "algorithmic_bytes": work["bytes"], "achieved": ach, "unit": unit, "peak": peak, "frac": ach / peak,
           "achieved_median": amount / k["median"] / scale, "frac_median": amount / k["median"] / scale / peak,
           # the whole call (plan + main kernel + merge), from the events around it in the same pass
           "call_achieved": amount / (step_ms or c["avg"]) / scale, "call_frac": amount / (step_ms or c["avg"]) / scale / peak,
           "call_frac_from": "wall time per step" if step_ms else "events around the call"}
    if not hbm:
        rep["algorithmic_flops"] = work["flops"]
    measured = (peaks or {}).get("hbm_read_GBs" if hbm else "mfma_bf16_TFLOPs")
    if measured:
        rep["frac_of_measured_peak"] = ach / measured
    return rep


def measure_peaks(dev):
    """What this GPU delivers at best in this run: a streaming read of 4 GiB, and a register-resident loop of the
    append kernel's matrix instruction.  Both kernels live in libbench_peaks.so, outside the library."""
    import torch
    from paper_2512_22560_amd import build as lib_build
    if not os.path.exists(lib_build.PEAKS_LIB):
        return None
    lib = ctypes.CDLL(lib_build.PEAKS_LIB)
    vp = ctypes.c_void_p
    lib.peaks_stream_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_float), vp]
    lib.peaks_mfma_bf16.argtypes = [ctypes.c_int, vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double), vp]
    nbytes = 4 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    buf.view(torch.int32).random_(0, 1 << 30)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ms = ctypes.c_float(0)
    rc = lib.peaks_stream_read(vp(buf.data_ptr()), nbytes, 5, vp(sink.data_ptr()), ctypes.byref(ms), stream)
    if rc:
        raise RuntimeError(f"peaks_stream_read: HIP error {rc}")
    read_gbs = nbytes / ms.value / 1e6
    flops = ctypes.c_double(0)
    rc = lib.peaks_mfma_bf16(20000, vp(sink.data_ptr()), ctypes.byref(ms), ctypes.byref(flops), stream)
    if rc:
        raise RuntimeError(f"peaks_mfma_bf16: HIP error {rc}")
    del buf
    torch.cuda.empty_cache()
    return {"hbm_read_GBs": read_gbs, "hbm_read_frac_of_nominal": read_gbs / HBM_PEAK_GBS,
            "mfma_bf16_TFLOPs": flops.value / ms.value / 1e9, "mfma_bf16_frac_of_nominal": flops.value / ms.value / 1e9 / MFMA_BF16_PEAK_TFLOPS,
            "how": "streaming read of 4 GiB (16-byte loads, 5 passes); v_mfma_f32_32x32x16_bf16 on register operands, 8 waves per CU x 4 chains"}


def _blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(batch, W, budget_s=15.0):
    """The oracle as it stands, on the host cores, on the same stored bytes (decode workload)."""
    from oracle import attention as O
    threads = _blas_threads()
    w = batch.workload
    args = dict(k_pages=W.raw_numpy(batch.k_pages), v_pages=W.raw_numpy(batch.v_pages),
                page_table=W.raw_numpy(batch.page_table), sm_scale=w.sm_scale, q_dtype=w.q_dtype,
                kv_dtype=w.kv_dtype, k_scale=W.raw_numpy(batch.k_scale), v_scale=W.raw_numpy(batch.v_scale))
    q = W.raw_numpy(batch.q)
    # probe on two rows, then take as many whole trajectories as fit the time budget
    order = np.random.default_rng(0).permutation(len(batch.ctx_lens_host))
    t0 = time.perf_counter()
    O.attn_decode(q[order[:2]], **dict(args, page_table=args["page_table"][order[:2]], ctx_lens=batch.ctx_lens_host[order[:2]]))
    probe = time.perf_counter() - t0
    per_tok = probe / max(1, int(batch.ctx_lens_host[order[:2]].sum()))
    csum = np.cumsum(batch.ctx_lens_host[order])
    n = int(max(2, min(len(order), np.searchsorted(csum, budget_s / per_tok) + 1)))
    rows = np.sort(order[:n])
    t0 = time.perf_counter()
    O.attn_decode(q[rows], **dict(args, page_table=args["page_table"][rows], ctx_lens=batch.ctx_lens_host[rows]))
    dt = time.perf_counter() - t0
    work = W.algorithmic_work(w, batch.ctx_lens_host[rows], np.ones(n, dtype=np.int64))
    return {"value": work["bytes"] / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {len(order)} trajectories of {w.name} ({int(batch.ctx_lens_host[rows].sum())} tokens), "
                      f"numpy float64 oracle, {dt:.1f} s", "seconds": dt}


def cpu_baseline_append(batch, W, budget_s=15.0):
    """The oracle on a bounded, seeded sample of an append workload's trajectories (the shortest context, then
    random ones while the budget lasts); the time for the whole batch is extrapolated by attended pairs."""
    from oracle import attention as O
    threads = _blas_threads()
    w = batch.workload

    def pairs(rows):
        n, L = batch.q_lens_host[rows].astype(np.int64), batch.ctx_lens_host[rows].astype(np.int64)
        return int((n * (L - n) + n * (n + 1) // 2).sum())

    def run(rows):
        sub = batch.select(np.asarray(rows))
        t0 = time.perf_counter()
        O.attn_append(W.raw_numpy(sub.q), sub.q_lens_host, k_pages=W.raw_numpy(sub.k_pages), v_pages=W.raw_numpy(sub.v_pages),
                      page_table=W.raw_numpy(sub.page_table), ctx_lens=sub.ctx_lens_host, sm_scale=w.sm_scale, q_dtype=w.q_dtype,
                      kv_dtype=w.kv_dtype, k_scale=W.raw_numpy(sub.k_scale), v_scale=W.raw_numpy(sub.v_scale))
        return time.perf_counter() - t0

    cost = batch.q_lens_host * batch.ctx_lens_host
    cheapest = int(np.argmin(np.where(batch.q_lens_host > 0, cost, cost.max() + 1)))
    probe = run([cheapest])
    rate = pairs([cheapest]) / max(probe, 1e-6)                      # attended pairs per second, first estimate
    order = [r for r in np.random.default_rng(0).permutation(len(cost)).tolist() if r != cheapest and batch.q_lens_host[r] > 0]
    rows, dt = [cheapest], probe
    for _ in range(2):                           # the first estimate comes from a small problem and is pessimistic: refine once
        spent = 0.0
        rows = [cheapest]
        for r in order:
            t = pairs([r]) / rate
            if spent + t <= budget_s:
                rows.append(r)
                spent += t
        rows = sorted(rows)
        dt = run(rows)
        if dt > 0.6 * budget_s:
            break
        rate = pairs(rows) / max(dt, 1e-6)
    all_rows = np.arange(len(cost))
    flops = 4 * w.num_q_heads * w.head_dim * pairs(rows)
    return {"value": flops / dt / 1e9, "unit": "GFLOP/s", "cores": threads, "kind": "oracle", "extrapolated": True,
            "sample": f"{len(rows)} of {len(cost)} trajectories of {w.name} ({pairs(rows)} of {pairs(all_rows)} attended pairs), "
                      f"numpy float64 oracle, {dt:.1f} s; whole batch extrapolated by attended pairs",
            "seconds": dt, "seconds_whole_batch_extrapolated": dt * pairs(all_rows) / max(1, pairs(rows))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--only", default=None, help="run a single workload: c2, c3, c4, c5, c5_one_call, recompute, kv_write_c4, kv_write_c5, shared_prompt or shared_prompt_plain; `peaks`: the two peak microbenchmarks alone; `copy`: 1 GiB copy for counter calibration")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baselines")
    ap.add_argument("--no-peaks", action="store_true", help="skip the peak microbenchmarks")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this library runs on one GPU; nothing here shards or communicates, so --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_22560_amd import binding as B
    from paper_2512_22560_amd import workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(B.LIB_PATH):      # fresh checkout: build once; what is built is used as it is
        import __graft_entry__
        __graft_entry__.build()
    B.lib()   # fails loudly if the HIP library still is not there
    dev = "cuda:0"

    if a.only == "copy":
        # counter calibration: a plain device-to-device copy of known size (1 GiB read, 1 GiB written)
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(max(1, a.steps)):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "copy", "bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": max(1, a.steps)}))
        return
    peaks = None if a.no_peaks else measure_peaks(dev)
    if a.only == "peaks":
        print(json.dumps({"measured_peaks": peaks}))
        return
    extra = {"recompute": W.RECOMPUTE, "kv_write_c4": W.CONFIGS[4], "kv_write_c5": W.CONFIGS[5], "c5_one_call": W.CONFIGS[5],
             "shared_prompt": W.SHARED_PROMPT, "shared_prompt_plain": W.SHARED_PROMPT}
    if a.only:
        selected = [a.only] if a.only in extra else [int(a.only.lstrip("c"))]
    else:
        selected = [HEADLINE, 3, 4, 5, "c5_one_call", "recompute", "kv_write_c4", "kv_write_c5", "shared_prompt", "shared_prompt_plain"]
    reports = {}
    headline = None
    cpu = cpu_app = None
    for c in selected:
        w = extra[c] if c in extra else W.CONFIGS[c]
        batch = W.build(w, dev)
        small = W.algorithmic_work(w, batch.ctx_lens_host, batch.q_lens_host)["kv_bytes"] < 2e9
        legs = [Leg(kind, bb, B, W, n_pools=3 if small else 1) for kind, bb in _parts(batch, c, W)]
        ms, timed, gms, append_clock = time_legs(legs, a.steps, a.warmup, B)
        leg_reps = [leg_report(l, k, call, peaks, ms if len(legs) == 1 else None) for l, (k, call) in zip(legs, timed)]
        for l, r in zip(legs, leg_reps):
            if r["kind"] in MAIN_KERNEL_SOURCES:
                r["hbm_traffic_bytes"] = counter_traffic(w.name, r["kind"])
            if append_clock and r["kind"] in ("append", "step", "decode_shared"):
                # the clock the MFMA append kernel got in the profiled pass (counted inside its tiles); at a lower
                # clock than the nominal one the nominal peak is out of reach by that factor
                r["append_kernel_clock_mhz"] = append_clock
                if r["bound"] == "mfma":
                    r["frac_of_peak_at_that_clock"] = r["frac"] * NOMINAL_CLOCK_MHZ / append_clock
        rep = {"ms_per_step": ms, "graph_ms_per_step": gms, "steps": a.steps, "legs": leg_reps,
               "batch": w.batch, "heads": [w.num_q_heads, w.num_kv_heads, w.head_dim], "kv_dtype": w.kv_dtype,
               "tokens": int(batch.ctx_lens_host.sum()), "query_rows": int(batch.q_lens_host.sum())}
        reports[c if isinstance(c, str) and c != "recompute" else w.name] = rep
        if c == selected[0]:
            headline = (w, rep, legs)
            if not a.no_cpu and c in (2, 3):
                cpu = cpu_baseline(batch, W)
        if c == 4 and not a.no_cpu:
            cpu_app = cpu_baseline_append(batch, W)
        del legs, batch
        torch.cuda.empty_cache()

    w, rep, legs = headline
    lead = rep["legs"][0]
    if lead["kind"] == "decode":
        value = legs[0].work["bytes"] / rep["ms_per_step"] / 1e6      # whole step: plan + main + merge
        unit = "GB/s"
    else:
        value = legs[0].work["flops"] / rep["ms_per_step"] / 1e9
        unit = "TFLOP/s"
    # the bar of the four benchmark configurations: decode legs against HBM, append legs against bf16 MFMA, kernel and whole call
    targets = {}
    for name, r in reports.items():
        if name in ("c5_one_call",) or name.startswith(("kv_write", "shared_prompt", "recompute")):
            continue
        for l in r["legs"]:
            targets[f"{name}:{l['kind']}"] = {"frac": l["frac"], "call_frac": l["call_frac"], "bar": 0.70 if l["bound"] == "hbm" else 0.50}
    line = {
        "metric": METRIC, "value": value, "unit": unit, "n_gpus": 1, "steps": rep["steps"], "warmup": a.warmup,
        "ms_per_step": rep["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "num_q_heads": w.num_q_heads, "num_kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "page_size": 16, "kv_dtype": w.kv_dtype, "tokens": rep["tokens"]},
        "roofline": {"bound": lead["bound"], "achieved": lead["achieved"], "peak": lead["peak"], "unit": lead["unit"],
                     "frac": lead["frac"], "traffic": lead.get("hbm_traffic_bytes"),
                     "kernel": "decode_mfma_kernel" if lead["kind"] == "decode" else "append_mfma_kernel",
                     "kernel_ms_avg": lead["kernel_ms_avg"], "kernel_ms_median": lead["kernel_ms_median"],
                     "frac_of_measured_peak": lead.get("frac_of_measured_peak")},
        "cpu_baseline": cpu,
        "cpu_baseline_append": cpu_app,
        "measured_peaks": peaks,
        "targets": targets,
        "workloads": reports,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
