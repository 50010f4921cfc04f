#!/usr/bin/env python3
"""Benchmark of librollattn on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME] [--no-cpu]

A step is one pass of the whole attention path over one synthetic batch that is already
resident in HBM: the device-side plan, the main kernel and (decode) the split-K merge.  The
headline workload is the mid-size bf16 decode batch; the long-tail decode, the
observation-append batch, the mixed FP8 rollout step and the KV-recomputation prefill (append
with an empty prefix over whole histories) and the KV write of the append chunks (bf16 and FP8
pools) and the decode step of grouped rollouts that share an 8k prompt (with the prompt read once
per group, and plain decode on the same aliased tables for comparison) are timed after it and
reported in the same JSON line under "workloads".  Every figure is throughput on ALGORITHMIC bytes /
flops (K and V of each KV head once per call, live page-table entries, page scales, Q in,
O out; 4*Hq*D flops per attended pair), never on what the kernels happen to move.

The "roofline" object is for the main kernel of the headline workload, timed with HIP events
that the library records around that kernel on the call's stream.  "cpu_baseline" is the
float64 oracle, untuned, on the host cores of the same box, on the same bytes.
"""
from __future__ import annotations

import argparse
import ctypes
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
HEADLINE = 2
# HBM bytes per launch of the headline workload's main kernel, from hardware counters (FETCH_SIZE and
# WRITE_SIZE, each scaled by its reading on a copy of known size; profiles/decode_mfma_c2_decode_bf16_b64.md
# has the commands and the raw readings).  Valid for the decode kernel as committed with that profile:
# set to None when the kernel changes, until the counters have been taken again.
HEADLINE_TRAFFIC_BYTES = {"decode_mfma_kernel": 814_387_200 + 5_121_024}


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
    """Wall time per step over exactly `steps` steps, then per-leg main-kernel time from HIP events."""
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
    kernel_ms = []
    for leg in legs:
        B.profile_enable(True)
        for _ in range(steps):
            leg.step()
        torch.cuda.synchronize()
        kernel_ms.append(B.profile_read())
        B.profile_enable(False)
    return ms_per_step, kernel_ms, graph_ms


def leg_report(leg, kms):
    if leg.kind in ("decode_shared", "step"):  # two main kernels per call (shared and private half; chunks and decode rows): their sum
        kms = np.asarray(kms)[: len(kms) // 2 * 2].reshape(-1, 2).sum(axis=1)
    avg = float(np.mean(kms))
    work = leg.work
    if leg.kind in ("decode", "kv_write", "decode_shared", "decode_aliased"):
        ach = work["bytes"] / avg / 1e6
        return {"kind": leg.kind, "bound": "hbm", "kernel_ms_avg": avg, "kernel_ms_min": float(np.min(kms)),
                "algorithmic_bytes": work["bytes"], "achieved": ach, "unit": "GB/s", "peak": HBM_PEAK_GBS,
                "frac": ach / HBM_PEAK_GBS}
    ach = work["flops"] / avg / 1e9
    return {"kind": leg.kind, "bound": "mfma", "kernel_ms_avg": avg, "kernel_ms_min": float(np.min(kms)),
            "algorithmic_flops": work["flops"], "algorithmic_bytes": work["bytes"], "achieved": ach,
            "unit": "TFLOP/s", "peak": MFMA_BF16_PEAK_TFLOPS, "frac": ach / MFMA_BF16_PEAK_TFLOPS}


def cpu_baseline(batch, W, budget_s=20.0):
    """The oracle as it stands, on the host cores, on the same stored bytes (headline workload)."""
    import torch
    from oracle import attention as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
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
    return {"value": work["bytes"] / dt / 1e9, "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} of {len(order)} trajectories of {w.name} ({int(batch.ctx_lens_host[rows].sum())} tokens), "
                      f"numpy float64 oracle, {dt:.1f} s", "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--only", default=None, help="run a single workload: c2, c3, c4, c5, c5_one_call, recompute, kv_write_c4, kv_write_c5, shared_prompt or shared_prompt_plain (or `copy`: 1 GiB copy for counter calibration)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
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
    extra = {"recompute": W.RECOMPUTE, "kv_write_c4": W.CONFIGS[4], "kv_write_c5": W.CONFIGS[5], "c5_one_call": W.CONFIGS[5],
             "shared_prompt": W.SHARED_PROMPT, "shared_prompt_plain": W.SHARED_PROMPT}
    if a.only:
        selected = [a.only] if a.only in extra else [int(a.only.lstrip("c"))]
    else:
        selected = [HEADLINE, 3, 4, 5, "c5_one_call", "recompute", "kv_write_c4", "kv_write_c5", "shared_prompt", "shared_prompt_plain"]
    reports = {}
    headline = None
    cpu = None
    for c in selected:
        w = extra[c] if c in extra else W.CONFIGS[c]
        batch = W.build(w, dev)
        small = W.algorithmic_work(w, batch.ctx_lens_host, batch.q_lens_host)["kv_bytes"] < 2e9
        legs = [Leg(kind, bb, B, W, n_pools=3 if small else 1) for kind, bb in _parts(batch, c, W)]
        steps = a.steps if c == selected[0] else max(5, min(a.steps, 20))
        ms, kms, gms = time_legs(legs, steps, a.warmup, B)
        rep = {"ms_per_step": ms, "graph_ms_per_step": gms, "steps": steps, "legs": [leg_report(l, k) for l, k in zip(legs, kms)],
               "batch": w.batch, "heads": [w.num_q_heads, w.num_kv_heads, w.head_dim], "kv_dtype": w.kv_dtype,
               "tokens": int(batch.ctx_lens_host.sum()), "query_rows": int(batch.q_lens_host.sum())}
        reports[c if isinstance(c, str) and c != "recompute" else w.name] = rep
        if c == selected[0]:
            headline = (w, rep, legs)
            if not a.no_cpu and c in (2, 3):
                cpu = cpu_baseline(batch, W)
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
    line = {
        "metric": METRIC, "value": value, "unit": unit, "n_gpus": 1, "steps": rep["steps"], "warmup": a.warmup,
        "ms_per_step": rep["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "num_q_heads": w.num_q_heads, "num_kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "page_size": 16, "kv_dtype": w.kv_dtype, "tokens": rep["tokens"]},
        "roofline": {"bound": lead["bound"], "achieved": lead["achieved"], "peak": lead["peak"], "unit": lead["unit"],
                     "frac": lead["frac"],
                     "traffic": HEADLINE_TRAFFIC_BYTES.get("decode_mfma_kernel") if (lead["kind"] == "decode" and w is W.CONFIGS[HEADLINE]) else None,
                     "kernel": "decode_mfma_kernel" if lead["kind"] == "decode" else "append_mfma_kernel",
                     "kernel_ms_avg": lead["kernel_ms_avg"]},
        "cpu_baseline": cpu,
        "workloads": reports,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
