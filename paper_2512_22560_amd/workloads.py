"""Seeded synthetic rollout batches: ragged multi-turn contexts over a paged KV cache.

This module only lays out inputs (lengths, page tables, random values, storage
formats).  It contains none of the attention arithmetic and imports neither the
HIP binding nor the CPU oracle; tests and the benchmark hand its output to both.

Shapes follow the workload the paper describes for agentic rollouts: contexts up to
32k tokens in the evaluation and tens of thousands in production, long-tailed
lengths whose maximum is several times the mean, a batch of 512 trajectories, and
turns that append an observation chunk to a cached history (Section 7.1 "Evaluation
Setup", Section 8 production statistics, Section 2.1 on multi-turn trajectories).
Values are i.i.d. N(0,1): attention cost depends on shapes and lengths only.

Recipe (all integers from numpy's PCG64 `default_rng(seed)`, drawn in this order:
context lengths, chunk lengths, which rows are append rows, physical page
permutation; values from a torch.Generator seeded with the same seed, filled in the
order Q, K pool, V pool):
  * pool size = sum_b ceil(L_b / page_size); one random permutation of the pool is
    dealt to the trajectories in logical order;
  * unused page-table entries are -1; unused slots of each trajectory's last page
    hold NaN (0x7F, the NaN code, for FP8) so that any read of them shows up;
  * FP8 pools: per physical page and per pool, scale = absmax over the live slots
    / 448 (1.0 for an all-zero page), codes = round-to-nearest-even of x / scale.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import numpy as np
import torch

PAGE_SIZE = 16
BASE_SEED = 251222560

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic configuration.  `ctx` / `qlen` are (kind, *params) tuples:
    ("uniform", lo, hi) inclusive integers; ("loguniform", lo, hi) floor(exp(U));
    ("lognormal", median, sigma, lo, hi) rint(median * exp(sigma N)) clipped;
    ("const", v)."""
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    q_dtype: str
    kv_dtype: str
    ctx: tuple
    qlen: tuple = ("const", 1)
    append_rows: Optional[int] = None      # None: every row has qlen drawn from `qlen`
    ctx_is_prefix: bool = False            # True: L_b = drawn context + n_b on append rows
    seed: int = BASE_SEED

    @property
    def sm_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


K = 1024
CONFIGS = {
    1: Workload("c1_tiny_decode_f32", 4, 8, 2, 64, "f32", "f32", ("uniform", 32, 256), seed=BASE_SEED + 1),
    2: Workload("c2_decode_bf16_b64", 64, 32, 8, 128, "bf16", "bf16", ("loguniform", 512, 8192), seed=BASE_SEED + 2),
    3: Workload("c3_longtail_decode_bf16_b256", 256, 64, 8, 128, "bf16", "bf16",
                ("lognormal", 6 * K, 0.8, 1 * K, 32 * K), seed=BASE_SEED + 3),
    4: Workload("c4_append_bf16_b64", 64, 32, 8, 128, "bf16", "bf16", ("uniform", 2 * K, 16 * K),
                qlen=("uniform", 64, 1024), ctx_is_prefix=True, seed=BASE_SEED + 4),
    5: Workload("c5_mixed_fp8_b512", 512, 64, 4, 128, "bf16", "fp8_e4m3",
                ("lognormal", 8 * K, 0.8, 256, 64 * K), qlen=("uniform", 32, 512), append_rows=128,
                ctx_is_prefix=True, seed=BASE_SEED + 5),
}


# KV recomputation after a weight update (Section 6.2, protocol step 5): every in-flight trajectory's
# whole history is prefilled again, i.e. an append step with an empty prefix.  Lengths as in config 2.
RECOMPUTE = Workload("recompute_bf16_b64", 64, 32, 8, 128, "bf16", "bf16", ("const", 0),
                     qlen=("loguniform", 512, 8192), ctx_is_prefix=True, seed=BASE_SEED + 6)


# Early turns of grouped rollouts (Section 7.1: batch 512 in groups of 8 per prompt, prefix caching on):
# the 8 members of a group share an 8k-token prompt and have generated 32 .. 1024 tokens of their own.
SHARED_PROMPT = Workload("shared_prompt_fp8_b512", 512, 64, 4, 128, "bf16", "fp8_e4m3",
                         ("uniform", 8 * K + 32, 8 * K + 1024), seed=BASE_SEED + 7)
SHARED_PROMPT_GROUP = 8
SHARED_PROMPT_TOKENS = 8 * K


def scaled(w: Workload, *, batch=None, ctx=None, qlen=None, append_rows=None, name=None, seed=None,
           num_q_heads=None, num_kv_heads=None, head_dim=None, q_dtype=None, kv_dtype=None) -> Workload:
    """A reduced (or otherwise altered) copy of a configuration for parity tests."""
    kw = {k: v for k, v in dict(batch=batch, ctx=ctx, qlen=qlen, append_rows=append_rows, name=name,
                                seed=seed, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads,
                                head_dim=head_dim, q_dtype=q_dtype, kv_dtype=kv_dtype).items()
          if v is not None}
    return dataclasses.replace(w, **kw)


def _draw(rng: np.random.Generator, spec: tuple, n: int) -> np.ndarray:
    kind = spec[0]
    if kind == "const":
        return np.full(n, spec[1], dtype=np.int64)
    if kind == "uniform":
        return rng.integers(spec[1], spec[2] + 1, n).astype(np.int64)
    if kind == "loguniform":
        return np.floor(np.exp(rng.uniform(np.log(spec[1]), np.log(spec[2]), n))).astype(np.int64)
    if kind == "lognormal":
        _, median, sigma, lo, hi = spec
        return np.clip(np.rint(median * np.exp(sigma * rng.standard_normal(n))), lo, hi).astype(np.int64)
    raise ValueError(f"unknown distribution {kind!r}")


@dataclasses.dataclass
class Batch:
    """Device-resident inputs of one engine step.  Rows with q_lens == 1 are decode rows."""
    workload: Workload
    q: torch.Tensor            # [total_q, Hq, D] packed in batch order
    k_pages: torch.Tensor      # [num_pages, Hkv, 16, D]  (uint8 codes for FP8)
    v_pages: torch.Tensor
    page_table: torch.Tensor   # [B, max_pages] int32, -1 where unused
    ctx_lens: torch.Tensor     # [B] int32, includes the chunk
    q_lens: torch.Tensor       # [B] int32
    q_offsets: torch.Tensor    # [B + 1] int32 exclusive scan of q_lens
    k_scale: Optional[torch.Tensor]   # [num_pages] float32 (FP8 only)
    v_scale: Optional[torch.Tensor]
    ctx_lens_host: np.ndarray
    q_lens_host: np.ndarray

    @property
    def num_pages(self) -> int:
        return int(self.k_pages.shape[0])

    @property
    def total_q(self) -> int:
        return int(self.q.shape[0])

    def select(self, rows: np.ndarray) -> "Batch":
        """Sub-batch of the given trajectories (same pools, copied table rows), e.g. the
        decode rows or the append rows of a mixed step."""
        rows = np.asarray(rows, dtype=np.int64)
        dev = self.q.device
        offs = np.concatenate([[0], np.cumsum(self.q_lens_host)])
        qidx = np.concatenate([np.arange(offs[r], offs[r + 1]) for r in rows]) if len(rows) else np.zeros(0, np.int64)
        ql = self.q_lens_host[rows]
        cl = self.ctx_lens_host[rows]
        ridx = torch.from_numpy(rows).to(dev)
        max_pages = max(1, int(((cl + PAGE_SIZE - 1) // PAGE_SIZE).max())) if len(rows) else 1
        return Batch(
            workload=self.workload,
            q=self.q[torch.from_numpy(qidx).to(dev)].contiguous(),
            k_pages=self.k_pages, v_pages=self.v_pages,
            page_table=self.page_table[ridx, :max_pages].contiguous(),
            ctx_lens=torch.from_numpy(cl.astype(np.int32)).to(dev),
            q_lens=torch.from_numpy(ql.astype(np.int32)).to(dev),
            q_offsets=torch.from_numpy(np.concatenate([[0], np.cumsum(ql)]).astype(np.int32)).to(dev),
            k_scale=self.k_scale, v_scale=self.v_scale,
            ctx_lens_host=cl.copy(), q_lens_host=ql.copy(),
        )

    def decode_rows(self) -> np.ndarray:
        return np.nonzero(self.q_lens_host == 1)[0]

    def append_rows(self) -> np.ndarray:
        return np.nonzero(self.q_lens_host != 1)[0]


def draw_structure(w: Workload):
    """Integer structure only (no values): ctx_lens, q_lens, page_table, num_pages."""
    rng = np.random.default_rng(w.seed)
    ctx = _draw(rng, w.ctx, w.batch)
    if w.append_rows is None:
        q_lens = _draw(rng, w.qlen, w.batch)
    else:
        n_app = _draw(rng, w.qlen, w.append_rows)
        rows = rng.permutation(w.batch)[: w.append_rows]
        q_lens = np.ones(w.batch, dtype=np.int64)
        q_lens[rows] = n_app
    if w.ctx_is_prefix:
        ctx_lens = ctx + np.where(q_lens != 1, q_lens, 0) if w.append_rows is not None else ctx + q_lens
    else:
        ctx_lens = ctx
        q_lens = np.minimum(q_lens, ctx_lens)
    pages_per = (ctx_lens + PAGE_SIZE - 1) // PAGE_SIZE
    num_pages = int(pages_per.sum())
    perm = rng.permutation(max(num_pages, 1))[:num_pages]
    max_pages = max(1, int(pages_per.max())) if len(pages_per) else 1
    table = np.full((w.batch, max_pages), -1, dtype=np.int32)
    start = 0
    for b in range(w.batch):
        n = int(pages_per[b])
        table[b, :n] = perm[start:start + n]
        start += n
    return ctx_lens.astype(np.int64), q_lens.astype(np.int64), table, num_pages


def _live_slots(ctx_lens, table, num_pages) -> np.ndarray:
    """Number of live slots of every physical page (16, or fewer on a last page)."""
    live = np.zeros(max(num_pages, 1), dtype=np.int64)[:num_pages]
    for b, length in enumerate(ctx_lens.tolist()):
        n = (length + PAGE_SIZE - 1) // PAGE_SIZE
        if n == 0:
            continue
        live[table[b, :n]] = PAGE_SIZE
        if length % PAGE_SIZE:
            live[table[b, n - 1]] = length % PAGE_SIZE
    return live


def build(w: Workload, device="cpu", *, slab_pages: int = 8192) -> Batch:
    """Draw the batch on `device` (values come from that device's generator, so a CPU
    batch and a GPU batch of the same seed share structure but not values)."""
    device = torch.device(device)
    ctx_lens, q_lens, table, num_pages = draw_structure(w)
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    total_q = int(q_lens.sum())
    qdt = _TORCH_DTYPE[w.q_dtype]
    q = torch.randn((total_q, w.num_q_heads, w.head_dim), generator=gen, device=device,
                    dtype=torch.float32).to(qdt)
    live = torch.from_numpy(_live_slots(ctx_lens, table, num_pages)).to(device)
    shape = (num_pages, w.num_kv_heads, PAGE_SIZE, w.head_dim)
    fp8 = w.kv_dtype == "fp8_e4m3"
    store_dt = torch.uint8 if fp8 else _TORCH_DTYPE[w.kv_dtype]
    pools, scales = [], []
    slot_ids = torch.arange(PAGE_SIZE, device=device).view(1, 1, PAGE_SIZE, 1)
    for _ in range(2):
        pool = torch.empty(shape, device=device, dtype=store_dt)
        scale = torch.ones(num_pages, device=device, dtype=torch.float32) if fp8 else None
        for p0 in range(0, num_pages, slab_pages):
            p1 = min(num_pages, p0 + slab_pages)
            x = torch.randn((p1 - p0,) + shape[1:], generator=gen, device=device, dtype=torch.float32)
            dead = slot_ids >= live[p0:p1].view(-1, 1, 1, 1)
            if fp8:
                amax = x.masked_fill(dead, 0.0).abs().amax(dim=(1, 2, 3))
                s = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
                codes = (x / s.view(-1, 1, 1, 1)).to(torch.float8_e4m3fn).view(torch.uint8)
                pool[p0:p1] = codes.masked_fill(dead, 0x7F)
                scale[p0:p1] = s
            else:
                pool[p0:p1] = x.masked_fill(dead, float("nan")).to(store_dt)
        pools.append(pool)
        scales.append(scale)
    return Batch(
        workload=w, q=q, k_pages=pools[0], v_pages=pools[1],
        page_table=torch.from_numpy(table).to(device),
        ctx_lens=torch.from_numpy(ctx_lens.astype(np.int32)).to(device),
        q_lens=torch.from_numpy(q_lens.astype(np.int32)).to(device),
        q_offsets=torch.from_numpy(np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)).to(device),
        k_scale=scales[0], v_scale=scales[1],
        ctx_lens_host=ctx_lens, q_lens_host=q_lens,
    )


def alias_shared_prefix(batch: Batch, group_size: int, shared_lens: np.ndarray) -> Batch:
    """The same batch with prompts shared inside groups of `group_size` consecutive trajectories (rollouts are
    sampled in groups per prompt, Section 7.1): the page-table entries that cover the first shared_lens[j]
    tokens of every member of group j are replaced by the first member's, so the members alias those
    physical pages.  Only whole pages are aliased (shared_lens is rounded down to the page size here) and
    never beyond a member's own context.  Pools are untouched; the pages the other members no longer
    reference simply go unused."""
    table = batch.page_table.clone()
    host = batch.page_table.detach().cpu().numpy().copy()
    lens = batch.ctx_lens_host
    for j, s in enumerate(np.asarray(shared_lens, dtype=np.int64)):
        members = range(j * group_size, (j + 1) * group_size)
        pages = int(min(int(s), min(int(lens[m]) for m in members))) // PAGE_SIZE
        for m in members:
            host[m, :pages] = host[j * group_size, :pages]
    table.copy_(torch.from_numpy(host))
    return dataclasses.replace(batch, page_table=table)


def raw_numpy(t: Optional[torch.Tensor]):
    """Host copy of a tensor's stored bytes in the raw form a CPU checker takes:
    float32 -> float32, bfloat16 -> uint16 bit patterns, uint8/int32 unchanged."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def algorithmic_work(w: Workload, ctx_lens: np.ndarray, q_lens: np.ndarray) -> dict:
    """Bytes the method has to move and flops it has to do, counting K and V of each KV
    head once per call, the live page-table entries, the page scales, Q in and O out;
    attended (query, key) pairs cost 4 * Hq * D flops."""
    kv_b = {"f32": 4, "bf16": 2, "fp8_e4m3": 1}[w.kv_dtype]
    q_b = {"f32": 4, "bf16": 2}[w.q_dtype]
    L = np.asarray(ctx_lens, dtype=np.int64)
    n = np.asarray(q_lens, dtype=np.int64)
    pages = int(((L + PAGE_SIZE - 1) // PAGE_SIZE).sum())
    kv = int(2 * w.num_kv_heads * w.head_dim * kv_b * L.sum())
    table = 4 * pages
    scales = 8 * pages if w.kv_dtype == "fp8_e4m3" else 0
    qo = int(2 * n.sum() * w.num_q_heads * w.head_dim * q_b)
    pairs = int((n * (L - n) + n * (n + 1) // 2).sum())
    return {"bytes": kv + table + scales + qo, "kv_bytes": kv, "qo_bytes": qo, "pairs": pairs,
            "flops": 4 * w.num_q_heads * w.head_dim * pairs}
