"""Shared test plumbing: turning a synthetic batch into the oracle's raw-array arguments."""
from __future__ import annotations

import numpy as np

from paper_2512_22560_amd import workloads as W


def oracle_args(batch: "W.Batch") -> dict:
    w = batch.workload
    return dict(
        k_pages=W.raw_numpy(batch.k_pages), v_pages=W.raw_numpy(batch.v_pages),
        page_table=W.raw_numpy(batch.page_table), ctx_lens=batch.ctx_lens_host,
        sm_scale=w.sm_scale, q_dtype=w.q_dtype, kv_dtype=w.kv_dtype,
        k_scale=W.raw_numpy(batch.k_scale), v_scale=W.raw_numpy(batch.v_scale),
    )


def tiny(name="t", batch=3, hq=4, hkv=2, d=16, q_dtype="f32", kv_dtype="f32", ctx=("uniform", 1, 70),
         qlen=("const", 1), seed=7, ctx_is_prefix=False, append_rows=None) -> "W.Batch":
    w = W.Workload(name, batch, hq, hkv, d, q_dtype, kv_dtype, ctx, qlen=qlen, seed=seed,
                   ctx_is_prefix=ctx_is_prefix, append_rows=append_rows)
    return W.build(w, "cpu")


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 values that are exactly representable in bfloat16 -> uint16 patterns."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not representable in bfloat16"
    return (u >> 16).astype(np.uint16)
