"""Plumbing for the GPU parity tests: run the HIP path through the C ABI binding, run the oracle on
host copies of the very same bytes, compare element by element."""
from __future__ import annotations

import numpy as np
import torch

from oracle import attention as O
from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.helpers import oracle_args

# Tolerances of the parity bar: float32 path max |err| <= 1e-4; bf16 / fp8 paths max |err| <= 2e-2
# and mean |err| <= 2e-3 over all output elements of the call, against the un-rounded float64 oracle
# run on the same stored (already quantised) inputs.
TOL = {"f32": (1e-4, 1e-4), "bf16": (2e-2, 2e-3)}


def gpu_decode(batch: W.Batch, **kw) -> torch.Tensor:
    w = batch.workload
    return B.attn_decode(batch.q, batch.k_pages, batch.v_pages, batch.page_table, batch.ctx_lens,
                         sm_scale=w.sm_scale, k_scale=batch.k_scale, v_scale=batch.v_scale, **kw)


def gpu_append(batch: W.Batch, **kw) -> torch.Tensor:
    w = batch.workload
    return B.attn_append(batch.q, batch.q_lens, batch.q_offsets, batch.k_pages, batch.v_pages, batch.page_table,
                         batch.ctx_lens, sm_scale=w.sm_scale, max_q_len=int(max(1, batch.q_lens_host.max(initial=1))),
                         k_scale=batch.k_scale, v_scale=batch.v_scale, **kw)


def oracle_decode(batch: W.Batch) -> np.ndarray:
    return O.attn_decode(W.raw_numpy(batch.q), **oracle_args(batch))


def oracle_append(batch: W.Batch) -> np.ndarray:
    return O.attn_append(W.raw_numpy(batch.q), batch.q_lens_host, **oracle_args(batch))


def check(got: torch.Tensor, ref: np.ndarray, q_dtype: str, what: str = ""):
    g = got.detach().to(torch.float64).cpu().numpy()
    assert g.shape == ref.shape, (g.shape, ref.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - ref)
    max_tol, mean_tol = TOL[q_dtype]
    mx = float(err.max(initial=0.0))
    mean = float(err.mean()) if err.size else 0.0
    assert mx <= max_tol, f"{what}: max abs err {mx:.3e} > {max_tol}"
    assert mean <= mean_tol, f"{what}: mean abs err {mean:.3e} > {mean_tol}"
    return mx, mean
