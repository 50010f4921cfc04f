"""attn_step: one call for a mixed engine step.  The oracle of the whole step is attn_append on the mixed batch
(a chunk of one token is a decode row); row for row the result must also be bit-identical to attn_decode and
attn_append on the two sub-batches a host-side scheduler would have made."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, gpu_append, gpu_decode, oracle_append

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _step(b, **kw):
    w = b.workload
    return B.attn_step(b.q, b.q_lens, b.q_offsets, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=w.sm_scale,
                       max_q_len=int(max(1, b.q_lens_host.max(initial=1))), k_scale=b.k_scale, v_scale=b.v_scale, **kw)


def _rows(b, sel):
    offs = np.concatenate([[0], np.cumsum(b.q_lens_host)])
    idx = np.concatenate([np.arange(offs[r], offs[r + 1]) for r in sel]) if len(sel) else np.zeros(0, dtype=np.int64)
    return torch.from_numpy(idx.astype(np.int64)).to(DEV)


@pytest.mark.parametrize("name,hq,hkv,d,qd,kvd", [
    ("step_bf16", 32, 4, 128, "bf16", "bf16"), ("step_fp8", 64, 4, 128, "bf16", "fp8_e4m3"),
    ("step_fp8_d64_g3", 6, 2, 64, "bf16", "fp8_e4m3"), ("step_f32", 8, 2, 64, "f32", "f32"),
])
def test_mixed_step_in_one_call(name, hq, hkv, d, qd, kvd):
    # 40 trajectories, 9 of them with an observation chunk of 2 .. 200 tokens, the rest generating
    w = W.Workload(name, 40, hq, hkv, d, qd, kvd, ("lognormal", 500, 0.9, 1, 3000), qlen=("uniform", 2, 200),
                   append_rows=9, ctx_is_prefix=True, seed=W.BASE_SEED + 51)
    b = W.build(w, DEV)
    assert (b.q_lens_host == 1).sum() == 31
    out = _step(b)
    torch.cuda.synchronize()
    check(out, oracle_append(b), qd, name)
    # the same rows through the two calls on sub-batches
    dec_rows, app_rows = b.decode_rows(), b.append_rows()
    dec, app = b.select(dec_rows), b.select(app_rows)
    if qd != "f32":      # (the float32 path uses one kernel for both kinds, so there is nothing to compare)
        assert torch.equal(out[_rows(b, dec_rows)].view(torch.int16), gpu_decode(dec).view(torch.int16))
        assert torch.equal(out[_rows(b, app_rows)].view(torch.int16), gpu_append(app).view(torch.int16))


@pytest.mark.parametrize("qlens", [[1] * 12, [0, 1, 0, 5, 1, 0, 64, 1, 1, 300, 0, 2], [7, 30, 2, 2, 90, 100, 3, 64, 65, 33, 17, 128]])
def test_only_decode_rows_only_chunks_and_rows_without_work(qlens):
    import dataclasses
    qn = np.asarray(qlens, dtype=np.int64)
    w = W.Workload("step_edges", len(qn), 16, 2, 128, "bf16", "bf16", ("uniform", 300, 900), seed=W.BASE_SEED + 52)
    b = W.build(w, DEV)
    offs = np.concatenate([[0], np.cumsum(qn)]).astype(np.int32)
    q = torch.randn((int(qn.sum()), 16, 128), generator=torch.Generator().manual_seed(5)).to(torch.bfloat16).to(DEV)
    b = dataclasses.replace(b, q=q, q_lens=torch.from_numpy(qn.astype(np.int32)).to(DEV),
                            q_offsets=torch.from_numpy(offs).to(DEV), q_lens_host=qn)
    out = _step(b)
    torch.cuda.synchronize()
    check(out, oracle_append(b), "bf16", f"q_lens {qlens}")


def test_full_size_mixed_step_equals_the_two_calls():
    b = W.build(W.CONFIGS[5], DEV)
    out = _step(b)
    dec_rows, app_rows = b.decode_rows(), b.append_rows()
    dec, app = b.select(dec_rows), b.select(app_rows)
    assert torch.equal(out[_rows(b, dec_rows)].view(torch.int16), gpu_decode(dec).view(torch.int16))
    assert torch.equal(out[_rows(b, app_rows)].view(torch.int16), gpu_append(app).view(torch.int16))


def test_one_call_step_replays_from_a_graph_like_eager():
    w = W.Workload("step_graph", 32, 32, 4, 128, "bf16", "fp8_e4m3", ("lognormal", 700, 0.8, 20, 4000),
                   qlen=("uniform", 2, 150), append_rows=8, ctx_is_prefix=True, seed=W.BASE_SEED + 53)
    b = W.build(w, DEV)
    out = torch.empty_like(b.q)
    desc = B.make_desc(b.q, b.k_pages, b.page_table, sm_scale=w.sm_scale, k_scale=b.k_scale, v_scale=b.v_scale)
    ws = torch.empty(int(B.lib().rollattn_step_workspace_bytes(desc, b.total_q)), dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _step(b, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(b, out=out, workspace=ws)
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(9)
    lens0 = b.ctx_lens.clone()
    is_dec = torch.from_numpy(b.q_lens_host == 1).to(DEV)
    for it in range(3):
        b.q.copy_(torch.randn(b.q.shape, generator=g).to(torch.bfloat16))
        # decode rows look at shorter histories each time: the device-side plan has to follow
        b.ctx_lens.copy_(torch.where(is_dec, torch.clamp(lens0 - 11 * it, min=1), lens0))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.zero_()
        torch.cuda.synchronize()
        _step(b, out=out, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), out.view(torch.int16)), f"replay {it}"


def test_mixed_step_on_a_batch_too_large_for_the_plans_lds_tables():
    # 9000 trajectories: the decode plan keeps its scan in global memory, the append plan does not rank; both
    # still have to tell decode rows from chunk rows
    w = W.Workload("step_wide", 9000, 4, 2, 64, "bf16", "bf16", ("uniform", 1, 60), qlen=("uniform", 2, 20),
                   append_rows=700, ctx_is_prefix=True, seed=W.BASE_SEED + 54)
    b = W.build(w, DEV)
    out = _step(b)
    torch.cuda.synchronize()
    check(out, oracle_append(b), "bf16", "9000 trajectories")
