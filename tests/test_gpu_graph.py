"""A whole engine step under a HIP graph: every entry point plans on the device, allocates nothing and
never synchronises, so the mixed step (KV write of the chunks, decode rows, append rows) can be captured
once and replayed while the inputs change in place (Section 7.1 runs rollouts with the engine's step
captured in a graph to remove launch overhead).  Each replay is checked against the same calls made
eagerly on the same inputs, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _step(dec, app, k_new, v_new, out_d, out_a, ws_d, ws_a, w):
    B.kv_write(k_new, v_new, app.q_lens, app.q_offsets, app.k_pages, app.v_pages, app.page_table, app.ctx_lens,
               max_q_len=int(app.q_lens_host.max()), k_scale=app.k_scale, v_scale=app.v_scale)
    B.attn_decode(dec.q, dec.k_pages, dec.v_pages, dec.page_table, dec.ctx_lens, sm_scale=w.sm_scale,
                  k_scale=dec.k_scale, v_scale=dec.v_scale, out=out_d, workspace=ws_d)
    B.attn_append(app.q, app.q_lens, app.q_offsets, app.k_pages, app.v_pages, app.page_table, app.ctx_lens,
                  sm_scale=w.sm_scale, max_q_len=int(app.q_lens_host.max()), k_scale=app.k_scale, v_scale=app.v_scale,
                  out=out_a, workspace=ws_a)


@pytest.mark.parametrize("kv", ["bf16", "fp8_e4m3"])
def test_mixed_step_replays_from_a_graph_like_eager(kv):
    w = W.Workload("graph_mixed", 24, 32, 4, 128, "bf16", kv, ("lognormal", 700, 0.8, 20, 4000),
                   qlen=("uniform", 2, 150), append_rows=8, ctx_is_prefix=True, seed=W.BASE_SEED + 41)
    b = W.build(w, DEV)
    dec, app = b.select(b.decode_rows()), b.select(b.append_rows())
    g = torch.Generator(device="cpu").manual_seed(3)
    shape = (app.total_q, w.num_kv_heads, w.head_dim)
    k_new = torch.randn(shape, generator=g).to(torch.bfloat16).to(DEV)
    v_new = torch.randn(shape, generator=g).to(torch.bfloat16).to(DEV)
    out_d, out_a = torch.empty_like(dec.q), torch.empty_like(app.q)
    ws_d = B.alloc_workspace(B.make_desc(dec.q, dec.k_pages, dec.page_table, sm_scale=w.sm_scale, k_scale=dec.k_scale, v_scale=dec.v_scale), dec.total_q, DEV)
    ws_a = B.alloc_workspace(B.make_desc(app.q, app.k_pages, app.page_table, sm_scale=w.sm_scale, k_scale=app.k_scale, v_scale=app.v_scale), app.total_q, DEV)
    args = (dec, app, k_new, v_new, out_d, out_a, ws_d, ws_a, w)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm up on the capture stream's side
        _step(*args)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(*args)
    torch.cuda.synchronize()

    dec_lens0 = dec.ctx_lens.clone()
    for it in range(4):
        # new inputs in place: queries, the chunk's rows, and shorter decode contexts (the plan must follow)
        dec.q.copy_(torch.randn(dec.q.shape, generator=g).to(torch.bfloat16))
        app.q.copy_(torch.randn(app.q.shape, generator=g).to(torch.bfloat16))
        k_new.copy_(torch.randn(shape, generator=g).to(torch.bfloat16) * (1.0 + it))
        v_new.copy_(torch.randn(shape, generator=g).to(torch.bfloat16))
        dec.ctx_lens.copy_(torch.clamp(dec_lens0 - 7 * it, min=1))
        pools = [t.clone() if t is not None else None for t in (b.k_pages, b.v_pages, b.k_scale, b.v_scale)]
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [out_d.clone(), out_a.clone(), b.k_pages.clone(), b.v_pages.clone()]
        if b.k_scale is not None:
            got += [b.k_scale.clone(), b.v_scale.clone()]
        # the same step eagerly from the same starting cache
        for t, saved in zip((b.k_pages, b.v_pages, b.k_scale, b.v_scale), pools):
            if t is not None:
                t.copy_(saved)
        out_d.zero_(); out_a.zero_()
        torch.cuda.synchronize()
        _step(*args)
        torch.cuda.synchronize()
        want = [out_d, out_a, b.k_pages, b.v_pages] + ([b.k_scale, b.v_scale] if b.k_scale is not None else [])
        for i, (x, y) in enumerate(zip(got, want)):
            assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), f"replay {it}: output {i} differs from the eager step"


def test_calls_on_two_streams_with_workspaces_of_their_own_do_not_disturb_each_other():
    # the library keeps no state between calls: decode and append of one step, each with its own workspace, may
    # run side by side on two streams (default priority) and must give exactly what they give one after the other
    w = W.Workload("two_streams", 96, 32, 4, 128, "bf16", "fp8_e4m3", ("lognormal", 3000, 0.8, 20, 20000),
                   qlen=("uniform", 200, 1500), append_rows=16, ctx_is_prefix=True, seed=W.BASE_SEED + 43)
    b = W.build(w, DEV)
    dec, app = b.select(b.decode_rows()), b.select(b.append_rows())
    out_d, out_a = torch.empty_like(dec.q), torch.empty_like(app.q)
    ws_d = B.alloc_workspace(B.make_desc(dec.q, dec.k_pages, dec.page_table, sm_scale=w.sm_scale, k_scale=dec.k_scale, v_scale=dec.v_scale), dec.total_q, DEV)
    ws_a = B.alloc_workspace(B.make_desc(app.q, app.k_pages, app.page_table, sm_scale=w.sm_scale, k_scale=app.k_scale, v_scale=app.v_scale), app.total_q, DEV)

    def decode(stream=None):
        B.attn_decode(dec.q, dec.k_pages, dec.v_pages, dec.page_table, dec.ctx_lens, sm_scale=w.sm_scale,
                      k_scale=dec.k_scale, v_scale=dec.v_scale, out=out_d, workspace=ws_d, stream=stream)

    def append(stream=None):
        B.attn_append(app.q, app.q_lens, app.q_offsets, app.k_pages, app.v_pages, app.page_table, app.ctx_lens,
                      sm_scale=w.sm_scale, max_q_len=int(app.q_lens_host.max()), k_scale=app.k_scale, v_scale=app.v_scale,
                      out=out_a, workspace=ws_a, stream=stream)

    decode(); append()
    torch.cuda.synchronize()
    want_d, want_a = out_d.clone(), out_a.clone()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):
        out_d.zero_(); out_a.zero_()
        torch.cuda.synchronize()
        append(s2)                       # the long call first, so that the short ones land inside it
        for _ in range(4):
            decode(s1)
        torch.cuda.synchronize()
        assert torch.equal(out_d.view(torch.int16), want_d.view(torch.int16))
        assert torch.equal(out_a.view(torch.int16), want_a.view(torch.int16))
