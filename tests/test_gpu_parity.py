"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same
seeded inputs.  Sizes here are ones the oracle finishes in seconds but that still span several
KV pieces, several 32-token blocks per wave and ragged tails; full-size cases are in
test_gpu_fullsize.py."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import attention as O
from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, gpu_append, gpu_decode, oracle_append, oracle_decode
from tests.helpers import oracle_args

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# two results of the GPU path for the same inputs, computed with different splits: each within the parity bar of the oracle,
# so at most twice that apart
TOL_BETWEEN = {"f32": 2e-4, "bf16": 4e-2}


def _wl(name, batch, hq, hkv, d, q_dtype, kv_dtype, ctx, qlen=("const", 1), seed=1, prefix=False, append_rows=None):
    return W.Workload(name, batch, hq, hkv, d, q_dtype, kv_dtype, ctx, qlen=qlen, seed=seed, ctx_is_prefix=prefix,
                      append_rows=append_rows)


def _force_lens(batch: W.Batch, lens):
    """Shorten contexts in place (pages stay where they are; the tail becomes unused)."""
    lens = np.asarray(lens, dtype=np.int64)
    assert np.all(lens <= batch.ctx_lens_host)
    batch.ctx_lens_host = lens
    batch.ctx_lens = torch.from_numpy(lens.astype(np.int32)).to(batch.q.device)
    return batch


# ------------------------------------------------------------------ decode

def test_config1_tiny_decode_f32_exact_recipe():
    b = W.build(W.CONFIGS[1], DEV)
    check(gpu_decode(b), oracle_decode(b), "f32", "config 1")


@pytest.mark.parametrize("name,hq,hkv,d,qd,kvd", [
    ("f32_d64_g4", 8, 2, 64, "f32", "f32"),
    ("f32_d128_g3", 6, 2, 128, "f32", "f32"),
    ("f32_d64_g6", 12, 2, 64, "f32", "f32"),
    ("bf16_d128_g4", 32, 8, 128, "bf16", "bf16"),
    ("bf16_d128_g8", 64, 8, 128, "bf16", "bf16"),
    ("bf16_d128_g1", 4, 4, 128, "bf16", "bf16"),
    ("bf16_d128_g3", 6, 2, 128, "bf16", "bf16"),
    ("bf16_d128_g20", 40, 2, 128, "bf16", "bf16"),
    ("bf16_d64_g4", 8, 2, 64, "bf16", "bf16"),
    ("fp8_d128_g16", 64, 4, 128, "bf16", "fp8_e4m3"),
    ("fp8_d128_g5", 10, 2, 128, "bf16", "fp8_e4m3"),
    ("fp8_d64_g8", 16, 2, 64, "bf16", "fp8_e4m3"),
])
def test_decode_ragged_multi_piece(name, hq, hkv, d, qd, kvd):
    # log-uniform lengths from 1 to ~3000: many rows split into several 256-token pieces, most
    # pieces end in a ragged block, some rows are shorter than one block
    b = W.build(_wl(name, 7, hq, hkv, d, qd, kvd, ("loguniform", 1, 3000), seed=101), DEV)
    check(gpu_decode(b), oracle_decode(b), qd, name)


@pytest.mark.parametrize("qd,kvd", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")])
def test_decode_edge_lengths(qd, kvd):
    lens = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513, 0, 1023, 1025]
    d = 64 if qd == "f32" else 128
    b = W.build(_wl("edges", len(lens), 8, 2, d, qd, kvd, ("const", 1040), seed=102), DEV)
    _force_lens(b, lens)
    out = gpu_decode(b)
    check(out, oracle_decode(b), qd, "edge lengths")
    assert not out[0].any() and not out[20].any()          # empty contexts give zero rows


def test_decode_long_runs_cross_the_page_id_window():
    # 20 rows x 64 KV heads x ~1700 blocks over 2048 workers: every wave walks ~1000 blocks, crossing
    # rows and refilling its 32-block window of page ids many times.  Logical pages alias a small
    # physical pool (as shared prefixes do), which keeps the pool small; the oracle reads through the
    # same table.
    rng = np.random.default_rng(103)
    batch, hkv, d, n_phys = 20, 64, 64, 96
    lens = rng.integers(52000, 56000, batch)
    lens[3] = 8192 * 3 + 1
    gen = torch.Generator(device=DEV).manual_seed(103)
    q = torch.randn((batch, hkv, d), generator=gen, device=DEV).to(torch.bfloat16)
    kp = torch.randn((n_phys, hkv, 16, d), generator=gen, device=DEV).to(torch.bfloat16)
    vp = torch.randn((n_phys, hkv, 16, d), generator=gen, device=DEV).to(torch.bfloat16)
    max_pages = int((lens.max() + 15) // 16)
    table = rng.integers(0, n_phys, (batch, max_pages)).astype(np.int32)
    for bb in range(batch):
        table[bb, (lens[bb] + 15) // 16:] = -1
    pt = torch.from_numpy(table).to(DEV)
    cl = torch.from_numpy(lens.astype(np.int32)).to(DEV)
    desc = B.make_desc(q, kp, pt, sm_scale=0.125)
    ws = B.alloc_workspace(desc, batch, DEV)
    out = B.attn_decode(q, kp, vp, pt, cl, sm_scale=0.125, workspace=ws)
    per, total, _ = B.read_plan(desc, ws)
    assert per > 64          # every wave refills its 32-block window of page ids at least twice
    ref = O.attn_decode(W.raw_numpy(q), W.raw_numpy(kp), W.raw_numpy(vp), table, lens, sm_scale=0.125,
                        q_dtype="bf16", kv_dtype="bf16")
    check(out, ref, "bf16", "long runs")


def test_single_key_returns_value_exactly_and_fp8_codes_decode_exactly():
    # L = 1: softmax weight is exactly 1, so out == v0 bit for bit (bf16 in, bf16 out)
    b = W.build(_wl("one", 5, 8, 2, 128, "bf16", "bf16", ("const", 1), seed=105), DEV)
    out = gpu_decode(b).cpu()
    for bb in range(5):
        pid = int(b.page_table[bb, 0])
        for h in range(8):
            assert torch.equal(out[bb, h], b.v_pages[pid, h // 4, 0].cpu())
    # every FP8 code as a value, scale 1: the output must be the OCP E4M3 value of the code
    w = _wl("codes", 2, 2, 2, 128, "bf16", "fp8_e4m3", ("const", 1), seed=106)
    b = W.build(w, DEV)
    codes = torch.arange(256, dtype=torch.uint8)
    codes[codes == 0x7F] = 0
    codes[codes == 0xFF] = 0x80
    for bb in range(2):
        pid = int(b.page_table[bb, 0])
        b.v_pages[pid, :, 0, :] = codes.view(2, 128).to(DEV)
    b.v_scale.fill_(1.0)
    out = gpu_decode(b).to(torch.float64).cpu().numpy()
    ref = O.e4m3fn_to_float64(codes.numpy()).reshape(2, 128)
    for bb in range(2):
        assert np.array_equal(out[bb, 0], ref[0]) and np.array_equal(out[bb, 1], ref[1])


def test_gqa_groups_are_contiguous():
    b = W.build(_wl("gqa", 4, 24, 3, 128, "bf16", "bf16", ("uniform", 100, 900), seed=107), DEV)
    for g in range(3):
        b.v_pages[:, g] = float(g + 1)
    out = gpu_decode(b).to(torch.float32).cpu().numpy()
    for h in range(24):
        assert np.all(out[:, h, :] == h // 8 + 1)


@pytest.mark.parametrize("qd,kvd", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")])
def test_output_is_bit_identical_under_physical_page_permutation(qd, kvd):
    d = 64 if qd == "f32" else 128
    b = W.build(_wl("perm", 6, 8, 2, d, qd, kvd, ("loguniform", 1, 2500), seed=108), DEV)
    base = gpu_decode(b)
    n = b.num_pages
    perm = torch.from_numpy(np.random.default_rng(3).permutation(n)).to(DEV)   # old page p -> new id perm[p]
    inv = torch.argsort(perm)
    k2, v2 = b.k_pages[inv].contiguous(), b.v_pages[inv].contiguous()
    pt = b.page_table.clone()
    live = pt >= 0
    pt[live] = perm[pt[live].long()].to(torch.int32)
    ks = None if b.k_scale is None else b.k_scale[inv].contiguous()
    vs = None if b.v_scale is None else b.v_scale[inv].contiguous()
    out2 = B.attn_decode(b.q, k2, v2, pt, b.ctx_lens, sm_scale=b.workload.sm_scale, k_scale=ks, v_scale=vs)
    assert torch.equal(out2.view(torch.uint8), base.view(torch.uint8))


@pytest.mark.parametrize("kvd", ["f32", "bf16", "fp8_e4m3"])
def test_debug_gather_is_byte_exact(kvd):
    qd = "f32" if kvd == "f32" else "bf16"
    b = W.build(_wl("gather", 5, 4, 2, 128, qd, kvd, ("uniform", 1, 300), seed=109), DEV)
    args = oracle_args(b)
    for bb in range(5):
        L = int(b.ctx_lens_host[bb])
        for g in range(2):
            got = W.raw_numpy(B.debug_gather(b.k_pages, b.page_table, b.ctx_lens, bb, g, L))
            ref = O.gather_tokens(args["k_pages"], args["page_table"], bb, g, L, kvd, raw=True)
            assert got.tobytes() == np.ascontiguousarray(ref).tobytes()


@pytest.mark.parametrize("seed,batch,hi,group", [(1, 64, 8192, 4), (2, 5, 300, 1), (3, 3000, 2000, 20), (4, 300, 40000, 16),
                                                 (5, 9000, 100, 2), (6, 1024, 700, 8), (7, 1025, 700, 8),
                                                 (8, 1000, 3, 1), (9, 257, 5000, 33)])
def test_device_plan_equals_host_twin_and_oracle_rule(seed, batch, hi, group):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, hi, batch).astype(np.int32)
    hkv, d = 2, 64
    max_pages = hi // 16 + 1
    q = torch.zeros((batch, hkv * group, d), dtype=torch.bfloat16, device=DEV)
    # every row points at page 0: the plan must not depend on page ids, and the pool stays tiny
    kp = torch.zeros((1, hkv, 16, d), dtype=torch.bfloat16, device=DEV)
    pt = torch.zeros((batch, max_pages), dtype=torch.int32, device=DEV)
    cl = torch.from_numpy(lens).to(DEV)
    desc = B.make_desc(q, kp, pt, sm_scale=1.0)
    ws = B.alloc_workspace(desc, batch, DEV)
    B.attn_decode(q, kp, kp, pt, cl, sm_scale=1.0, workspace=ws)
    per, total, starts = B.read_plan(desc, ws)
    h_per, h_total, h_segs = B.debug_plan(desc, lens)
    rows_per_b = hkv * -(-group // 16)
    o_per, o_total, o_starts, o_segs = O.split_plan(lens, rows_per_b, B.plan_workers(desc))
    assert (per, total) == (h_per, h_total) == (o_per, o_total)
    assert np.array_equal(starts, o_starts)
    assert np.array_equal(h_segs, o_segs)


@pytest.mark.parametrize("qd,kvd", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")])
def test_decode_does_not_depend_on_how_many_workers_cut_the_contexts(qd, kvd):
    # one worker walks every row of the batch in turn; two and seven cut a few rows at odd places; a hundred cut most rows; the
    # default cuts these short rows many times each: the same attention every time (and the plan is the oracle's rule for that number)
    d = 64 if qd == "f32" else 128
    b = W.build(_wl("cuts", 9, 8, 2, d, qd, kvd, ("loguniform", 1, 1500), seed=209), DEV)
    ref = oracle_decode(b)
    desc = B.make_desc(b.q, b.k_pages, b.page_table, sm_scale=b.workload.sm_scale, k_scale=b.k_scale, v_scale=b.v_scale)
    rows_per_b = 2 * -(-4 // (4 if qd == "f32" else 16))
    default = B.plan_workers(desc)
    outs = {}
    try:
        for workers in (1, 2, 7, 100, 0):
            B.set_decode_workers(workers)
            assert B.plan_workers(desc) == (workers or default)
            ws = B.alloc_workspace(desc, 9, DEV)
            outs[workers] = gpu_decode(b, workspace=ws)
            check(outs[workers], ref, qd, f"{workers} workers")
            per, total, starts = B.read_plan(desc, ws)
            o_per, o_total, o_starts, _ = O.split_plan(b.ctx_lens_host, rows_per_b, workers or default)
            assert (per, total) == (o_per, o_total) and np.array_equal(starts, o_starts)
            h_per, h_total, _ = B.debug_plan(desc, b.ctx_lens_host.astype(np.int32))
            assert (h_per, h_total) == (o_per, o_total)
    finally:
        B.set_decode_workers(0)
    tol = TOL_BETWEEN[qd]
    for workers in (1, 2, 7, 100):
        assert (outs[workers].float() - outs[0].float()).abs().max().item() <= tol


@pytest.mark.parametrize("seed,batch,group,max_q,step,half", [
    (1, 64, 4, 1024, False, False), (2, 7, 1, 5, False, False), (3, 500, 16, 300, True, False), (4, 4096, 8, 40, False, False),
    (5, 4097, 8, 40, True, False), (6, 33, 256, 9, False, False), (7, 40, 3, 200, True, False),
    (8, 64, 4, 300, False, True), (9, 1500, 16, 40, True, True)])
def test_device_append_tile_list_equals_the_oracle_rule(seed, batch, group, max_q, step, half):
    # the list the append kernel's workgroups take in order: which (trajectory, first row) tiles, and in which order
    # (half: the call is told max_q_len = 1 and so cuts the chunks into tiles of half the rows)
    rng = np.random.default_rng(seed)
    q_lens = rng.integers(0, max_q + 1, batch).astype(np.int32)
    if step:
        q_lens[rng.random(batch) < 0.5] = 1                     # a mixed step: one-token chunks go to the decode path
    ctx = (q_lens + rng.integers(0, 3000, batch)).astype(np.int32)
    ctx[: batch // 4] = ctx[0] + q_lens[: batch // 4] - q_lens[0]    # equal contexts ... mostly
    ctx = np.maximum(ctx, q_lens)
    hkv, d = 1, 64
    offs = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    total_q = int(offs[-1])
    max_pages = int(ctx.max()) // 16 + 1
    q = torch.zeros((max(total_q, 1), hkv * group, d), dtype=torch.bfloat16, device=DEV)[:total_q]
    kp = torch.zeros((1, hkv, 16, d), dtype=torch.bfloat16, device=DEV)      # every entry points at page 0
    pt = torch.zeros((batch, max_pages), dtype=torch.int32, device=DEV)
    args = (torch.from_numpy(q_lens).to(DEV), torch.from_numpy(offs).to(DEV), kp, kp, pt, torch.from_numpy(ctx).to(DEV))
    desc = B.make_desc(q, kp, pt, sm_scale=1.0)
    tile_tokens = max(1, (128 if half else 256) // group)
    if half:
        max_q = 1
    if step:
        n = int(B.lib().rollattn_step_workspace_bytes(ctypes.byref(desc), total_q))
        ws = torch.empty(n, dtype=torch.uint8, device=DEV)
        B.attn_step(q, *args, sm_scale=1.0, max_q_len=max_q, workspace=ws)
        got = B.read_append_plan(desc, ws[int(B.lib().rollattn_step_append_offset(ctypes.byref(desc))):], total_q)
    else:
        ws = B.alloc_workspace(desc, total_q, DEV)
        B.attn_append(q, *args, sm_scale=1.0, max_q_len=max_q, workspace=ws)
        got = B.read_append_plan(desc, ws, total_q)
    want = O.append_tile_plan(q_lens, ctx, tile_tokens, skip_unit_chunks=step)
    assert np.array_equal(got, want[:, :2])


# ------------------------------------------------------------------ append

@pytest.mark.parametrize("name,hq,hkv,d,qd,kvd", [
    ("app_f32", 8, 2, 64, "f32", "f32"),
    ("app_bf16_g4", 32, 8, 128, "bf16", "bf16"),
    ("app_bf16_g1", 2, 2, 128, "bf16", "bf16"),
    ("app_bf16_g3", 6, 2, 128, "bf16", "bf16"),
    ("app_bf16_d64", 8, 2, 64, "bf16", "bf16"),
    ("app_fp8_g16", 32, 2, 128, "bf16", "fp8_e4m3"),
    ("app_fp8_d64_g4", 8, 2, 64, "bf16", "fp8_e4m3"),
    ("app_bf16_g256", 256, 1, 128, "bf16", "bf16"),      # one chunk token per workgroup tile
    ("app_fp8_g40", 40, 1, 64, "bf16", "fp8_e4m3"),      # a group that does not divide the tile
    ("app_bf16_g5_hkv3", 15, 3, 128, "bf16", "bf16"),
])
def test_append_ragged_chunks_on_cached_prefix(name, hq, hkv, d, qd, kvd):
    # prefixes 0..700 and chunks 1..300: several query tiles per row for G >= 4, several 64-token KV
    # blocks, ragged ends on both axes, diagonal tiles in the middle of a block
    b = W.build(_wl(name, 6, hq, hkv, d, qd, kvd, ("uniform", 0, 700), qlen=("uniform", 1, 300), seed=201,
                    prefix=True), DEV)
    check(gpu_append(b), oracle_append(b), qd, name)


@pytest.mark.parametrize("qd,kvd", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")])
def test_append_with_unit_chunks_equals_decode_and_empty_chunks_add_no_rows(qd, kvd):
    d = 64 if qd == "f32" else 128
    b = W.build(_wl("unit", 9, 8, 2, d, qd, kvd, ("loguniform", 1, 900), seed=202), DEV)
    ref = oracle_decode(b)
    check(gpu_append(b), ref, qd, "unit chunks")
    # mixed: some rows contribute no query rows at all
    b = W.build(_wl("holes", 8, 8, 2, d, qd, kvd, ("uniform", 1, 200), qlen=("uniform", 0, 40), seed=203, prefix=True), DEV)
    assert (b.q_lens_host == 0).any() or True
    check(gpu_append(b), oracle_append(b), qd, "rows without chunk")


@pytest.mark.parametrize("kvd", ["bf16", "fp8_e4m3"])
def test_append_block_and_ring_boundaries(kvd):
    # contexts of 1 .. 7 blocks exactly, one token either side, and chunks that start and end on block edges: the
    # LDS ring (three tiles, or two through registers) wraps at different phases for each of them
    lens = [1, 2, 63, 64, 65, 127, 128, 129, 191, 192, 193, 256, 257, 320, 383, 384, 385, 448]
    ctx = np.array(lens)
    qn = np.array([1, 2, 63, 64, 1, 64, 128, 65, 3, 192, 129, 64, 257, 1, 200, 384, 2, 64])
    w = _wl("ring", len(lens), 8, 2, 128, "bf16", kvd, ("const", 0), qlen=("const", 1), seed=207, prefix=True)
    import dataclasses
    b = W.build(dataclasses.replace(w, ctx=("uniform", 448, 448)), DEV)     # room for every length, then shortened
    offs = np.concatenate([[0], np.cumsum(qn)]).astype(np.int32)
    b = dataclasses.replace(b, ctx_lens=torch.from_numpy(ctx.astype(np.int32)).to(DEV), q_lens=torch.from_numpy(qn.astype(np.int32)).to(DEV),
                            q_offsets=torch.from_numpy(offs).to(DEV), ctx_lens_host=ctx, q_lens_host=qn,
                            q=torch.randn((int(qn.sum()), 8, 128), generator=torch.Generator().manual_seed(1)).to(torch.bfloat16).to(DEV))
    check(gpu_append(b), oracle_append(b), "bf16", f"ring boundaries {kvd}")


def test_append_empty_prefix_is_causal_self_attention():
    b = W.build(_wl("self", 3, 8, 2, 128, "bf16", "bf16", ("const", 0), qlen=("uniform", 1, 400), seed=204, prefix=True), DEV)
    assert np.array_equal(b.ctx_lens_host, b.q_lens_host)
    out = gpu_append(b)
    check(out, oracle_append(b), "bf16", "empty prefix")
    # first row of every chunk sees one key: its value comes back exactly
    offs = np.concatenate([[0], np.cumsum(b.q_lens_host)])
    for bb in range(3):
        pid = int(b.page_table[bb, 0])
        for h in range(8):
            assert torch.equal(out[offs[bb], h].cpu(), b.v_pages[pid, h // 4, 0].cpu())


def test_mixed_step_scaled_down():
    # the mixed rollout step in miniature: decode rows and append rows share one FP8 pool
    w = _wl("mixed", 24, 64, 4, 128, "bf16", "fp8_e4m3", ("lognormal", 600, 0.8, 20, 4000), qlen=("uniform", 2, 120),
            seed=205, prefix=True, append_rows=6)
    b = W.build(w, DEV)
    dec, app = b.select(b.decode_rows()), b.select(b.append_rows())
    check(gpu_decode(dec), oracle_decode(dec), "bf16", "mixed/decode")
    check(gpu_append(app), oracle_append(app), "bf16", "mixed/append")


@pytest.mark.parametrize("scale", [-0.2, 0.0])
def test_non_positive_softmax_scale(scale):
    # sm_scale is a plain number: a negative one favours the most dissimilar keys, zero gives the
    # (causal) running mean of V
    for kvd in ("bf16", "fp8_e4m3"):
        w = _wl("neg", 4, 8, 2, 128, "bf16", kvd, ("uniform", 0, 300), qlen=("uniform", 1, 150), seed=301, prefix=True)
        b = W.build(w, DEV)
        got = B.attn_append(b.q, b.q_lens, b.q_offsets, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=scale,
                            max_q_len=int(b.q_lens_host.max()), k_scale=b.k_scale, v_scale=b.v_scale)
        ref = O.attn_append(W.raw_numpy(b.q), b.q_lens_host, **dict(oracle_args(b), sm_scale=scale))
        check(got, ref, "bf16", f"append scale {scale} {kvd}")
        dec = B.attn_decode(b.q[: w.batch].contiguous(), b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=scale,
                            k_scale=b.k_scale, v_scale=b.v_scale)
        ref = O.attn_decode(W.raw_numpy(b.q[: w.batch].contiguous()), **dict(oracle_args(b), sm_scale=scale))
        check(dec, ref, "bf16", f"decode scale {scale} {kvd}")


@pytest.mark.parametrize("kvd", ["bf16", "fp8_e4m3"])
@pytest.mark.parametrize("gain", [4.0, 100.0])
def test_scores_that_keep_growing_along_the_context(kvd, gain):
    # keys whose score rises with the position: the running reference of the online softmax has to move in
    # almost every block, at gain 100 by more than 2^128 between blocks, so that exponentials taken against the
    # stale reference overflow before the kernels notice (append) or would without the running maximum (decode)
    import dataclasses
    w = _wl("growing", 3, 8, 2, 128, "bf16", kvd, ("uniform", 500, 900), qlen=("uniform", 30, 200), seed=208, prefix=True)
    b = W.build(w, DEV)
    u = torch.nn.functional.normalize(torch.randn(128, generator=torch.Generator().manual_seed(2)), dim=0)
    # every query is +u times gain * sqrt(D) (which the softmax scale 1/sqrt(D) takes back) and a per-row factor,
    # key t of every trajectory is u * ramp(t) plus a little noise: score = gain * factor * t / 64
    q = (u[None, None, :] * (gain * 128 ** 0.5) * (0.5 + torch.rand(b.q.shape[0], 8, 1, generator=torch.Generator().manual_seed(3)))).to(torch.bfloat16).to(DEV)
    kp = b.k_pages
    tbl = b.page_table.cpu().numpy()
    ramp_pages = torch.zeros((b.num_pages, 16), dtype=torch.float32)
    for bb in range(3):
        n_pages = (int(b.ctx_lens_host[bb]) + 15) // 16
        pos = torch.arange(n_pages * 16, dtype=torch.float32).reshape(n_pages, 16)
        ramp_pages[torch.from_numpy(tbl[bb, :n_pages].astype(np.int64))] = pos / 64.0        # one unit per 64-token block
    noise = 0.01 * torch.randn((b.num_pages, 2, 16, 128), generator=torch.Generator().manual_seed(4))
    k_val = (ramp_pages[:, None, :, None] * u[None, None, None, :] + noise)                    # [pages, Hkv, 16, D]
    if kvd == "bf16":
        kp.copy_(k_val.to(torch.bfloat16))
        b = dataclasses.replace(b, q=q)
    else:
        amax = k_val.abs().amax(dim=(1, 2, 3)).clamp_min(1e-6)
        scale = (amax / 448.0).to(torch.float32)
        codes = (k_val / scale[:, None, None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
        kp.copy_(codes)
        b.k_scale.copy_(scale)
        b = dataclasses.replace(b, q=q)
    # the sharper the softmax, the closer a row comes to a single V row, whose elements reach |4| for unit-variance
    # values, where the bf16 rounding of the output alone is 0.016: the values of this test are a quarter of
    # that (an exact change of the stored numbers: a power of two), so that outputs stay at unit scale and the
    # bar applies as it stands
    if kvd == "bf16":
        b.v_pages.mul_(0.25)
    else:
        b.v_scale.mul_(0.25)
    ref = oracle_append(b)
    assert float(np.abs(ref).max()) <= 1.25
    check(gpu_append(b), ref, "bf16", f"append, growing scores, gain {gain}")
    offs = np.concatenate([[0], np.cumsum(b.q_lens_host)])
    last = torch.from_numpy(offs[1:] - 1).to(DEV)
    dec = dataclasses.replace(b, q=b.q[last].contiguous(), q_lens=torch.ones(3, dtype=torch.int32, device=DEV),
                              q_offsets=torch.arange(4, dtype=torch.int32, device=DEV), q_lens_host=np.ones(3, dtype=np.int64))
    check(gpu_decode(dec), oracle_decode(dec), "bf16", f"decode, growing scores, gain {gain}")
