"""The softmax denominators the attention calls can hand out (attn_decode_lse, attn_append_lse) and the merge of
two results over disjoint token ranges (attn_merge), against the oracle's definitions."""
from __future__ import annotations

import dataclasses

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
LSE_TOL = {"f32": 1e-4, "bf16": 2e-3}      # absolute, in log2 units (values reach ~ 20)
# The append kernel over bf16 pools multiplies the query by sm_scale * log2(e) and rounds it to bf16 once, when it loads
# it: every product q_d k_d of a score then carries an independent relative error of at most 2^-9, which for unit-variance
# inputs and D = 128 is about 1.6e-3 (rms) in log2 units per score.  The logarithm of the denominator moves by a weighted
# mean of these, at most by the largest of them: a few standard deviations.  (The outputs themselves stay inside the bar
# of the bf16 paths, which the same tests check.)
LSE_TOL_APPEND_BF16_POOLS = 1e-2


def _oracle_lse(b, q_lens):
    a = oracle_args(b)
    return O.attn_lse(W.raw_numpy(b.q), q_lens, a["k_pages"], a["page_table"], a["ctx_lens"], sm_scale=a["sm_scale"],
                      q_dtype=a["q_dtype"], kv_dtype=a["kv_dtype"], k_scale=a["k_scale"])


def _check_lse(got, ref, qd, what, tol=None):
    tol = LSE_TOL[qd] if tol is None else tol
    g = got.double().cpu().numpy()
    assert g.shape == ref.shape
    empty = np.isneginf(ref)
    assert np.array_equal(np.isneginf(g), empty), f"{what}: rows without tokens"
    err = np.abs(g[~empty] - ref[~empty])
    assert err.size == 0 or err.max() <= tol, f"{what}: lse max abs err {err.max():.3e}"


@pytest.mark.parametrize("hq,hkv,d,qd,kvd", [(8, 2, 64, "f32", "f32"), (32, 8, 128, "bf16", "bf16"), (32, 2, 128, "bf16", "fp8_e4m3"),
                                             (6, 2, 64, "bf16", "fp8_e4m3")])
def test_decode_denominators(hq, hkv, d, qd, kvd):
    b = W.build(W.Workload("lse_dec", 9, hq, hkv, d, qd, kvd, ("loguniform", 1, 1500), seed=W.BASE_SEED + 71), DEV)
    lens = b.ctx_lens_host.copy()
    lens[4] = 0                                             # a trajectory without tokens: zero row, lse = -inf
    b = dataclasses.replace(b, ctx_lens=torch.from_numpy(lens.astype(np.int32)).to(DEV), ctx_lens_host=lens)
    w = b.workload
    out, lse = B.attn_decode_lse(b.q, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=w.sm_scale, k_scale=b.k_scale,
                                 v_scale=b.v_scale)
    torch.cuda.synchronize()
    assert torch.equal(out, gpu_decode(b))                  # the extra output changes nothing else
    check(out, oracle_decode(b), qd, "decode with lse")
    _check_lse(lse, _oracle_lse(b, None), qd, "decode")


@pytest.mark.parametrize("hq,hkv,d,qd,kvd", [(8, 2, 64, "f32", "f32"), (32, 8, 128, "bf16", "bf16"), (32, 2, 128, "bf16", "fp8_e4m3")])
def test_append_denominators(hq, hkv, d, qd, kvd):
    b = W.build(W.Workload("lse_app", 6, hq, hkv, d, qd, kvd, ("uniform", 0, 600), qlen=("uniform", 0, 150), ctx_is_prefix=True,
                           seed=W.BASE_SEED + 72), DEV)
    w = b.workload
    out, lse = B.attn_append_lse(b.q, b.q_lens, b.q_offsets, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=w.sm_scale,
                                 max_q_len=int(max(1, b.q_lens_host.max())), k_scale=b.k_scale, v_scale=b.v_scale)
    torch.cuda.synchronize()
    assert torch.equal(out, gpu_append(b))
    check(out, oracle_append(b), qd, "append with lse")
    _check_lse(lse, _oracle_lse(b, b.q_lens_host), qd, "append", tol=LSE_TOL_APPEND_BF16_POOLS if kvd == "bf16" else None)


@pytest.mark.parametrize("kvd", ["bf16", "fp8_e4m3"])
@pytest.mark.parametrize("name,hq,hkv,d,max_q", [("half_g16", 64, 4, 128, 8), ("half_g1", 8, 8, 128, 128), ("half_d64_g8", 16, 2, 64, 16),
                                                 ("half_g40", 40, 1, 64, 3)])
def test_append_half_tiles(name, hq, hkv, d, max_q, kvd):
    # No chunk fills more than half a query tile: the kernel then lets the two waves of a SIMD split every KV block
    # (32 tokens each) and merges their two running states when the tile ends.  Prefixes from 0 on: in contexts of up to 32
    # tokens the second wave of a pair sees nothing at all, in ragged last blocks only part of its share.
    b = W.build(W.Workload(name, 40, hq, hkv, d, "bf16", kvd, ("uniform", 0, 300), qlen=("uniform", 1, max_q), ctx_is_prefix=True,
                           seed=W.BASE_SEED + 74), DEV)
    assert int(b.q_lens_host.max()) * (hq // hkv) <= 128 and b.ctx_lens_host.min() <= 64 and b.ctx_lens_host.max() > 256
    w = b.workload
    out, lse = B.attn_append_lse(b.q, b.q_lens, b.q_offsets, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=w.sm_scale,
                                 max_q_len=int(b.q_lens_host.max()), k_scale=b.k_scale, v_scale=b.v_scale)
    torch.cuda.synchronize()
    check(out, oracle_append(b), "bf16", name)
    _check_lse(lse, _oracle_lse(b, b.q_lens_host), "bf16", name, tol=LSE_TOL_APPEND_BF16_POOLS if kvd == "bf16" else None)
    # a max_q_len above half a tile selects whole tiles: same rows, the other kernel variant, the same result within rounding
    whole = B.attn_append(b.q, b.q_lens, b.q_offsets, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=w.sm_scale,
                          max_q_len=256, k_scale=b.k_scale, v_scale=b.v_scale)
    torch.cuda.synchronize()
    check(whole, oracle_append(b), "bf16", name + " (whole tiles)")
    assert (out.float() - whole.float()).abs().max().item() <= 2e-2


def test_append_with_an_understated_max_q_len_is_still_right():
    # max_q_len = 1 selects half tiles although the chunks have up to 300 tokens: they are then cut into many
    # half tiles (causal edges inside them), and the work list has room for them
    b = W.build(W.Workload("half_many", 6, 32, 2, 128, "bf16", "fp8_e4m3", ("uniform", 0, 700), qlen=("uniform", 1, 300), ctx_is_prefix=True,
                           seed=W.BASE_SEED + 75), DEV)
    w = b.workload
    out = B.attn_append(b.q, b.q_lens, b.q_offsets, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, sm_scale=w.sm_scale,
                        max_q_len=1, k_scale=b.k_scale, v_scale=b.v_scale)
    torch.cuda.synchronize()
    check(out, oracle_append(b), "bf16", "half tiles, many per chunk")


@pytest.mark.parametrize("qd,kvd,d", [("f32", "f32", 64), ("bf16", "bf16", 128), ("bf16", "fp8_e4m3", 128)])
def test_a_context_split_over_two_calls_and_merged(qd, kvd, d):
    # what a second GPU holding the later pages would do: range 1 = the first S_b tokens, range 2 = the rest through a
    # table that starts S_b / 16 entries later; the merge must give the attention over the whole context
    b = W.build(W.Workload("split", 10, 16, 4, d, qd, kvd, ("uniform", 100, 1200), seed=W.BASE_SEED + 73), DEV)
    w = b.workload
    lens = b.ctx_lens_host
    cut = (np.random.default_rng(3).integers(0, lens // 16 + 1) * 16).astype(np.int64)      # whole pages, 0 .. L_b
    cut[0], cut[1] = 0, (lens[1] // 16) * 16                                                 # an empty first range; a (nearly) empty second
    table = b.page_table.cpu().numpy()
    shifted = np.zeros_like(table)
    for bb in range(10):
        shifted[bb, :table.shape[1] - cut[bb] // 16] = table[bb, cut[bb] // 16:]
    kw = dict(sm_scale=w.sm_scale, k_scale=b.k_scale, v_scale=b.v_scale)
    o1, l1 = B.attn_decode_lse(b.q, b.k_pages, b.v_pages, b.page_table, torch.from_numpy(cut.astype(np.int32)).to(DEV), **kw)
    o2, l2 = B.attn_decode_lse(b.q, b.k_pages, b.v_pages, torch.from_numpy(shifted).to(DEV),
                               torch.from_numpy((lens - cut).astype(np.int32)).to(DEV), **kw)
    out, lse = B.attn_merge(o1, l1, o2, l2)
    torch.cuda.synchronize()
    assert torch.isneginf(l1[0]).all() and (o1[0] == 0).all()
    check(out, oracle_decode(b), qd, "merged halves")
    _check_lse(lse, _oracle_lse(b, None), qd, "merged halves")
    # the oracle's merge of the oracle's halves says the same about these very halves
    ref_o, ref_l = O.merge_states(o1.double().cpu().numpy(), l1.double().cpu().numpy(), o2.double().cpu().numpy(), l2.double().cpu().numpy())
    check(out, ref_o, qd, "merge kernel alone")
    _check_lse(lse, ref_l, qd, "merge kernel alone")


def test_merge_edges():
    g = torch.Generator().manual_seed(5)
    o1 = torch.randn((7, 4, 128), generator=g).to(torch.bfloat16).to(DEV)
    o2 = torch.randn((7, 4, 128), generator=g).to(torch.bfloat16).to(DEV)
    l1 = torch.randn((7, 4), generator=g).mul(5).to(DEV)
    l2 = torch.randn((7, 4), generator=g).mul(5).to(DEV)
    l1[2] = float("-inf"); l2[3] = float("-inf"); l1[5] = float("-inf"); l2[5] = float("-inf")
    o1[2] = float("nan")                                   # an empty side is never looked at
    out, lse = B.attn_merge(o1, l1, o2, l2)
    torch.cuda.synchronize()
    assert torch.equal(out[2], o2[2]) and torch.equal(lse[2], l2[2])
    assert torch.equal(out[3], o1[3]) and torch.equal(lse[3], l1[3])
    assert (out[5] == 0).all() and torch.isneginf(lse[5]).all()
    ref_o, ref_l = O.merge_states(torch.nan_to_num(o1.double()).cpu().numpy(), l1.double().cpu().numpy(), o2.double().cpu().numpy(),
                                  l2.double().cpu().numpy())
    check(out, ref_o, "bf16", "merge")
    _check_lse(lse, ref_l, "bf16", "merge")
    # in place: the result may overwrite one of its inputs
    keep = out.clone()
    B.attn_merge(o1, l1, o2, l2, out=o1, lse_out=l1)
    torch.cuda.synchronize()
    assert torch.equal(o1, keep) and torch.equal(l1, lse)


def test_profiling_reports_the_append_kernels_clock():
    # while profiling is on the MFMA append kernel counts cycles and constant-rate ticks inside its tiles
    b = W.build(W.Workload("clk", 8, 32, 8, 128, "bf16", "bf16", ("uniform", 200, 900), qlen=("uniform", 64, 300), ctx_is_prefix=True,
                           seed=W.BASE_SEED + 76), DEV)
    plain = gpu_append(b)
    B.profile_enable(True)
    try:
        B.profile_read()
        B.profile_append_clock()
        timed = gpu_append(b)
        torch.cuda.synchronize()
        assert len(B.profile_read()) == 1
        mhz = B.profile_append_clock()
        assert 300.0 < mhz < 2600.0, mhz
        assert B.profile_append_clock() == 0.0          # read and cleared
    finally:
        B.profile_enable(False)
    assert torch.equal(plain, timed)
