"""Pins for the CPU oracle against what mathematics and library routines fix.

The paper prints no formula, worked example or error bound for the engine's attention
step (Section 6.1 only names the decode / prefill step; Section 3.1 the two phases), so
every pin here is a closed form, an invariant, a brute-force sum or a library routine
on the special case it covers.  Each is chosen to fail under a plausible slip: a
dropped softmax scale, a wrong head-group map, an off-by-one causal boundary, swapped
K/V scales, a transposed operand, a wrong page/slot index.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention as O
from oracle import brute
from paper_2512_22560_amd import workloads as W
from tests.helpers import bf16_bits, oracle_args, tiny


def _single(q, k, v, page_table=None, ctx_lens=None, **kw):
    """Decode on hand-made float32 pools: k, v given as [L, D] for one trajectory, one head."""
    L, D = k.shape
    n_pages = (L + 15) // 16
    kp = np.full((n_pages, 1, 16, D), np.nan, dtype=np.float32)
    vp = np.full((n_pages, 1, 16, D), np.nan, dtype=np.float32)
    kp.reshape(-1, D)[:L] = k
    vp.reshape(-1, D)[:L] = v
    table = np.arange(n_pages, dtype=np.int32)[None, :]
    return O.attn_decode(q.reshape(1, 1, D).astype(np.float32), kp, vp, table, np.array([L]),
                         sm_scale=kw.get("sm_scale", 1.0), q_dtype="f32", kv_dtype="f32")[0, 0]


# ---------------------------------------------------------------- storage formats

def test_e4m3_definition_points():
    t = O.e4m3fn_to_float64(np.arange(256, dtype=np.uint8))
    assert t[0x00] == 0.0 and t[0x80] == 0.0 and math.copysign(1.0, t[0x80]) == -1.0
    assert t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9      # subnormals
    assert t[0x08] == 2.0 ** -6                                   # smallest normal
    assert t[0x38] == 1.0 and t[0x3C] == 1.5 and t[0x40] == 2.0
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0                 # largest finite
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])                # the only NaN codes
    assert np.isfinite(np.delete(t, [0x7F, 0xFF])).all()          # no infinities
    assert np.all(np.diff(t[:0x7F]) > 0)                          # strictly increasing codes
    assert np.array_equal(t[0x80:0xFF], -t[0x00:0x7F])


def test_e4m3_matches_library_cast():
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    got = O.e4m3fn_to_float64(codes.numpy())
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])


def test_bf16_matches_library_cast():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = O.decode_storage(bits, "bf16")
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])


# ---------------------------------------------------------------- closed forms

def test_single_key_returns_its_value_exactly():
    rng = np.random.default_rng(1)
    q, k, v = rng.standard_normal(8), rng.standard_normal((1, 8)), rng.standard_normal((1, 8))
    out = _single(q, k.astype(np.float32), v.astype(np.float32), sm_scale=0.3)
    assert np.array_equal(out, v.astype(np.float32)[0].astype(np.float64))


@pytest.mark.parametrize("L", [2, 16, 17, 40])
def test_identical_keys_give_mean_of_values(L):
    rng = np.random.default_rng(2)
    q = rng.standard_normal(8)
    k = np.repeat(rng.standard_normal((1, 8)), L, axis=0).astype(np.float32)
    v = rng.standard_normal((L, 8)).astype(np.float32)
    np.testing.assert_allclose(_single(q, k, v), v.astype(np.float64).mean(axis=0), rtol=0, atol=1e-15)
    # a zero query does the same whatever the keys are
    k2 = rng.standard_normal((L, 8)).astype(np.float32)
    np.testing.assert_allclose(_single(np.zeros(8), k2, v), v.astype(np.float64).mean(axis=0), rtol=0, atol=1e-15)


@pytest.mark.parametrize("scale", [1.0, 0.125, 1 / math.sqrt(64)])
def test_two_keys_logistic_closed_form(scale):
    # keys 0 and b*e1, query a*e1: weights are (1 - s, s) with s = logistic(scale * a * b)
    a, b = 3.0, 0.75
    q = np.array([a, 0, 0, 0.0])
    k = np.array([[0, 0, 0, 0.0], [b, 0, 0, 0]], dtype=np.float32)
    v = np.array([[1, 2, 3, 4.0], [-2, 0, 5, 8]], dtype=np.float32)
    s = 1.0 / (1.0 + math.exp(-float(np.float32(scale)) * a * b))
    v64 = v.astype(np.float64)
    expect = (1 - s) * v64[0] + s * v64[1]
    np.testing.assert_allclose(_single(q, k, v, sm_scale=scale), expect, rtol=0, atol=1e-15)


def test_geometric_weights_closed_form():
    # keys t*e1 (t = 0..L-1), query a*e1, values t: out = sum t r^t / sum r^t with r = exp(scale a)
    L, a, scale = 37, 0.5, 0.25
    k = np.zeros((L, 4), dtype=np.float32); k[:, 0] = np.arange(L)
    v = np.zeros((L, 4), dtype=np.float32); v[:, 2] = np.arange(L)
    r = math.exp(scale * a)
    expect = sum(t * r ** t for t in range(L)) / sum(r ** t for t in range(L))
    out = _single(np.array([a, 0, 0, 0.0]), k, v, sm_scale=scale)
    assert abs(out[2] - expect) < 1e-12 and out[0] == 0 and out[1] == 0 and out[3] == 0


def test_argmax_limit():
    rng = np.random.default_rng(3)
    q = rng.standard_normal(8).astype(np.float32)
    k = np.zeros((20, 8), dtype=np.float32); k[13] = 200.0 * q
    v = rng.standard_normal((20, 8)).astype(np.float32)
    np.testing.assert_allclose(_single(q, k, v), v[13].astype(np.float64), atol=1e-30)


def test_shift_of_all_keys_changes_nothing_and_values_enter_linearly():
    rng = np.random.default_rng(4)
    q = rng.standard_normal(8).astype(np.float32)
    k = rng.standard_normal((33, 8)).astype(np.float32)
    v1 = rng.integers(-8, 8, (33, 8)).astype(np.float32)
    v2 = rng.integers(-8, 8, (33, 8)).astype(np.float32)
    base = _single(q, k, v1)
    c = np.float32(2.0) * np.ones(8, dtype=np.float32)            # k + c is exact here? not needed:
    shifted = _single(q, (k.astype(np.float64) + c).astype(np.float32), v1)
    np.testing.assert_allclose(shifted, base, atol=1e-6)          # float32 rounding of k + c only
    np.testing.assert_allclose(_single(q, k, v1 + v2), base + _single(q, k, v2), atol=1e-13)
    assert np.all(base <= v1.max(axis=0) + 1e-12) and np.all(base >= v1.min(axis=0) - 1e-12)


# ---------------------------------------------------------------- paging, heads

def test_gqa_heads_map_to_kv_heads_in_contiguous_groups():
    b = tiny(hq=12, hkv=3, d=8, ctx=("uniform", 5, 50), seed=11)
    args = oracle_args(b)
    v = args["v_pages"].copy()
    for g in range(3):
        v[:, g] = float(g + 1)
    args["v_pages"] = v
    out = O.attn_decode(W.raw_numpy(b.q), **args)
    for h in range(12):
        np.testing.assert_allclose(out[:, h, :], h // 4 + 1, atol=1e-14)


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16", "fp8_e4m3"])
def test_physical_page_permutation_is_invisible(kv_dtype):
    q_dtype = "f32" if kv_dtype == "f32" else "bf16"
    b = tiny(q_dtype=q_dtype, kv_dtype=kv_dtype, ctx=("uniform", 1, 90), seed=12)
    args = oracle_args(b)
    base = O.attn_decode(W.raw_numpy(b.q), **args)
    rng = np.random.default_rng(0)
    n = b.num_pages
    perm = rng.permutation(n)                     # new id of old page p is perm[p]
    inv = np.argsort(perm)
    args2 = dict(args)
    args2["k_pages"] = args["k_pages"][inv]
    args2["v_pages"] = args["v_pages"][inv]
    if kv_dtype == "fp8_e4m3":
        args2["k_scale"] = args["k_scale"][inv]
        args2["v_scale"] = args["v_scale"][inv]
    pt = args["page_table"].copy()
    live = pt >= 0
    pt[live] = perm[pt[live]]
    args2["page_table"] = pt
    assert np.array_equal(O.attn_decode(W.raw_numpy(b.q), **args2), base)


def test_gather_reads_slots_in_logical_order_and_never_the_poison():
    b = tiny(ctx=("uniform", 1, 60), seed=13, d=8)
    args = oracle_args(b)
    kp = args["k_pages"].copy()
    # stamp every live element with (trajectory, token) so the expected gather is known in closed form
    for bb, L in enumerate(b.ctx_lens_host.tolist()):
        for t in range(L):
            kp[args["page_table"][bb, t // 16], :, t % 16, :] = 1000 * bb + t
    for bb, L in enumerate(b.ctx_lens_host.tolist()):
        got = O.gather_tokens(kp, args["page_table"], bb, 1, L, "f32")
        assert np.array_equal(got[:, 0], 1000.0 * bb + np.arange(L))
    out = O.attn_decode(W.raw_numpy(b.q), **args)
    assert np.isfinite(out).all()                 # NaN slots and -1 entries were never read
    with pytest.raises(IndexError):
        O.gather_tokens(kp, args["page_table"], 0, 0, int(b.ctx_lens_host[0]) + 16, "f32")


def test_fp8_scales_apply_per_page_to_the_right_pool():
    b = tiny(q_dtype="bf16", kv_dtype="fp8_e4m3", ctx=("uniform", 20, 80), seed=14)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    got = O.attn_decode(q, **args)
    # dequantise with the library cast, then run the float32 path
    def deq(codes, scale):
        x = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32)
        x = x * torch.from_numpy(scale).view(-1, 1, 1, 1)
        return torch.nan_to_num(x, nan=float("nan")).numpy()
    args32 = dict(args, kv_dtype="f32", k_scale=None, v_scale=None,
                  k_pages=deq(args["k_pages"], args["k_scale"]), v_pages=deq(args["v_pages"], args["v_scale"]))
    np.testing.assert_allclose(got, O.attn_decode(q, **args32), atol=1e-6)   # float32 rounding of code * scale
    swapped = dict(args, k_scale=args["v_scale"], v_scale=args["k_scale"])
    assert np.abs(O.attn_decode(q, **swapped) - got).max() > 1e-4


# ---------------------------------------------------------------- brute force and library cross-checks

@pytest.mark.parametrize("q_dtype,kv_dtype", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")])
def test_decode_agrees_with_scalar_c_twin(q_dtype, kv_dtype):
    for L in (1, 15, 16, 17, 31, 32, 33):
        b = tiny(batch=2, hq=4, hkv=2, d=8, q_dtype=q_dtype, kv_dtype=kv_dtype, ctx=("const", L), seed=20 + L)
        args = oracle_args(b)
        q = W.raw_numpy(b.q)
        np.testing.assert_allclose(O.attn_decode(q, **args), brute.paged_attention(q, None, **args), atol=1e-13)
    b = tiny(batch=5, hq=6, hkv=2, d=16, q_dtype=q_dtype, kv_dtype=kv_dtype, ctx=("uniform", 0, 120), seed=21)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    np.testing.assert_allclose(O.attn_decode(q, **args), brute.paged_attention(q, None, **args), atol=1e-13)


@pytest.mark.parametrize("q_dtype,kv_dtype", [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")])
def test_append_agrees_with_scalar_c_twin(q_dtype, kv_dtype):
    b = tiny(batch=4, hq=4, hkv=2, d=8, q_dtype=q_dtype, kv_dtype=kv_dtype, ctx=("uniform", 0, 50),
             qlen=("uniform", 0, 35), ctx_is_prefix=True, seed=22)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    got = O.attn_append(q, b.q_lens_host, **args)
    ref = brute.paged_attention(q, b.q_lens_host, **args)
    assert got.shape == ref.shape and got.shape[0] == b.q_lens_host.sum()
    np.testing.assert_allclose(got, ref, atol=1e-13)


def _contiguous(b, args, bb, g):
    """K, V of (trajectory, kv head) as float64 torch tensors, gathered by a plain loop."""
    L = int(b.ctx_lens_host[bb])
    ks, vs = [], []
    for t in range(L):
        p = int(args["page_table"][bb, t // 16])
        ks.append(torch.from_numpy(args["k_pages"][p, g, t % 16].astype(np.float64)))
        vs.append(torch.from_numpy(args["v_pages"][p, g, t % 16].astype(np.float64)))
    return torch.stack(ks), torch.stack(vs)


def test_against_library_sdpa_decode_causal_and_prefixed():
    sdpa = torch.nn.functional.scaled_dot_product_attention
    # (a) decode == unmasked SDPA of one query over the whole context
    b = tiny(batch=3, hq=4, hkv=2, d=16, ctx=("uniform", 1, 70), seed=30)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    out = O.attn_decode(q, **args)
    for bb in range(3):
        for h in range(4):
            k, v = _contiguous(b, args, bb, h // 2)
            ref = sdpa(torch.from_numpy(q[bb, h].astype(np.float64))[None, None], k[None], v[None], scale=b.workload.sm_scale)
            np.testing.assert_allclose(out[bb, h], ref[0, 0].numpy(), atol=1e-7)
    # (b) empty prefix, chunk = whole context: textbook causal self-attention
    b = tiny(batch=2, hq=2, hkv=1, d=16, ctx=("const", 0), qlen=("uniform", 3, 40), ctx_is_prefix=True, seed=31)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    out = O.attn_append(q, b.q_lens_host, **args)
    row = 0
    for bb in range(2):
        n = int(b.q_lens_host[bb])
        for h in range(2):
            k, v = _contiguous(b, args, bb, 0)
            ref = sdpa(torch.from_numpy(q[row:row + n, h].astype(np.float64))[None], k[None], v[None], is_causal=True,
                       scale=b.workload.sm_scale)
            np.testing.assert_allclose(out[row:row + n, h], ref[0].numpy(), atol=1e-7)
        row += n
    # (c) cached prefix + chunk: SDPA with the boolean mask "key position <= query position"
    b = tiny(batch=2, hq=2, hkv=1, d=16, ctx=("uniform", 5, 40), qlen=("uniform", 2, 20), ctx_is_prefix=True, seed=32)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    out = O.attn_append(q, b.q_lens_host, **args)
    row = 0
    for bb in range(2):
        n, L = int(b.q_lens_host[bb]), int(b.ctx_lens_host[bb])
        mask = torch.zeros(n, L, dtype=torch.bool)
        for i in range(n):
            mask[i, : L - n + i + 1] = True
        for h in range(2):
            k, v = _contiguous(b, args, bb, 0)
            ref = sdpa(torch.from_numpy(q[row:row + n, h].astype(np.float64))[None], k[None], v[None], attn_mask=mask,
                       scale=b.workload.sm_scale)
            np.testing.assert_allclose(out[row:row + n, h], ref[0].numpy(), atol=1e-7)
        row += n


# ---------------------------------------------------------------- causal boundary, append vs decode

def test_causal_boundary_by_perturbation():
    b = tiny(batch=1, hq=2, hkv=1, d=8, ctx=("const", 21), qlen=("const", 9), ctx_is_prefix=True, seed=40)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    L, n = 30, 9
    assert int(b.ctx_lens_host[0]) == L
    base = O.attn_append(q, b.q_lens_host, **args)
    for i in range(n):
        pos = L - n + i
        for t, must_change in ((pos, True), (pos + 1, False)):
            if t >= L:
                continue
            a2 = dict(args)
            vp = args["v_pages"].copy()
            vp[args["page_table"][0, t // 16], 0, t % 16, :] += 1.0
            a2["v_pages"] = vp
            changed = np.abs(O.attn_append(q, b.q_lens_host, **a2)[i] - base[i]).max() > 1e-9
            assert changed == must_change, (i, t)


@pytest.mark.parametrize("q_dtype,kv_dtype", [("f32", "f32"), ("bf16", "fp8_e4m3")])
def test_append_row_equals_decode_at_truncated_context(q_dtype, kv_dtype):
    b = tiny(batch=3, hq=4, hkv=2, d=8, q_dtype=q_dtype, kv_dtype=kv_dtype, ctx=("uniform", 0, 40),
             qlen=("uniform", 1, 20), ctx_is_prefix=True, seed=41)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    out = O.attn_append(q, b.q_lens_host, **args)
    row = 0
    for bb in range(3):
        n, L = int(b.q_lens_host[bb]), int(b.ctx_lens_host[bb])
        for i in range(n):
            a2 = dict(args, page_table=args["page_table"][bb:bb + 1], ctx_lens=np.array([L - n + i + 1]))
            dec = O.attn_decode(q[row + i:row + i + 1], **a2)
            np.testing.assert_allclose(out[row + i], dec[0], atol=1e-13)
        row += n
    # all chunks of length one: the append call is the decode call
    b = tiny(batch=4, hq=4, hkv=2, d=8, q_dtype=q_dtype, kv_dtype=kv_dtype, ctx=("uniform", 1, 60), seed=42)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    np.testing.assert_allclose(O.attn_append(q, b.q_lens_host, **args), O.attn_decode(q, **args), atol=1e-13)


def test_empty_context_and_empty_chunk():
    b = tiny(batch=4, hq=2, hkv=1, d=8, ctx=("const", 0), seed=43)
    args = oracle_args(b)
    assert not O.attn_decode(W.raw_numpy(b.q), **args).any()
    out = O.attn_append(np.zeros((0, 2, 8), np.float32), np.zeros(4, int), **args)
    assert out.shape == (0, 2, 8)


# ---------------------------------------------------------------- split-K identity and plans

@pytest.mark.parametrize("chunk", [16, 48, 64, 1000])
def test_split_then_combine_equals_unsplit(chunk):
    b = tiny(batch=2, hq=2, hkv=1, d=16, ctx=("uniform", 100, 300), seed=50)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    whole = O.attn_decode(q, **args)
    for bb in range(2):
        L = int(b.ctx_lens_host[bb])
        k = O.gather_tokens(args["k_pages"], args["page_table"], bb, 0, L, "f32")
        v = O.gather_tokens(args["v_pages"], args["page_table"], bb, 0, L, "f32")
        for h in range(2):
            parts = [O.partial_softmax_attention(q[bb, h].astype(np.float64), k[s:s + chunk], v[s:s + chunk],
                                                 b.workload.sm_scale) for s in range(0, L, chunk)]
            ms, ls, os_ = zip(*parts)
            np.testing.assert_allclose(O.combine_partials(ms, ls, os_), whole[bb, h], atol=1e-12)


def test_split_plan_covers_every_block_once_in_equal_runs():
    rng = np.random.default_rng(5)
    for rows_per_b, workers, lens in ((8, 64, rng.integers(0, 4000, 30)), (4, 2048, rng.integers(1, 300, 10)),
                                      (8, 16, np.array([0, 0])), (2, 7, rng.integers(0, 90, 50)),
                                      (1, 5, np.array([0, 33, 0, 0, 1, 64, 0]))):
        per, total, starts, segs = O.split_plan(lens, rows_per_b, workers)
        n_blocks = (lens + 31) // 32
        assert total == rows_per_b * n_blocks.sum() and per == max(1, -(-total // workers))
        seen = {}
        by_worker = {}
        for w, b, r, k, cnt, slot in segs.tolist():
            assert cnt > 0 and k + cnt <= n_blocks[b]
            for kk in range(k, k + cnt):
                assert (b, r, kk) not in seen
                seen[(b, r, kk)] = w
            by_worker.setdefault(w, []).append((b, r, k, cnt, slot))
        assert len(seen) == total                                   # every block exactly once
        for w, pieces in by_worker.items():
            assert sum(p[3] for p in pieces) == min(per, total - w * per)   # equal runs
            assert (starts[w][0], starts[w][1] >> 20, starts[w][1] & 0xFFFFF) == pieces[0][:3]
            assert starts[w][2] == lens[pieces[0][0]] and starts[w][3] == sum(p[3] for p in pieces)
            for i, (b, r, k, cnt, slot) in enumerate(pieces):
                whole = k == 0 and cnt == n_blocks[b]
                assert slot == (-1 if whole else (0 if i == 0 else 1))
                if 0 < i < len(pieces) - 1:
                    assert whole                                    # only the ends of a run can be partial
        assert sorted(by_worker) == list(range(len(by_worker)))     # workers are used in order
        assert all(starts[w][0] == -1 for w in range(len(by_worker), workers))


def test_append_tile_plan_covers_every_chunk_row_once_most_expensive_tiles_first():
    rng = np.random.default_rng(6)
    cases = [(rng.integers(0, 300, 40), 64, False), (rng.integers(0, 40, 25), 16, True), (np.array([0, 1, 1, 0, 5]), 4, True),
             (np.array([7]), 1, False), (np.zeros(6, dtype=np.int64), 16, False), (rng.integers(1, 9, 30), 256, False)]
    for q_lens, tile_tokens, skip_unit in cases:
        ctx = q_lens + rng.integers(0, 5000, len(q_lens))
        ctx[: len(ctx) // 3] = ctx[0]                                # ties in the ranking
        tiles = O.append_tile_plan(q_lens, ctx, tile_tokens, skip_unit_chunks=skip_unit)
        covered = {b: [] for b in range(len(q_lens))}
        for b, start, rows in tiles.tolist():
            assert 0 < rows <= tile_tokens and start % tile_tokens == 0 and start + rows <= q_lens[b]
            assert rows == tile_tokens or start + rows == q_lens[b]  # only a chunk's last tile is short
            covered[b].extend(range(start, start + rows))
        for b, n in enumerate(q_lens.tolist()):
            want = [] if (skip_unit and n == 1) else list(range(n))
            assert sorted(covered[b]) == want                        # every row of every chunk exactly once
        # cost order: contexts never increase along the list, a trajectory's tiles are adjacent, last tile first
        bs = tiles[:, 0].tolist()
        assert all(ctx[bs[i]] >= ctx[bs[i + 1]] for i in range(len(bs) - 1))
        assert all(bs[i] < bs[i + 1] for i in range(len(bs) - 1) if bs[i] != bs[i + 1] and ctx[bs[i]] == ctx[bs[i + 1]])
        firsts = [i for i in range(len(bs)) if i == 0 or bs[i] != bs[i - 1]]
        assert len(firsts) == len(set(bs))
        for i in range(len(bs) - 1):
            if bs[i] == bs[i + 1]:
                assert tiles[i, 1] == tiles[i + 1, 1] + tile_tokens
    # beyond the ranking limit the list is in index order
    q_lens = rng.integers(0, 3, 50)
    tiles = O.append_tile_plan(q_lens, rng.integers(2, 99, 50), 2, rank_limit=49)
    assert tiles[:, 0].tolist() == sorted(tiles[:, 0].tolist())


# ---------------------------------------------------------------- softmax denominators and the merge of two ranges

def _lse_single(q, k, **kw):
    L, D = k.shape
    n_pages = (L + 15) // 16
    kp = np.full((n_pages, 1, 16, D), np.nan, dtype=np.float32)
    kp.reshape(-1, D)[:L] = k
    table = np.arange(n_pages, dtype=np.int32)[None, :]
    return O.attn_lse(q.reshape(1, 1, D).astype(np.float32), None, kp, table, np.array([L]), sm_scale=kw.get("sm_scale", 1.0),
                      q_dtype="f32", kv_dtype="f32")[0, 0]


def test_lse_closed_forms():
    rng = np.random.default_rng(60)
    q, k = rng.standard_normal(8).astype(np.float32), rng.standard_normal((1, 8)).astype(np.float32)
    z = float(np.float64(np.float32(0.37)) * (np.float64(k[0]) @ np.float64(q)))
    assert abs(_lse_single(q, k, sm_scale=0.37) - z * math.log2(math.e)) < 1e-12          # one key: log2 exp(z)
    for L in (2, 17, 100):                                                                 # L equal keys: + log2 L
        assert abs(_lse_single(q, np.repeat(k, L, axis=0), sm_scale=0.37) - (z * math.log2(math.e) + math.log2(L))) < 1e-12


def test_lse_matches_library_logsumexp_with_causal_rows():
    from scipy.special import logsumexp
    b = tiny(batch=3, hq=4, hkv=2, d=16, ctx=("uniform", 20, 90), qlen=("uniform", 0, 9), seed=61, ctx_is_prefix=True)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    got = O.attn_lse(q, b.q_lens_host, args["k_pages"], args["page_table"], args["ctx_lens"], sm_scale=args["sm_scale"],
                     q_dtype="f32", kv_dtype="f32")
    row = 0
    for bb in range(3):
        n, L = int(b.q_lens_host[bb]), int(b.ctx_lens_host[bb])
        for i in range(n):
            for h in range(4):
                k = O.gather_tokens(args["k_pages"], args["page_table"], bb, h // 2, L, "f32")
                z = [float(np.float64(np.float32(args["sm_scale"])) * sum(float(k[t, e]) * float(q[row, h, e]) for e in range(16)))
                     for t in range(L - n + i + 1)]                                        # scores by plain loops
                assert abs(got[row, h] - logsumexp(z) / math.log(2.0)) < 1e-10
            row += 1
    assert row == got.shape[0]


def test_merging_two_ranges_equals_attention_over_their_union():
    b = tiny(batch=4, hq=4, hkv=2, d=16, ctx=("uniform", 40, 200), seed=62)
    args = oracle_args(b)
    q = W.raw_numpy(b.q)
    whole = O.attn_decode(q, **args)
    lse_args = dict(sm_scale=args["sm_scale"], q_dtype="f32", kv_dtype="f32")
    whole_lse = O.attn_lse(q, None, args["k_pages"], args["page_table"], args["ctx_lens"], **lse_args)
    # range 1: the first S_b tokens (whole pages); range 2: the rest, through a table shifted by S_b / 16 entries
    cut = np.array([16, 32, 0, 48])
    table = args["page_table"]
    shifted = np.zeros_like(table)
    for bb in range(4):
        shifted[bb, :table.shape[1] - cut[bb] // 16] = table[bb, cut[bb] // 16:]
    a1 = dict(args, ctx_lens=cut)
    a2 = dict(args, ctx_lens=b.ctx_lens_host - cut, page_table=shifted)
    o1, o2 = O.attn_decode(q, **a1), O.attn_decode(q, **a2)
    l1 = O.attn_lse(q, None, a1["k_pages"], a1["page_table"], a1["ctx_lens"], **lse_args)
    l2 = O.attn_lse(q, None, a2["k_pages"], a2["page_table"], a2["ctx_lens"], **lse_args)
    assert np.all(np.isneginf(l1[2])) and np.all(o1[2] == 0)                               # an empty range: weight 0
    o, lse = O.merge_states(o1, l1, o2, l2)
    np.testing.assert_allclose(o, whole, atol=1e-12)
    np.testing.assert_allclose(lse, whole_lse, atol=1e-12)
    # both sides empty: zeros and -inf; merging is symmetric
    o0, l0 = O.merge_states(o1[2:3], l1[2:3], o1[2:3], l1[2:3])
    assert np.all(o0 == 0) and np.all(np.isneginf(l0))
    o_sw, l_sw = O.merge_states(o2, l2, o1, l1)
    np.testing.assert_allclose(o_sw, o, atol=1e-15)
    np.testing.assert_allclose(l_sw, lse, atol=1e-15)
