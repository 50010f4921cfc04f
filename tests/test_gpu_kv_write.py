"""KV write on the GPU against its oracle: pools and page scales compared bit for bit (the codes are
integers, the scales single float32 operations), on the stored bytes of the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from oracle import kv_write as KW
from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SRC = {"f32": torch.float32, "bf16": torch.bfloat16}


def _wl(name, batch, hkv, d, q_dtype, kv_dtype, ctx, qlen, seed):
    return W.Workload(name, batch, hkv * 2, hkv, d, q_dtype, kv_dtype, ctx, qlen=qlen, seed=seed, ctx_is_prefix=True)


def _new_rows(b, seed, scale_choices=(0.02, 1.0, 6.0)):
    """Random K / V rows for the batch's chunks, token magnitudes spread over two orders."""
    w = b.workload
    g = torch.Generator(device="cpu").manual_seed(seed)
    shape = (b.total_q, w.num_kv_heads, w.head_dim)
    mag = torch.tensor(scale_choices)[torch.randint(0, len(scale_choices), (b.total_q, 1, 1), generator=g)]
    k = (torch.randn(shape, generator=g) * mag).to(SRC[w.q_dtype]).to(DEV)
    v = (torch.randn(shape, generator=g) * mag.flip(0)).to(SRC[w.q_dtype]).to(DEV)
    return k, v


def _run_both(b, k_new, v_new, kp, vp, ks, vs):
    """One write on the GPU (in place on clones) and in the oracle; returns both states as raw numpy."""
    w = b.workload
    kp_g, vp_g = kp.clone(), vp.clone()
    ks_g, vs_g = (None, None) if ks is None else (ks.clone(), vs.clone())
    B.kv_write(k_new, v_new, b.q_lens, b.q_offsets, kp_g, vp_g, b.page_table, b.ctx_lens,
               max_q_len=int(max(1, b.q_lens_host.max(initial=1))), k_scale=ks_g, v_scale=vs_g)
    torch.cuda.synchronize()
    ref = KW.kv_write(W.raw_numpy(k_new), W.raw_numpy(v_new), b.q_lens_host, b.ctx_lens_host, W.raw_numpy(b.page_table),
                      W.raw_numpy(kp), W.raw_numpy(vp), src_dtype=w.q_dtype, kv_dtype=w.kv_dtype,
                      k_scale=W.raw_numpy(ks), v_scale=W.raw_numpy(vs))
    return (kp_g, vp_g, ks_g, vs_g), ref


def _assert_same(gpu, ref, what):
    for name, g, r in zip(("k_pages", "v_pages", "k_scale", "v_scale"), gpu, ref):
        if r is None:
            continue
        g = W.raw_numpy(g)
        if g.dtype == np.float32:                      # compare bit patterns: NaN sentinels included
            g, r = g.view(np.uint32), np.asarray(r, dtype=np.float32).view(np.uint32)
        bad = np.argwhere(g != r)
        assert bad.size == 0, f"{what}: {name} differs at {bad[:4].tolist()} ({len(bad)} elements)"


@pytest.mark.parametrize("dt,hkv,d", [("bf16", 8, 128), ("bf16", 2, 64), ("f32", 2, 64), ("f32", 1, 128)])
def test_pools_of_the_source_type_take_the_rows_bit_for_bit(dt, hkv, d):
    # prefixes 0..90, chunks 0..70: starts in the middle of a page, spans several pages, empty rows
    b = W.build(_wl("kvw", 9, hkv, d, dt, dt, ("uniform", 0, 90), ("uniform", 0, 70), 301), DEV)
    k_new, v_new = _new_rows(b, 1)
    sentinel_k = torch.full_like(b.k_pages, -3.0)
    sentinel_v = torch.full_like(b.v_pages, 5.0)
    gpu, ref = _run_both(b, k_new, v_new, sentinel_k, sentinel_v, None, None)
    _assert_same(gpu, ref, f"{dt} pool")


@pytest.mark.parametrize("hkv,d", [(4, 128), (8, 128), (1, 64)])
def test_fp8_pools_codes_and_scales_over_three_turns(hkv, d):
    # turn 1 fills fresh and partly filled pages; turn 2 is small (scales stay); turn 3 is large (scales grow, old
    # codes are re-quantised); each turn starts from the previous GPU state, which equals the oracle's bit for bit
    rng = np.random.default_rng(11)
    batch = 7
    w0 = _wl("kvw8", batch, hkv, d, "bf16", "fp8_e4m3", ("uniform", 0, 60), ("uniform", 1, 50), 302)
    b1 = W.build(w0, DEV)
    kp = torch.full_like(b1.k_pages, 0x7F)
    vp = torch.full_like(b1.v_pages, 0x7F)
    ks = torch.full_like(b1.k_scale, float("nan"))
    vs = torch.full_like(b1.v_scale, float("nan"))
    # the prefix of every trajectory first (so that partly filled pages hold real codes), then three chunks
    import dataclasses
    def turn(prev_ctx, qn):
        ctx = prev_ctx + qn
        offs = np.concatenate([[0], np.cumsum(qn)]).astype(np.int32)
        return dataclasses.replace(b1, ctx_lens=torch.from_numpy(ctx.astype(np.int32)).to(DEV), q_lens=torch.from_numpy(qn.astype(np.int32)).to(DEV),
                                   q_offsets=torch.from_numpy(offs).to(DEV), ctx_lens_host=ctx, q_lens_host=qn,
                                   q=torch.empty((int(qn.sum()), w0.num_q_heads, d), dtype=torch.bfloat16, device=DEV))
    total = b1.ctx_lens_host.copy()                    # capacity of each trajectory's page table row
    prefix = total - b1.q_lens_host
    room = b1.q_lens_host
    q1 = np.minimum(room, np.maximum(1, room // 3)); q2 = np.minimum(room - q1, np.maximum(0, room // 3)); q3 = room - q1 - q2
    state = (kp, vp, ks, vs)
    ctx = np.zeros(batch, dtype=np.int64)
    for t, (qn, mags) in enumerate([(prefix, (1.0,)), (q1, (0.5, 2.0)), (q2, (0.01, 0.1)), (q3, (3.0, 40.0))]):
        bt = turn(ctx, qn.astype(np.int64))
        k_new, v_new = _new_rows(bt, 100 + t, mags)
        gpu, ref = _run_both(bt, k_new, v_new, *state)
        _assert_same(gpu, ref, f"fp8 turn {t}")
        state = gpu
        ctx = ctx + qn
    assert np.isfinite(W.raw_numpy(state[2])[np.unique(W.raw_numpy(b1.page_table)[W.raw_numpy(b1.page_table) >= 0])]).all()


def test_fp8_codes_for_bf16_values_of_every_magnitude():
    # The kernel divides every new element by its page's scale; for scales of moderate magnitude it does so with a reciprocal
    # shared by the page and the correction steps of an IEEE division.  Pages whose values sit anywhere between the smallest
    # and the largest bf16 exponents (scales from 2^-135 to 2^118: both sides of the range where the shortcut applies), with
    # arbitrary mantissas, signs, zeros and subnormals below the page's maximum: codes and scales bit for bit.
    rng = np.random.default_rng(77)
    batch, hkv, d = 384, 2, 64
    w0 = _wl("kvw_mag", batch, hkv, d, "bf16", "fp8_e4m3", ("const", 0), ("uniform", 1, 48), 305)
    b = W.build(w0, DEV)
    kp = torch.full_like(b.k_pages, 0x7F); vp = torch.full_like(b.v_pages, 0x7F)
    ks = torch.full_like(b.k_scale, float("nan")); vs = torch.full_like(b.v_scale, float("nan"))
    def rows():
        top = rng.integers(1, 255, size=(b.total_q, 1, 1))                  # biased exponent the token's values reach at most
        exp = np.maximum(top - rng.integers(0, 40, size=(b.total_q, hkv, d)), 0)
        bits = (rng.integers(0, 2, size=exp.shape) << 15) | (exp << 7) | rng.integers(0, 128, size=exp.shape)
        bits[rng.random(exp.shape) < 0.02] = 0
        return torch.from_numpy(bits.astype(np.uint16).view(np.int16)).view(torch.bfloat16).to(DEV)
    k_new, v_new = rows(), rows()
    gpu, ref = _run_both(b, k_new, v_new, kp, vp, ks, vs)
    _assert_same(gpu, ref, "fp8 codes, every magnitude")
    used = np.unique(W.raw_numpy(b.page_table)[W.raw_numpy(b.page_table) >= 0])
    sc = W.raw_numpy(gpu[2])[used]
    sc = sc[np.isfinite(sc)]
    assert (sc < 2.0 ** -100).any() and (sc > 2.0 ** 100).any() and ((sc > 2.0 ** -20) & (sc < 2.0 ** 20)).any()


def test_fp8_decode_step_writes_one_token_per_trajectory():
    b = W.build(W.Workload("kvw1", 300, 8, 4, 128, "bf16", "fp8_e4m3", ("uniform", 1, 200), seed=303), DEV)
    k_new, v_new = _new_rows(b, 5, (0.1, 1.0, 20.0))
    gpu, ref = _run_both(b, k_new, v_new, b.k_pages, b.v_pages, b.k_scale, b.v_scale)
    _assert_same(gpu, ref, "fp8 decode step")


def test_written_chunk_is_what_attention_then_reads():
    # kv_write followed by attn_append on the GPU against the two oracles chained on the CPU
    w = _wl("kvw_attn", 5, 2, 128, "bf16", "fp8_e4m3", ("uniform", 0, 300), ("uniform", 1, 120), 304)
    b = W.build(w, DEV)
    k_new, v_new = _new_rows(b, 9, (0.25, 0.5, 1.0))   # unit-scale values: the attention tolerance is absolute
    gpu, ref = _run_both(b, k_new, v_new, b.k_pages, b.v_pages, b.k_scale, b.v_scale)
    _assert_same(gpu, ref, "fp8 chunk")
    out = B.attn_append(b.q, b.q_lens, b.q_offsets, gpu[0], gpu[1], b.page_table, b.ctx_lens, sm_scale=w.sm_scale,
                        max_q_len=int(b.q_lens_host.max()), k_scale=gpu[2], v_scale=gpu[3])
    want = A.attn_append(W.raw_numpy(b.q), b.q_lens_host, k_pages=ref[0], v_pages=ref[1], page_table=W.raw_numpy(b.page_table),
                         ctx_lens=b.ctx_lens_host, sm_scale=w.sm_scale, q_dtype="bf16", kv_dtype="fp8_e4m3", k_scale=ref[2], v_scale=ref[3])
    check(out, want, "bf16", "attention over the written chunk")


def test_mixed_step_chunks_full_size():
    # the append rows of the mixed FP8 configuration, in the launch shape the bench times: the chunk region of the
    # cache is overwritten with new rows on top of real prefixes (partly filled pages keep or raise their scale)
    b = W.build(W.CONFIGS[5], DEV)
    sub = b.select(b.append_rows())
    k_new, v_new = _new_rows(sub, 13, (0.2, 1.0, 5.0))
    gpu, ref = _run_both(sub, k_new, v_new, sub.k_pages, sub.v_pages, sub.k_scale, sub.v_scale)
    _assert_same(gpu, ref, "mixed step chunks")
