"""Pins of the KV-write oracle (CPU only): the E4M3 encoder against the format's definition and a
library cast, the write itself against the attention oracle's own paging routine, a library-built
recipe for fresh pages, and closed-form error bounds for the rescale rule."""
import numpy as np
import torch

from oracle import attention as A
from oracle import kv_write as KW


def _bf16_bits(x):
    return (torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy()).view(np.uint16)


def _bf16_val(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------- encoder

def test_encoder_inverts_the_decoder_on_every_code():
    codes = np.arange(256, dtype=np.uint8)
    vals = A.e4m3fn_to_float64(codes)
    ok = ~np.isnan(vals)
    assert ok.sum() == 254
    back = KW.float32_to_e4m3fn(vals[ok].astype(np.float32))
    assert np.array_equal(back, codes[ok])          # includes -0 -> 0x80 and both 448s


def test_encoder_ties_go_to_the_even_mantissa_and_nearest_otherwise():
    pos = np.arange(0, 0x7E, dtype=np.uint8)         # every adjacent pair of non-negative finite codes
    lo, hi = A.e4m3fn_to_float64(pos), A.e4m3fn_to_float64(pos + 1)
    mid = ((lo + hi) / 2).astype(np.float32)         # exactly representable in float32
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)
    want = np.where(pos % 2 == 0, pos, pos + 1)
    assert np.array_equal(KW.float32_to_e4m3fn(mid), want)
    assert np.array_equal(KW.float32_to_e4m3fn(-mid), want | 0x80)
    below = np.nextafter(mid, np.float32(0)).astype(np.float32)
    above = np.nextafter(mid, np.float32(np.inf)).astype(np.float32)
    assert np.array_equal(KW.float32_to_e4m3fn(below), pos)
    assert np.array_equal(KW.float32_to_e4m3fn(above), pos + 1)


def test_encoder_clamps_and_marks_nan():
    x = np.array([448, 449, 464, 465, 1e9, np.inf, -449, -1e30, np.nan], dtype=np.float32)
    assert KW.float32_to_e4m3fn(x).tolist() == [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE, 0x7F]
    tiny = np.array([2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -9, 0.0, 1e-30], dtype=np.float32)
    assert KW.float32_to_e4m3fn(tiny).tolist() == [0, 1, 1, 0, 0]   # half the smallest subnormal ties to zero


def test_encoder_agrees_with_the_library_cast_inside_its_range():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(200000) * s for s in (1e-3, 0.02, 1.0, 30.0, 150.0)]).astype(np.float32)
    x = x[np.abs(x) <= 464]                          # the library cast turns larger magnitudes into NaN instead of clamping
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(KW.float32_to_e4m3fn(x), lib)


# ---------------------------------------------------------------- the write

def _layout(rng, ctx, hkv, d, spare=3):
    """Random physical placement: pools with `spare` extra pages, a permuted page table."""
    pages_of = (np.asarray(ctx) + 15) // 16
    n_pages = int(pages_of.sum()) + spare
    perm = rng.permutation(n_pages)
    table = np.full((len(ctx), max(1, int(pages_of.max()))), -1, dtype=np.int32)
    k = 0
    for b, n in enumerate(pages_of):
        table[b, :n] = perm[k:k + n]
        k += n
    return n_pages, table


def test_stamped_rows_come_back_through_the_attention_oracles_gather_and_nothing_else_moves():
    rng = np.random.default_rng(1)
    hkv, d = 3, 8
    ctx = np.array([37, 16, 5, 64, 1, 0])
    qn = np.array([21, 16, 2, 33, 1, 0])             # crosses pages, fills one exactly, starts mid page, empty row
    n_pages, table = _layout(rng, ctx, hkv, d)
    sentinel = np.float32(-777.0)
    pools = [np.full((n_pages, hkv, 16, d), sentinel, dtype=np.float32) for _ in range(2)]
    total = int(qn.sum())
    offs = np.concatenate([[0], np.cumsum(qn)])
    stamp = lambda pool, b, pos, h, dd: np.float32(pool * 1e6 + b * 1e5 + pos * 100 + h * 10 + dd)
    new = [np.zeros((total, hkv, d), dtype=np.float32) for _ in range(2)]
    for pool in range(2):
        for b in range(len(ctx)):
            for i in range(qn[b]):
                for h in range(hkv):
                    for dd in range(d):
                        new[pool][offs[b] + i, h, dd] = stamp(pool, b, ctx[b] - qn[b] + i, h, dd)
    kp, vp, _, _ = KW.kv_write(new[0], new[1], qn, ctx, table, pools[0], pools[1], src_dtype="f32", kv_dtype="f32")
    written = np.zeros((n_pages, hkv, 16), dtype=bool)
    for pool, pages in enumerate((kp, vp)):
        for b in range(len(ctx)):
            for h in range(hkv):
                got = A.gather_tokens(pages, table, b, h, ctx[b], "f32", raw=True)
                for pos in range(ctx[b]):
                    if pos >= ctx[b] - qn[b]:
                        want = [stamp(pool, b, pos, h, dd) for dd in range(d)]
                        assert got[pos].tolist() == want, (pool, b, h, pos)
                        written[table[b, pos // 16], h, pos % 16] = True
                    else:
                        assert (got[pos] == sentinel).all()
        assert (pages[~written] == sentinel).all()   # unused pages, older slots, slots past the context
    assert (pools[0] == sentinel).all()              # inputs untouched


def test_bf16_pools_take_the_source_bits():
    rng = np.random.default_rng(2)
    hkv, d = 2, 16
    ctx, qn = np.array([40, 9]), np.array([40, 3])
    n_pages, table = _layout(rng, ctx, hkv, d)
    k_new = _bf16_bits(rng.standard_normal((43, hkv, d)))
    v_new = _bf16_bits(rng.standard_normal((43, hkv, d)))
    zero = np.zeros((n_pages, hkv, 16, d), dtype=np.uint16)
    kp, vp, _, _ = KW.kv_write(k_new, v_new, qn, ctx, table, zero, zero, src_dtype="bf16", kv_dtype="bf16")
    assert np.array_equal(A.gather_tokens(kp, table, 0, 1, 40, "bf16", raw=True), k_new[:40, 1])
    assert np.array_equal(A.gather_tokens(vp, table, 1, 0, 9, "bf16", raw=True)[6:], v_new[40:, 0])


def test_fresh_fp8_pages_match_the_recipe_built_from_library_routines():
    # whole trajectories written into empty pools: per page and pool, scale = absmax of the live slots / 448
    # (1 for an all-zero page) and codes = library cast of x / scale
    rng = np.random.default_rng(3)
    hkv, d = 4, 32
    ctx = np.array([50, 16, 7])
    n_pages, table = _layout(rng, ctx, hkv, d)
    total = int(ctx.sum())
    xk = (rng.standard_normal((total, hkv, d)) * rng.choice([0.01, 1.0, 40.0], size=(total, 1, 1))).astype(np.float32)
    xv = rng.standard_normal((total, hkv, d)).astype(np.float32)
    xv[50:66] = 0                                    # an all-zero page
    kb, vb = _bf16_bits(xk), _bf16_bits(xv)
    codes0 = np.full((n_pages, hkv, 16, d), 0x7F, dtype=np.uint8)
    s0 = np.full(n_pages, np.nan, dtype=np.float32)
    kp, vp, ks, vs = KW.kv_write(kb, vb, ctx, ctx, table, codes0, codes0, src_dtype="bf16", kv_dtype="fp8_e4m3", k_scale=s0, v_scale=s0)
    offs = np.concatenate([[0], np.cumsum(ctx)])
    for bits, pages, scales in ((kb, kp, ks), (vb, vp, vs)):
        x = torch.from_numpy(_bf16_val(bits))
        for b in range(len(ctx)):
            for p in range((ctx[b] + 15) // 16):
                live = x[offs[b] + 16 * p: offs[b] + min(ctx[b], 16 * p + 16)]             # [slots, Hkv, D]
                amax = live.abs().max()
                s = amax / 448.0 if amax > 0 else torch.tensor(1.0)
                want = (live / s).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                phys = table[b, p]
                assert np.float32(scales[phys]) == np.float32(s)
                assert np.array_equal(np.swapaxes(pages[phys, :, :live.shape[0], :], 0, 1), want)
                assert (pages[phys, :, live.shape[0]:, :] == 0x7F).all()


def test_fp8_error_bound_and_scale_rule_when_a_partly_filled_page_grows():
    rng = np.random.default_rng(4)
    hkv, d = 2, 64
    table = np.array([[0]], dtype=np.int32)
    codes0 = np.zeros((1, hkv, 16, d), dtype=np.uint8)
    s_init = np.ones(1, dtype=np.float32)
    x1 = rng.standard_normal((5, hkv, d)).astype(np.float32)
    b1 = _bf16_bits(x1); x1 = _bf16_val(b1)
    kp, vp, ks, vs = KW.kv_write(b1, b1, [5], [5], table, codes0, codes0, src_dtype="bf16", kv_dtype="fp8_e4m3", k_scale=s_init, v_scale=s_init)
    s1 = ks[0]
    assert s1 == np.float32(np.abs(x1).max() / np.float32(448))

    def err_ok(x, codes, s, rounds):
        deq = A.e4m3fn_to_float64(codes) * np.float64(s)
        q = np.abs(x.astype(np.float64) / np.float64(s))
        # half a grid step per rounding: step is 2**-3 relative to the binade, 2**-9 absolute under 2**-6
        bound = rounds * np.float64(s) * np.maximum(q * 2.0 ** -4, 2.0 ** -10) * 1.001
        return np.all(np.abs(deq - x) <= bound)

    assert err_ok(np.swapaxes(x1, 0, 1), kp[0, :, :5], s1, 1)
    # smaller second chunk: scale and old codes stay, new codes use the old scale
    x2 = (0.25 * rng.standard_normal((4, hkv, d))).astype(np.float32)
    b2 = _bf16_bits(x2); x2 = _bf16_val(b2)
    kp2, _, ks2, _ = KW.kv_write(b2, b2, [4], [9], table, kp, vp, src_dtype="bf16", kv_dtype="fp8_e4m3", k_scale=ks, v_scale=vs)
    assert ks2[0] == s1 and np.array_equal(kp2[0, :, :5], kp[0, :, :5])
    assert np.array_equal(np.swapaxes(kp2[0, :, 5:9], 0, 1), KW.float32_to_e4m3fn(x2 / s1))
    # larger third chunk: scale grows to its absmax / 448, old codes are re-quantised (two roundings), nothing exceeds 448
    x3 = (10.0 * rng.standard_normal((7, hkv, d))).astype(np.float32)
    b3 = _bf16_bits(x3); x3 = _bf16_val(b3)
    kp3, _, ks3, _ = KW.kv_write(b3, b3, [7], [16], table, kp2, vp, src_dtype="bf16", kv_dtype="fp8_e4m3", k_scale=ks2, v_scale=vs)
    assert ks3[0] == np.float32(np.abs(x3).max() / np.float32(448)) and ks3[0] > s1
    assert err_ok(np.swapaxes(x3, 0, 1), kp3[0, :, 9:16], ks3[0], 1)
    assert err_ok(np.swapaxes(np.concatenate([x1, x2]), 0, 1), kp3[0, :, :9], ks3[0], 2.2)
    assert (np.abs(A.e4m3fn_to_float64(kp3)) <= 448).all()
    # the attention oracle reads the result back through the same scales
    got = A.gather_tokens(kp3, table, 0, 1, 16, "fp8_e4m3", scale=ks3)
    assert np.abs(got - np.concatenate([x1, x2, x3])[:, 1]).max() <= 2.2 * ks3[0] * 448 * 2.0 ** -4


def test_token_by_token_equals_one_chunk_when_the_scale_never_grows():
    rng = np.random.default_rng(5)
    hkv, d = 2, 16
    table = np.array([[1, 0]], dtype=np.int32)
    x = rng.standard_normal((20, hkv, d)).astype(np.float32)
    x[0] *= 8; x[16] *= 8                              # first token of each page carries the page's absmax
    bits = _bf16_bits(x)
    codes0 = np.zeros((2, hkv, 16, d), dtype=np.uint8)
    s0 = np.ones(2, dtype=np.float32)
    whole = KW.kv_write(bits, bits, [20], [20], table, codes0, codes0, src_dtype="bf16", kv_dtype="fp8_e4m3", k_scale=s0, v_scale=s0)
    state = (codes0, codes0, s0, s0)
    for t in range(20):
        state = KW.kv_write(bits[t:t + 1], bits[t:t + 1], [1], [t + 1], table, state[0], state[1], src_dtype="bf16",
                            kv_dtype="fp8_e4m3", k_scale=state[2], v_scale=state[3])
    for a, b in zip(whole, state):
        assert np.array_equal(a, b)
