"""Plain definition of the KV write (cache append) that precedes an attention step.

TEST INFRASTRUCTURE ONLY -- see the package docstring.  numpy only; loops over
trajectories and pages, nothing blocked or fused.

What it defines.  Every turn of a multi-turn trajectory appends tokens to the history
(Section 2.1: observations and actions accumulate in the context; Section 7.1: the
history's KV stays cached), so before the engine's attention step the K and V rows of
the new tokens are put into the paged cache: trajectory b brings n_b new tokens (1 for a
decode step, the observation chunk for a prefill step), ctx_lens[b] = L_b already
counts them, and new token i sits at position pos = L_b - n_b + i, i.e. in physical page
page_table[b, pos // 16], slot pos % 16, for every KV head:
    pool[page, head, slot, :] = row (i, head) of the new K (resp. V).
Pools that store the source type (float32 or bf16 bit patterns) take the rows bit for bit.

FP8 pools (E4M3 codes times one float32 scale per physical page and pool, shared by all
heads and slots of the page) need a rule for the scale, which the paper does not give; the
reading taken here, per page p that receives new tokens in slots [s0, s1) and per pool:
    amax   = largest |x| over the new rows of the page, all heads, all dims (float32)
    fresh page (s0 == 0):   scale = amax / 448, or 1 if amax == 0
    partly filled page:     scale = max(old scale, amax / 448); if that exceeds the old
                            scale, the codes already in slots [0, s0) are re-quantised:
                            code <- enc(dec(code) * old_scale / scale)
    new rows:               code = enc(x / scale)
with every product and quotient a single float32 operation, in the order written, and
enc = round to nearest even onto the E4M3 grid after clamping to [-448, 448].  Because the
codes are integers decided by float arithmetic, the precision is part of the definition:
float32, as in the HIP path.  Inputs are finite; a page written here belongs to exactly one
trajectory of the batch (shared prefix pages are complete and never written again).
The paper prints nothing to check this against: parity unpinned by the paper; the pins in
the CPU tests are the format's definition, a library cast, closed-form error bounds and
the stamped-gather test through the attention oracle's own paging routine.
"""
from __future__ import annotations

import numpy as np

__all__ = ["float32_to_e4m3fn", "kv_write"]

PAGE = 16
E4M3_MAX = np.float32(448.0)


def float32_to_e4m3fn(x) -> np.ndarray:
    """Round float32 values to OCP E4M3 codes: nearest, ties to the even mantissa,
    magnitudes above 448 clamp to 448, NaN gives S.1111.111.  Written from the format:
    normal numbers (1 + m/8) * 2**(e-7) for e in 1..15, subnormals (m/8) * 2**-6, so
    the grid step is 2**(E-3) in binade E >= -6 and 2**-9 below 2**-6."""
    x = np.asarray(x, dtype=np.float32)
    a = np.abs(x).astype(np.float64)                       # exact
    sign = (np.signbit(x)).astype(np.uint8) << 7
    nan = np.isnan(a)
    a = np.where(nan, 0.0, np.minimum(a, 448.0))
    # binade of a, not below the subnormal one
    _, ex = np.frexp(a)                                    # a = f * 2**ex, f in [0.5, 1)
    binade = np.maximum(ex - 1, -6)
    step = np.exp2((binade - 3).astype(np.float64))
    r = np.rint(a / step)                                  # rint rounds halves to even; a / step is exact
    v = r * step                                           # may have carried into the next binade
    _, ex2 = np.frexp(v)
    e_field = np.where(v < 2.0 ** -6, 0, ex2 - 1 + 7)
    m_field = np.where(v < 2.0 ** -6, v / 2.0 ** -9, (v / np.exp2((ex2 - 1).astype(np.float64)) - 1.0) * 8.0)
    code = (e_field.astype(np.int64) << 3) | np.rint(m_field).astype(np.int64)
    code = np.where(nan, 0x7F, code).astype(np.uint8)
    return code | sign


def _e4m3fn_to_float32(codes) -> np.ndarray:
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    e = (c >> 3) & 0xF
    m = (c & 7).astype(np.float64)
    mag = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & ((c & 7) == 7), np.nan, mag)
    return (np.where(c >> 7, -mag, mag)).astype(np.float32)   # every E4M3 value is a float32


def _to_float32(raw, dtype):
    if dtype == "f32":
        return np.asarray(raw, dtype=np.float32)
    if dtype == "bf16":
        return (np.asarray(raw, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)
    raise ValueError(dtype)


def kv_write(k_new, v_new, q_lens, ctx_lens, page_table, k_pages, v_pages, *, src_dtype, kv_dtype,
             k_scale=None, v_scale=None):
    """Returns (k_pages, v_pages, k_scale, v_scale) after the write; inputs are not modified.

    k_new, v_new [total_q, Hkv, D] raw (float32, or uint16 bf16 patterns), rows packed in batch
    order; pools [num_pages, Hkv, 16, D] raw (same type as the source, or uint8 E4M3 codes);
    scales float32 [num_pages] for FP8 pools."""
    k_pages, v_pages = np.array(k_pages, copy=True), np.array(v_pages, copy=True)
    fp8 = kv_dtype == "fp8_e4m3"
    if fp8:
        k_scale, v_scale = np.array(k_scale, dtype=np.float32, copy=True), np.array(v_scale, dtype=np.float32, copy=True)
    elif kv_dtype != src_dtype:
        raise ValueError("a pool stores either the source type or E4M3 codes")
    q_lens = np.asarray(q_lens, dtype=np.int64)
    ctx_lens = np.asarray(ctx_lens, dtype=np.int64)
    offs = np.concatenate([[0], np.cumsum(q_lens)])
    for b in range(len(q_lens)):
        n, length = int(q_lens[b]), int(ctx_lens[b])
        if n > length:
            raise ValueError("ctx_lens counts the new tokens")
        first = length - n
        for page_i in range(first // PAGE, (length + PAGE - 1) // PAGE if n else first // PAGE):
            lo, hi = max(first, page_i * PAGE), min(length, (page_i + 1) * PAGE)     # positions written in this page
            s0, s1 = lo - page_i * PAGE, hi - page_i * PAGE
            phys = int(page_table[b, page_i])
            if not 0 <= phys < k_pages.shape[0]:
                raise IndexError("page table entry outside the pool")
            rows = slice(offs[b] + lo - first, offs[b] + hi - first)
            for new, pool, scale in ((k_new, k_pages, k_scale), (v_new, v_pages, v_scale)):
                src = np.asarray(new)[rows]                                           # [slots, Hkv, D]
                if not fp8:
                    pool[phys, :, s0:s1, :] = np.swapaxes(src, 0, 1)
                    continue
                x = _to_float32(src, src_dtype)
                amax = np.float32(np.max(np.abs(x))) if x.size else np.float32(0)
                need = np.float32(amax / E4M3_MAX)
                if s0 == 0:
                    s_new = need if amax > 0 else np.float32(1.0)
                else:
                    s_old = np.float32(scale[phys])
                    s_new = s_old
                    if need > s_old:
                        s_new = need
                        old = _e4m3fn_to_float32(pool[phys, :, :s0, :])
                        old = (old * s_old).astype(np.float32)
                        pool[phys, :, :s0, :] = float32_to_e4m3fn((old / s_new).astype(np.float32))
                scale[phys] = s_new
                pool[phys, :, s0:s1, :] = np.swapaxes(float32_to_e4m3fn((x / s_new).astype(np.float32)), 0, 1)
    return k_pages, v_pages, k_scale, v_scale
