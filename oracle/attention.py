"""Plain float64 definition of paged-KV attention (decode and observation-append).

TEST INFRASTRUCTURE ONLY -- see the package docstring.  numpy only, no blocking,
no online softmax, no fusion: gather the trajectory's tokens through its page
table, convert every stored number exactly to float64, take scaled dot products,
mask, softmax, weight the values.

Storage formats (raw arrays, decoded here and nowhere else in this package):
  "f32"       numpy float32
  "bf16"      numpy uint16 holding the upper half of an IEEE binary32 pattern
  "fp8_e4m3"  numpy uint8 holding OCP 8-bit E4M3 ("fn": no infinity, S.1111.111 is
              NaN, bias 7, subnormal step 2**-9, largest finite 448), to be
              multiplied by a per-page float32 scale (one scale per physical page
              of each pool, covering all KV heads and slots of the page)

Layouts: q [B or total_q, Hq, D]; pools [num_pages, Hkv, page_size, D];
page_table [B, max_pages] int32; ctx_lens [B]; q_lens [B].

Definition (trajectory b, query head h, chunk row i of n_b; decode is n_b = 1):
  g   = h // (Hq // Hkv)                       query heads map to KV heads in
                                               contiguous groups
  pos = L_b - n_b + i                          absolute position of the query; the
                                               chunk's own K/V are already in the
                                               cache, ctx_lens counts them
  token t in [0, pos] lives in physical page page_table[b, t // page_size],
  slot t % page_size
  z_t = sm_scale * <q, k_t>;  w_t = exp(z_t - max z);  out = sum w_t v_t / sum w_t
  L_b = 0 gives a zero row.
This is the engine step of Section 6.1 (decode or prefill for a batch of requests)
with the history served from the prefix cache (Section 7.1); causal inside the
chunk, full attention to the cached prefix.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "e4m3fn_to_float64",
    "decode_storage",
    "gather_tokens",
    "attn_decode",
    "attn_append",
    "partial_softmax_attention",
    "combine_partials",
    "split_plan",
    "append_tile_plan",
]


def e4m3fn_to_float64(codes: np.ndarray) -> np.ndarray:
    """Decode OCP FP8 E4M3 bytes by the format's definition (OCP 8-bit Floating
    Point Specification, E4M3: 1 sign, 4 exponent bits with bias 7, 3 mantissa
    bits, no infinities, exponent 15 with mantissa 7 is NaN)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where((c >> 7) & 1, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    subnormal = (m / 8.0) * 2.0 ** (-6)
    mag = np.where(e == 0, subnormal, normal)
    mag = np.where((e == 15) & ((c & 0x7) == 7), np.nan, mag)
    return sign * mag


def decode_storage(raw: np.ndarray, dtype: str) -> np.ndarray:
    """Exact conversion of a stored array (without any page scale) to float64."""
    if dtype == "f32":
        a = np.asarray(raw)
        if a.dtype != np.float32:
            raise TypeError("f32 storage must be numpy float32")
        return a.astype(np.float64)
    if dtype == "bf16":
        a = np.asarray(raw)
        if a.dtype != np.uint16:
            raise TypeError("bf16 storage must be numpy uint16 bit patterns")
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype == "fp8_e4m3":
        a = np.asarray(raw)
        if a.dtype != np.uint8:
            raise TypeError("fp8_e4m3 storage must be numpy uint8 codes")
        return e4m3fn_to_float64(a)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def gather_tokens(pages, page_table, b, g, length, dtype, scale=None, raw=False):
    """Logical tokens [0, length) of trajectory b, KV head g, in order: [length, D].

    Token t is read from physical page page_table[b, t // page_size], slot
    t % page_size; table entries past the last live page and slots past the
    context length are never touched.  raw=True returns the stored elements
    unconverted (for byte-exact comparison of the paging logic)."""
    page_size = pages.shape[2]
    t = np.arange(int(length), dtype=np.int64)
    phys = np.asarray(page_table)[b, t // page_size].astype(np.int64)
    slot = t % page_size
    if length and (phys.min() < 0 or phys.max() >= pages.shape[0]):
        raise IndexError("page table entry outside the pool")
    rows = pages[phys, g, slot, :]
    if raw:
        return rows
    x = decode_storage(rows, dtype)
    if dtype == "fp8_e4m3":
        if scale is None:
            raise ValueError("fp8_e4m3 pools need a per-page scale")
        x = x * np.asarray(scale, dtype=np.float32).astype(np.float64)[phys][:, None]
    return x


def _softmax_rows(z: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """Row-wise softmax over the visible entries (others get weight 0)."""
    zm = np.where(visible, z, -np.inf)
    top = zm.max(axis=1, keepdims=True)
    w = np.where(visible, np.exp(zm - top), 0.0)
    return w / w.sum(axis=1, keepdims=True)


def attn_append(q_chunk, q_lens, k_pages, v_pages, page_table, ctx_lens, *, sm_scale,
                q_dtype, kv_dtype, k_scale=None, v_scale=None) -> np.ndarray:
    """Observation-append attention: rows of trajectory b are packed consecutively in
    q_chunk (n_b = q_lens[b] rows each, in batch order).  Returns float64
    [total_q, Hq, D], un-rounded."""
    q = decode_storage(q_chunk, q_dtype)
    total_q, hq, d = q.shape
    hkv = k_pages.shape[1]
    if hq % hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    group = hq // hkv
    q_lens = np.asarray(q_lens, dtype=np.int64)
    ctx_lens = np.asarray(ctx_lens, dtype=np.int64)
    if q_lens.sum() != total_q:
        raise ValueError("q_lens do not add up to the packed row count")
    if np.any(q_lens > ctx_lens):
        raise ValueError("a chunk cannot be longer than its context")
    out = np.zeros((total_q, hq, d), dtype=np.float64)
    scale = np.float64(np.float32(sm_scale))
    row0 = 0
    for b in range(len(q_lens)):
        n, length = int(q_lens[b]), int(ctx_lens[b])
        if n == 0:
            continue
        pos = length - n + np.arange(n)                       # absolute query positions
        visible = np.arange(length)[None, :] <= pos[:, None]  # [n, L]
        for g in range(hkv):
            k = gather_tokens(k_pages, page_table, b, g, length, kv_dtype, k_scale)
            v = gather_tokens(v_pages, page_table, b, g, length, kv_dtype, v_scale)
            for h in range(g * group, (g + 1) * group):
                z = scale * (q[row0:row0 + n, h, :] @ k.T)    # [n, L]
                out[row0:row0 + n, h, :] = _softmax_rows(z, visible) @ v
        row0 += n
    return out


def attn_decode(q, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, q_dtype, kv_dtype,
                k_scale=None, v_scale=None) -> np.ndarray:
    """Decode attention: one query row per trajectory, at position L_b - 1 (its own
    K/V already cached).  Float64 [B, Hq, D].  Written out separately from the append
    routine (not as a call to it) so that the two can be checked against each other."""
    qf = decode_storage(q, q_dtype)
    bsz, hq, d = qf.shape
    hkv = k_pages.shape[1]
    if hq % hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    group = hq // hkv
    out = np.zeros((bsz, hq, d), dtype=np.float64)
    scale = np.float64(np.float32(sm_scale))
    for b in range(bsz):
        length = int(ctx_lens[b])
        if length == 0:
            continue
        for g in range(hkv):
            k = gather_tokens(k_pages, page_table, b, g, length, kv_dtype, k_scale)
            v = gather_tokens(v_pages, page_table, b, g, length, kv_dtype, v_scale)
            for h in range(g * group, (g + 1) * group):
                z = scale * (k @ qf[b, h, :])                 # [L]
                w = np.exp(z - z.max())
                out[b, h, :] = (w / w.sum()) @ v
    return out


def attn_lse(q, q_lens, k_pages, page_table, ctx_lens, *, sm_scale, q_dtype, kv_dtype, k_scale=None) -> np.ndarray:
    """Base-2 logarithm of every row's softmax denominator, lse = log2 sum_t exp(z_t) over the tokens the row sees
    (z_t = sm_scale <q, k_t>), float64 [rows, Hq]; -inf for a row that sees no token.  q_lens None: decode rows
    (row b at position L_b - 1), else chunk rows as in attn_append.  It is what a caller needs, next to the
    output, to merge attention over two disjoint token ranges (merge_states below): the engine's step over a
    context that is split across calls, or across GPUs that each hold a slice of the pages."""
    qf = decode_storage(q, q_dtype)
    rows, hq, d = qf.shape
    hkv = k_pages.shape[1]
    group = hq // hkv
    ctx_lens = np.asarray(ctx_lens, dtype=np.int64)
    q_lens = np.ones(len(ctx_lens), dtype=np.int64) if q_lens is None else np.asarray(q_lens, dtype=np.int64)
    scale = np.float64(np.float32(sm_scale))
    lse = np.full((rows, hq), -np.inf, dtype=np.float64)
    row0 = 0
    for b in range(len(ctx_lens)):
        n, length = int(q_lens[b]), int(ctx_lens[b])
        for g in range(hkv):
            k = gather_tokens(k_pages, page_table, b, g, length, kv_dtype, k_scale)
            for i in range(n):
                seen = length - n + i + 1                   # tokens [0, seen) are visible to chunk row i
                if seen <= 0:
                    continue
                for h in range(g * group, (g + 1) * group):
                    z = scale * (k[:seen] @ qf[row0 + i, h, :])
                    top = z.max()
                    lse[row0 + i, h] = (top + np.log(np.exp(z - top).sum())) / np.log(2.0)
        row0 += n
    return lse


def merge_states(o1, lse1, o2, lse2):
    """Attention over the union of two disjoint token ranges from the results over each: with weights
    w_i = 2^lse_i the output is (w_1 o_1 + w_2 o_2) / (w_1 + w_2) and the denominator's logarithm
    log2(w_1 + w_2); a side that saw nothing (lse = -inf) has weight 0, and rows where both saw nothing give
    zeros and -inf.  o [rows, Hq, D], lse [rows, Hq]; returns (o, lse) in float64."""
    o1, o2 = np.asarray(o1, dtype=np.float64), np.asarray(o2, dtype=np.float64)
    l1, l2 = np.asarray(lse1, dtype=np.float64), np.asarray(lse2, dtype=np.float64)
    top = np.maximum(l1, l2)
    safe = np.where(np.isfinite(top), top, 0.0)
    w1, w2 = np.exp2(l1 - safe), np.exp2(l2 - safe)        # exp2(-inf) = 0
    tot = w1 + w2
    with np.errstate(divide="ignore", invalid="ignore"):
        o = np.where(tot[..., None] > 0, (w1[..., None] * o1 + w2[..., None] * o2) / tot[..., None], 0.0)
        lse = np.where(tot > 0, safe + np.log2(tot), -np.inf)
    return o, lse


def partial_softmax_attention(q_row, k, v, sm_scale):
    """Attention of one query over one slice of tokens, returned as the triple the
    split-K partition exchanges: (m, l, o) with m the slice's largest score, l the
    sum of exp(z - m) and o the slice's own normalised output."""
    z = np.float64(np.float32(sm_scale)) * (k @ q_row)
    m = z.max()
    w = np.exp(z - m)
    l = w.sum()
    return m, l, (w @ v) / l


def combine_partials(ms, ls, os_):
    """Merge per-slice triples: with M = max m_s and a_s = exp(m_s - M) l_s the result
    is sum a_s o_s / sum a_s, which equals the softmax over the union of slices."""
    ms = np.asarray(ms, dtype=np.float64)
    ls = np.asarray(ls, dtype=np.float64)
    os_ = np.asarray(os_, dtype=np.float64)
    a = np.exp(ms - ms.max()) * ls
    return (a[:, None] * os_).sum(axis=0) / a.sum()


# ----------------------------------------------------------------------------------
# Integer structure of the partition over the KV length (compared bit for bit with the
# library's plan).  The rule is stated here by brute enumeration of the block sequence.
# ----------------------------------------------------------------------------------

def split_plan(ctx_lens, rows_per_b, workers, block_tokens=32):
    """Decode partition.  Trajectory b has n_b = ceil(L_b / block_tokens) blocks; the rows
    (b, r), r in [0, rows_per_b), are laid end to end with b outermost, n_b blocks each; the
    resulting sequence of T blocks is dealt to the workers in equal contiguous runs of
    per = max(1, ceil(T / workers)) blocks.  Returns (per, T, starts, segments): starts is
    int32 [workers, 4] with (b, r << 20 | block, L_b, blocks in the run) for the block each run
    begins at ((-1, 0, 0, 0) for workers without blocks); segments is int32 [n, 6] with one line per maximal piece of a row
    inside one run, in worker order: (worker, b, r, first block, block count, slot) where slot
    is -1 if the piece is the whole row, else 0 if it is the first piece of the run, else 1."""
    lens = np.asarray(ctx_lens, dtype=np.int64)
    n_blocks = (lens + block_tokens - 1) // block_tokens
    # global position of every block: rows in (b, r) order
    rows = [(b, r) for b in range(len(lens)) for r in range(rows_per_b) if n_blocks[b] > 0]
    seq = [(b, r, k) for (b, r) in rows for k in range(int(n_blocks[b]))]
    total = len(seq)
    per = max(1, -(-total // workers))
    starts = np.zeros((workers, 4), dtype=np.int32)
    starts[:, 0] = -1
    segments = []
    for w in range(workers):
        run = seq[w * per:(w + 1) * per]
        if not run:
            continue
        b, r, k = run[0]
        starts[w] = (b, (r << 20) | k, lens[b], len(run))
        pieces = []
        for (b, r, k) in run:
            if pieces and pieces[-1][0] == b and pieces[-1][1] == r:
                pieces[-1][3] += 1
            else:
                pieces.append([b, r, k, 1])
        for i, (b, r, k, cnt) in enumerate(pieces):
            whole = k == 0 and cnt == n_blocks[b]
            segments.append((w, b, r, k, cnt, -1 if whole else (0 if i == 0 else 1)))
    return per, total, starts, np.asarray(segments, dtype=np.int32).reshape(-1, 6)


def append_tile_plan(q_lens, ctx_lens, tile_tokens, rank_limit=4096, skip_unit_chunks=False):
    """Append work list, in the order the workgroups take it.  Each chunk is cut into tiles of
    tile_tokens query tokens counted from its first token (so only its last tile can be short).
    A tile's cost grows with the context of its trajectory and with its position in the chunk, and
    tiles are handed out in list order, so the list starts with the expensive ones: trajectories by
    context length, longest first (equal lengths: lower index first), and within a chunk the last
    tile first.  Batches of more than rank_limit trajectories are listed in index order instead.
    With skip_unit_chunks (the mixed step, where one-token chunks are decode rows) chunks of one
    token contribute no tile.  Returns int32 [n_tiles, 3] of (b, first row in the chunk, rows)."""
    q = np.asarray(q_lens, dtype=np.int64).tolist()
    ctx = np.asarray(ctx_lens, dtype=np.int64).tolist()
    order = list(range(len(q)))
    if len(q) <= rank_limit:
        order.sort(key=lambda b: (-ctx[b], b))
    tiles = []
    for b in order:
        if skip_unit_chunks and q[b] == 1:
            continue
        starts = list(range(0, q[b], tile_tokens))
        for start in reversed(starts):
            tiles.append((b, start, min(tile_tokens, q[b] - start)))
    return np.asarray(tiles, dtype=np.int32).reshape(-1, 3)
