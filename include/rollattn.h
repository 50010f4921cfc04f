/*
 * librollattn -- batched attention over a paged KV cache for multi-turn rollouts,
 * hand-written for gfx950 (MI355X).  C ABI, plain pointers and sizes only.
 *
 * The operation is the inference engine's per-step attention during the rollout
 * stage: every engine step runs a decode or a prefill step for a batch of requests
 * (Section 6.1, inference worker loop, "Step Wise Command Processing"); decode is the
 * memory-bandwidth-bound phase and prefill the compute-bound one (Section 3.1,
 * "Stage Computation"); with prefix caching on (Section 7.1, "Evaluation Setup") the
 * history of a multi-turn trajectory stays cached, so a new turn only prefills the
 * observation chunk on top of it.  The paper names these phases and their workload
 * shape; the result itself is textbook softmax attention:
 *
 *   trajectory b, query head h, chunk row i of n_b (decode: n_b = 1)
 *   g   = h / (Hq / Hkv)                         KV head of query head h
 *   pos = L_b - n_b + i                          position of the query token; the
 *                                                chunk's own K/V are already cached and
 *                                                counted in L_b = ctx_lens[b]
 *   token t in [0, pos] lives in physical page page_table[b][t / 16], slot t % 16
 *   out = sum_t softmax_t(sm_scale * <q, k_t>) v_t ,   an all-zero row when L_b = 0
 *
 * Memory.  All array arguments are DEVICE pointers unless marked "host".  The caller
 * owns every buffer; the library allocates nothing, frees nothing and keeps no state
 * between calls apart from the optional profiling events below (created by
 * rollattn_profile_enable, never by an attention call) and the built-in scratch array of
 * attn_decode_static.  Inputs are only
 * read; `out` and `workspace` are the only memory written (kv_write writes the pools and the
 * page scales instead).  Every device pointer must
 * be 16-byte aligned.  Layouts are dense row-major:
 *   q, out        [rows][Hq][D]                 rows = B (decode) or total_q (append)
 *   k_pages,
 *   v_pages       [num_pages][Hkv][16][D]       one page table serves both pools
 *   page_table    [B][max_pages_per_seq] int32  entries past ceil(L_b/16)-1 are never
 *                                               read, nor are slots >= L_b % 16 of a
 *                                               trajectory's last page
 *   k_scale,
 *   v_scale       [num_pages] float             FP8 pools only: element = code * scale
 *                                               of its physical page (per pool)
 * Supported element types: q/out F32 with kv F32 (D = 64 or 128); q/out BF16 with kv
 * BF16 or FP8_E4M3 (OCP E4M3, no infinities, max 448; D = 64 or 128; page scales must be
 * positive and finite, as absmax / 448 is).  Accumulation is float.  Hq / Hkv may be any positive integer (at most 256 for BF16 attn_append).
 *
 * Execution.  Calls enqueue kernels on `hip_stream` (a hipStream_t passed as void*,
 * NULL = the default stream) and return without synchronising; nothing is copied to
 * the host.  Two calls that share a workspace must be ordered on one stream.
 *
 * Errors.  Every entry point returns 0 on success or a negative rollattn_status.
 * All argument checks run on the host before anything is launched, so they behave
 * the same without a GPU.  Contents of device arrays are not checked: a page id
 * outside [0, num_pages) or L_b > 16 * max_pages_per_seq is undefined behaviour.
 */
#ifndef ROLLATTN_H
#define ROLLATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ROLLATTN_F32 = 0,
  ROLLATTN_BF16 = 1,
  ROLLATTN_FP8_E4M3 = 2
} rollattn_dtype;

typedef enum {
  ROLLATTN_OK = 0,
  ROLLATTN_EINVAL = -1,     /* null pointer, negative size, NULL descriptor            */
  ROLLATTN_ESHAPE = -2,     /* Hq % Hkv != 0, unsupported head_dim or page_size,
                               num_pages * Hkv >= 2^31                                 */
  ROLLATTN_EDTYPE = -3,     /* unsupported q/kv type pair, FP8 without scales          */
  ROLLATTN_EALIGN = -4,     /* a device pointer is not 16-byte aligned                 */
  ROLLATTN_EWORKSPACE = -5, /* workspace smaller than rollattn_workspace_bytes()       */
  ROLLATTN_EHIP = -6,       /* a HIP call failed; text via rollattn_last_hip_error()   */
  ROLLATTN_ELIMIT = -7      /* attn_decode_static: the batch needs more scratch than the
                               built-in array of rollattn_static_scratch_bytes() holds */
} rollattn_status;

typedef struct {
  int32_t batch;             /* B >= 0                                              */
  int32_t num_q_heads;       /* Hq                                                  */
  int32_t num_kv_heads;      /* Hkv, Hq % Hkv == 0                                  */
  int32_t head_dim;          /* D, 64 or 128                                        */
  int32_t page_size;         /* 16                                                  */
  int32_t max_pages_per_seq; /* row stride of page_table, >= 1                      */
  int64_t num_pages;         /* physical pool size                                  */
  int32_t q_dtype;           /* rollattn_dtype of q and out                         */
  int32_t kv_dtype;          /* rollattn_dtype of both pools                        */
  float sm_scale;            /* softmax scale, e.g. 1/sqrt(D)                       */
  const float *k_scale;      /* device [num_pages], FP8 only, else NULL             */
  const float *v_scale;      /* device [num_pages], FP8 only, else NULL             */
} rollattn_desc;

/* Decode step: one query token per trajectory at position L_b - 1 (Section 3.1, the
 * bandwidth-bound phase; Section 6.1, the engine's decode step).  The KV range of each
 * trajectory is partitioned over wavefronts by a plan computed on the device from
 * ctx_lens alone (never from page ids) and partial results are merged with the
 * log-sum-exp rule in a fixed order, so results are reproducible bit for bit and do not
 * depend on where pages sit physically.
 *   q [B][Hq][D], out [B][Hq][D], ctx_lens [B] int32 (device).
 * B == 0 succeeds without a launch. */
int attn_decode(const rollattn_desc *desc, const void *q, const void *k_pages, const void *v_pages,
                const int32_t *page_table, const int32_t *ctx_lens, void *out, void *workspace,
                size_t workspace_bytes, void *hip_stream);

/* attn_decode for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit for bit
 * the same result as attn_decode, but the plan and the split partials live in an array that is part of the
 * library's code object (rollattn_static_scratch_bytes() = 36 MiB, held by every GPU the library runs on until
 * the process ends) instead of a caller's workspace.  The call allocates and frees nothing.  A descriptor whose
 * decode workspace (rollattn_workspace_bytes(desc, batch), which grows by 4 bytes per trajectory) exceeds the
 * array is refused with ROLLATTN_ELIMIT before anything is launched: BF16/FP8 D = 128 fits up to about 800,000
 * trajectories.  Every call on a GPU uses that GPU's one array and nothing in it needs clearing between calls
 * (each call rewrites the plan and every partial it reads), so calls on one GPU must be ordered on one stream or
 * otherwise serialised: two that overlap race.  The array's device address is looked up on the first call on each
 * device (hipGetSymbolAddress, no allocation); rollattn_static_init() does that lookup for the current device
 * ahead of time, e.g. before a stream capture begins. */
int attn_decode_static(const rollattn_desc *desc, const void *q, const void *k_pages, const void *v_pages,
                       const int32_t *page_table, const int32_t *ctx_lens, void *out, void *hip_stream);
size_t rollattn_static_scratch_bytes(void);
int rollattn_static_init(void);

/* Observation-append step: trajectory b contributes n_b = q_lens[b] query rows (its new
 * chunk, packed consecutively in q_chunk in batch order) that attend causally inside the
 * chunk and fully to the cached prefix (Section 3.1, the compute-bound prefill phase, on
 * top of the prefix cache of Section 7.1).  ctx_lens INCLUDES the chunk.  q_offsets is the
 * exclusive scan of q_lens ([B+1], device); total_q = q_offsets[B] and max_q_len >=
 * max n_b are host scalars.  max_q_len only picks the tile shape: when no chunk has
 * more than 128 / (Hq / Hkv) tokens the call uses half-size tiles that two waves share
 * (same result within rounding, faster); a value that understates the longest chunk
 * costs speed, not correctness.  Requires n_b <= L_b.  With every n_b == 1 the result equals attn_decode.
 * total_q == 0 succeeds without a launch. */
int attn_append(const rollattn_desc *desc, const void *q_chunk, const int32_t *q_lens,
                const int32_t *q_offsets, int32_t total_q, int32_t max_q_len, const void *k_pages,
                const void *v_pages, const int32_t *page_table, const int32_t *ctx_lens, void *out,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same two calls with one more output, lse [rows][Hq] float (device): the base-2 logarithm of every row's
 * softmax denominator, log2 sum_t exp(sm_scale <q, k_t>) over the tokens the row sees; -inf for a row that sees
 * none.  Next to `out` it is what merges attention over two disjoint token ranges (attn_merge): a context whose
 * pages are split across calls, or across GPUs that each hold a slice of them -- every multi-turn trajectory
 * keeps growing (Section 2.1), and the longest ones are the ones a single cache cannot hold. */
int attn_decode_lse(const rollattn_desc *desc, const void *q, const void *k_pages, const void *v_pages,
                    const int32_t *page_table, const int32_t *ctx_lens, void *out, float *lse, void *workspace,
                    size_t workspace_bytes, void *hip_stream);
int attn_append_lse(const rollattn_desc *desc, const void *q_chunk, const int32_t *q_lens,
                    const int32_t *q_offsets, int32_t total_q, int32_t max_q_len, const void *k_pages,
                    const void *v_pages, const int32_t *page_table, const int32_t *ctx_lens, void *out,
                    float *lse, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Merge of two results over disjoint token ranges, row by row: with w_i = 2^lse_i,
 *   out = (w_1 o_1 + w_2 o_2) / (w_1 + w_2),   lse_out = log2(w_1 + w_2)   (lse_out may be NULL)
 * which is the attention over the union of the ranges.  A side with lse = -inf has weight 0 (its o is not
 * looked at); where both are -inf the row is zero and lse_out -inf.  o_1, o_2, out: [rows][Hq][D] of
 * desc->q_dtype (only num_q_heads, head_dim and q_dtype of desc are used besides the usual checks), lse:
 * [rows][Hq] float.  out may alias o_1 or o_2.  No workspace. */
int attn_merge(const rollattn_desc *desc, int64_t rows, const void *o1, const float *lse1, const void *o2,
               const float *lse2, void *out, float *lse_out, void *hip_stream);

/* One engine step on a mixed batch in one call: during a rollout some requests of the batch generate (one new
 * token) while others have just received an observation and prefill it (Section 6.1, the inference worker takes
 * a decode or a prefill step per request; Section 3.1, the two phases).  Arguments as attn_append, with the
 * rows of ALL trajectories packed in q: a trajectory with q_lens[b] == 1 is a decode row and goes through the
 * decode path (planned over those trajectories only), one with q_lens[b] > 1 through the append path, one with
 * q_lens[b] == 0 contributes nothing.  The result is that of attn_append on the same arguments, and row for row
 * bit-identical to what attn_decode and attn_append give on the two sub-batches.  The partition into the two
 * kinds is made on the device from q_lens; nothing is copied to the host, so the call can be captured in a HIP
 * graph.  workspace of at least rollattn_step_workspace_bytes(desc, total_q) bytes. */
int attn_step(const rollattn_desc *desc, const void *q, const int32_t *q_lens, const int32_t *q_offsets,
              int32_t total_q, int32_t max_q_len, const void *k_pages, const void *v_pages,
              const int32_t *page_table, const int32_t *ctx_lens, void *out, void *workspace,
              size_t workspace_bytes, void *hip_stream);
size_t rollattn_step_workspace_bytes(const rollattn_desc *desc, int32_t total_q);

/* Decode step for groups of trajectories that share a prompt: rollouts are sampled in groups of
 * group_size per prompt with prefix caching on (Section 7.1), so the members of a group alias the
 * same physical pages for their first tokens.  The result is that of attn_decode on the same
 * arguments (to rounding: the two halves below are each rounded to BF16 before they are merged);
 * the shared range is read once per group for all of the group's query heads instead of once per
 * trajectory.  Trajectories b = j * group_size .. (j + 1) * group_size - 1 form group j; B must be a
 * multiple of group_size.  shared_lens [B / group_size] int32 (device): the caller promises that
 * page_table rows of a group agree on the pages of tokens [0, shared_lens[j]); the library uses
 * S_j = that value, lowered to the group's smallest L_b - 1 and then to a multiple of 32 (S_j = 0
 * is allowed and leaves the plain decode).  Tokens [0, S_j) are attended through the first member's
 * table row for all members (non-causal, all query rows of the group against the same K/V tiles on
 * the matrix cores), tokens [S_j, L_b) per trajectory as in attn_decode, and the two are merged with
 * the log-sum-exp rule.  BF16 queries only (BF16 or FP8 pools).  workspace of at least
 * rollattn_shared_workspace_bytes(desc, group_size) bytes. */
int attn_decode_shared(const rollattn_desc *desc, const void *q, const void *k_pages, const void *v_pages,
                       const int32_t *page_table, const int32_t *ctx_lens, int32_t group_size,
                       const int32_t *shared_lens, void *out, void *workspace, size_t workspace_bytes,
                       void *hip_stream);
size_t rollattn_shared_workspace_bytes(const rollattn_desc *desc, int32_t group_size);

/* KV write, the step before either attention call: every turn of a trajectory appends tokens to its
 * history (Section 2.1), whose KV stays cached (Section 7.1), so the K and V rows of the new tokens
 * (one per trajectory before attn_decode, the chunk before attn_append) are put into the pages.
 * ctx_lens INCLUDES the new tokens, as in attn_append: new row i of trajectory b goes to position
 * L_b - n_b + i, page page_table[b][pos / 16], slot pos % 16, for every KV head.
 *   k_new, v_new [total_q][Hkv][D], elements of desc->q_dtype (F32 or BF16), rows packed in batch
 *   order as q_chunk is; q_offsets [B+1] their exclusive scan; max_q_len >= max n_b (host): it sizes
 *   the launch, so rows of a chunk beyond an understated max_q_len would silently stay unwritten.
 *   Pools of the source type take the rows bit for bit.  FP8 pools (BF16 source) hold E4M3 codes
 *   times one float scale per physical page and pool, k_scale / v_scale [num_pages] (device, read
 *   and written here; desc->k_scale / v_scale are ignored).  Per page that receives new rows in
 *   slots [s0, s1): amax = largest |x| of those rows over all heads; s0 == 0: scale = amax / 448,
 *   or 1 if amax == 0; otherwise scale = max(old scale, amax / 448), and if that raised it the
 *   codes in slots [0, s0) are replaced by enc(dec(code) * old / scale); new codes are
 *   enc(x / scale).  Every product and quotient is one float32 operation, enc rounds to nearest
 *   even after clamping to [-448, 448]: the result is defined bit for bit.
 * A page written here must belong to exactly one trajectory of the batch (shared prefix pages are
 * complete and are never written again); inputs must be finite; B <= 65535.  Pool slots and scales
 * of pages that receive nothing are left untouched.  No workspace; total_q == 0 succeeds without a
 * launch. */
int kv_write(const rollattn_desc *desc, const void *k_new, const void *v_new, const int32_t *q_lens,
             const int32_t *q_offsets, int32_t total_q, int32_t max_q_len, void *k_pages, void *v_pages,
             const int32_t *page_table, const int32_t *ctx_lens, float *k_scale, float *v_scale,
             void *hip_stream);

/* Bytes of workspace either call needs for this descriptor; total_q is the number of
 * query rows (B for decode).  Depends on the descriptor only, never on device data.
 * Returns 0 for an invalid descriptor. */
size_t rollattn_workspace_bytes(const rollattn_desc *desc, int32_t total_q);

/* Paging logic alone (Section 7.1's prefix cache as a data structure): copies logical
 * tokens [0, L_b) of trajectory b, KV head kv_head, unconverted, from `pages` to dst
 * ([L_b][D] elements of kv_dtype, device), reading L_b from ctx_lens on the device. */
int rollattn_debug_gather(const rollattn_desc *desc, const void *pages, const int32_t *page_table,
                          const int32_t *ctx_lens, int32_t b, int32_t kv_head, void *dst,
                          void *hip_stream);

/* What the attention and KV-write calls take on trust, checked on the device for callers that want to be sure
 * before they launch (an index outside a pool is a GPU memory fault, not an error code).  Counts into
 * counts_out (host, int32[4]):
 *   [0] trajectories with L_b outside [0, 16 * max_pages_per_seq]
 *   [1] page-table entries of live pages (page < ceil(L_b / 16)) outside [0, num_pages)
 *   [2] trajectories with n_b outside [0, L_b]                        (only when q_lens is given)
 *   [3] trajectories where q_offsets is not the exclusive scan of q_lens (only when both are given)
 * counts_dev: device int32[4] scratch the caller owns.  Synchronises the stream; returns 0 whenever the check
 * itself ran, whatever it counted. */
int rollattn_debug_check_inputs(const rollattn_desc *desc, const int32_t *page_table, const int32_t *ctx_lens,
                                const int32_t *q_lens, const int32_t *q_offsets, int32_t *counts_dev,
                                int32_t *counts_out, void *hip_stream);

/* Host twin of the decode partition rule, for bit-exact plan tests; runs without a GPU.
 * The rule: each trajectory is cut into blocks of 32 tokens; a "row" is (trajectory b, r) with
 * r = kv_head * tiles + head_tile enumerating KV heads and, when the group is larger than one
 * tile (16 query heads for BF16, 4 for F32), the tiles of the group; rows are laid end to end,
 * b outermost, each with ceil(L_b / 32) blocks; the sequence of T blocks is dealt to the W =
 * rollattn_plan_workers() workers in equal contiguous runs of per = max(1, ceil(T / W)) blocks.
 * ctx_lens_host [B] (host).  Writes per and T, the number of row segments the workers walk to
 * *n_segments and, when segments_out is not NULL, 6 int32 per segment in worker order:
 * (worker, b, r, first block, block count, slot) with slot = -1 when the segment is the whole
 * row (the worker writes the output itself), else the partial slot (0: first segment of the
 * worker's run, 1: its last) handed to the merge.  segments_out must hold
 * 6 * rollattn_plan_capacity(desc) int32. */
int rollattn_debug_plan(const rollattn_desc *desc, const int32_t *ctx_lens_host, int32_t *per_out,
                        int32_t *total_out, int32_t *segments_out, int32_t *n_segments);
int32_t rollattn_plan_capacity(const rollattn_desc *desc);
int32_t rollattn_plan_workers(const rollattn_desc *desc);
/* Testing aid: from now on every decode partition of this process (attn_decode and its variants, the decode rows
 * of attn_step, the private half of attn_decode_shared, rollattn_debug_plan) is cut for min(workers, all) workers
 * instead of all of them; the rest of the launch finds no blocks.  One worker walks every row in turn, a few
 * cut rows at odd places, all of them cut short rows many times: the results must agree whatever the number
 * (Section 3.1's decoding step does not depend on how the context is split).  0 restores the default.  Returns
 * the previous setting.  rollattn_plan_workers() reports the number in force. */
int32_t rollattn_debug_set_decode_workers(int32_t workers);

/* Copies the plan the last attn_decode call left in `workspace` back to the host
 * (synchronises the stream): per, T, and 4 int32 per worker, (b, r << 20 | block, L_b, blocks
 * in its run) for the first block of its run, or (-1, 0, 0, 0) for a worker without blocks.
 * starts_out must hold 4 * rollattn_plan_workers(desc) int32. */
int rollattn_debug_read_plan(const rollattn_desc *desc, const void *workspace, int32_t *per_out,
                             int32_t *total_out, int32_t *starts_out, void *hip_stream);

/* Copies the tile list that the last attn_append call (BF16 queries) left in `workspace` back to the host
 * (synchronises the stream), for bit-exact tests of the append plan.  The rule: every chunk is cut into tiles of
 * max(1, 256 / (Hq / Hkv)) query tokens counted from its first token; the list holds the trajectories by context
 * length, longest first (equal lengths: lower index first; batches of more than 4096 trajectories: index order),
 * and a chunk's tiles last tile first, because workgroups take the list in order and the expensive tiles should
 * start first.  Writes the number of tiles and 2 int32 per tile, (b, first row of the tile in its chunk);
 * tiles_out must hold 2 * rollattn_append_plan_capacity(desc, total_q) int32. */
int rollattn_debug_read_append_plan(const rollattn_desc *desc, const void *workspace, int32_t total_q,
                                    int32_t *n_tiles_out, int32_t *tiles_out, void *hip_stream);
int32_t rollattn_append_plan_capacity(const rollattn_desc *desc, int32_t total_q);
/* attn_step keeps its append tile list at this byte offset of its workspace (the decode part comes first):
 * rollattn_debug_read_append_plan(desc, (char *)workspace + offset, ...) reads the list of a mixed step, in which
 * chunks of one token are decode rows and contribute no tile. */
size_t rollattn_step_append_offset(const rollattn_desc *desc);

/* Optional per-kernel timing.  rollattn_profile_enable(1) creates a pool of 1024 HIP event pairs (the one place
 * where the library creates anything, and only on request); while enabled, attn_decode / attn_append / kv_write
 * bracket their main kernel (not the planning or merge kernels) with a pair from the pool on the call's stream,
 * as long as pairs are left and the stream is not being captured into a graph (events recorded during a capture
 * cannot be read back, so such calls record nothing).  rollattn_profile_read synchronises the recorded events,
 * returns up to `cap` durations in milliseconds, oldest first, and makes the pairs available again. */
int rollattn_profile_enable(int on);
int rollattn_profile_read(float *ms_out, int cap);
/* While profiling is on, the MFMA append kernel also counts, per tile, shader-clock cycles and ticks of the GPU's
 * constant 100 MHz counter (two 8-byte sums in a device variable of the library, on the device that was current
 * when profiling was switched on).  This call synchronises the device, sets *mhz_out (host) to the clock those
 * sums give for all append launches since the last call, 0 if there were none, and clears the sums. */
int rollattn_profile_append_clock(double *mhz_out);

const char *rollattn_status_string(int status);
const char *rollattn_last_hip_error(void);
int rollattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ROLLATTN_H */
