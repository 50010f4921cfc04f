// Internal declarations shared by the host entry points and the HIP kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rollattn.h"

namespace rollattn {

constexpr int kPageSize = 16;
constexpr int kNumCUs = 256;            // MI355X
constexpr int kBlockTokens = 32;        // unit of the decode partition: two pages
constexpr int kMfmaDecodeWgs = 2 * kNumCUs;   // 4 wave-workers each
constexpr int kMfmaHeadTile = 16;       // query heads per MFMA decode row
constexpr int kF32DecodeWgs = 4 * kNumCUs;    // one workgroup-worker each
constexpr int kF32HeadTile = 4;         // query heads per float32 decode row
constexpr int kAppendTileRows = 256;    // query rows (token, head-in-group pairs) per append workgroup
constexpr int kXcds = 8;                // accelerator dies, each with its own L2; workgroups are dealt to them round-robin
constexpr int kTileRecWords = 8;       // append: int32 per tile record (32 bytes: one scalar load)
constexpr int kAppendXcdRun = 16;       // append: consecutive tiles of the list that one XCD takes in a row (one per CU)

// Header words of the plan, at the start of the workspace.
enum PlanWord { kPlanPer = 0, kPlanTotal = 1, kPlanWorkers = 2, kPlanRowsPerB = 3, kPlanTiles = 4, kPlanWords = 64 };

// Byte offsets of the workspace regions (all multiples of 256).
struct WorkspaceLayout {
  int32_t workers;        // decode: number of workers W; append: capacity in query tiles
  int32_t head_tile;      // decode: query heads per row (16 or 4)
  int32_t rows_per_b;     // decode: rows per trajectory = Hkv * ceil(G / head_tile)
  size_t header;          // int32[kPlanWords]
  size_t prefix;          // decode: int32[B + 1] exclusive scan of per-trajectory block counts
  size_t wstart;          // decode: int32[W][4] first (b, row, block) of every worker; append: int32[cap][8] tile records
  size_t partial_ml;      // float[2 W][head_tile][2]   (max in log2 units, sum)
  size_t partial_o;       // float[2 W][head_tile][D]   un-normalised
  size_t total;
};

WorkspaceLayout decode_layout(const rollattn_desc& d);
WorkspaceLayout append_layout(const rollattn_desc& d, int32_t total_q);

// Kernel arguments (passed by value).
struct DecodeArgs {
  const void* q;
  const void* k_pages;
  const void* v_pages;
  const int32_t* page_table;
  const int32_t* ctx_lens;
  void* out;
  const float* k_scale;
  const float* v_scale;
  const int32_t* header;
  const int32_t* prefix;
  const int32_t* wstart;
  float* partial_ml;
  float* partial_o;
  int32_t batch, hq, hkv, group, max_pages, head_tile, rows_per_b;
  float scale_log2;     // sm_scale * log2(e)
  float* lse;           // optional [B][Hq]: log2 of each row's softmax denominator (reference included)
  // Mixed step (both null otherwise): only trajectories with q_lens[b] == 1 are decode rows, the others count
  // as empty here; the query and output row of trajectory b is q_offsets[b] instead of b.
  const int32_t* q_lens;
  const int32_t* q_offsets;
};

struct AppendArgs {
  const void* q;
  const void* k_pages;
  const void* v_pages;
  const int32_t* page_table;
  const int32_t* ctx_lens;
  const int32_t* q_lens;
  const int32_t* q_offsets;
  void* out;
  const float* k_scale;
  const float* v_scale;
  int32_t* header;
  const int32_t* tile_rec;   // [tile_cap][kTileRecWords]: (b, first row of the tile in its chunk, n_b, L_b, q_offsets[b], 0, 0, 0)
  int32_t tile_cap;
  int32_t batch, hq, hkv, group, max_pages, tile_tokens, total_q;
  float scale_log2;
  float* lse;           // optional [total_q][Hq], as in DecodeArgs
  int32_t noncausal;    // every row sees all of [0, L_b); the rows' own tokens are not in that range
  // Optional (profiling): two sums over the launch's tiles as wave 0 sees them, shader-clock cycles and ticks of the
  // constant-rate counter; their ratio is the clock the kernel ran at.
  unsigned long long* clock_sums;
};

// Launchers (defined in the .hip files).  Each returns the hipError_t of its launch.
// workers: how many the partition is cut for; slots >= workers: records written (those past `workers` say "no blocks")
hipError_t launch_plan_decode(const int32_t* ctx_lens, const int32_t* q_lens, int32_t batch, int32_t rows_per_b,
                              int32_t workers, int32_t slots, int32_t* header, int32_t* prefix, int32_t* wstart, hipStream_t s);
hipError_t launch_plan_append(const int32_t* q_lens, const int32_t* q_offsets, const int32_t* ctx_lens, int32_t batch,
                              int32_t tile_tokens, int32_t cap, bool skip_unit_chunks, int32_t* header, int32_t* tile_rec,
                              hipStream_t s);
hipError_t launch_decode_f32(const DecodeArgs& a, int head_dim, int grid, hipStream_t s);
hipError_t launch_decode_mfma(const DecodeArgs& a, int head_dim, bool fp8, int grid, hipStream_t s);
hipError_t launch_combine(const DecodeArgs& a, int head_dim, bool out_bf16, hipStream_t s);
// half_tiles: every tile has at most kAppendTileRows / 2 rows (a.tile_tokens is set accordingly) and the
// two waves of a SIMD split each block of a tile between them instead of owning different rows
hipError_t launch_append_mfma(const AppendArgs& a, int head_dim, bool fp8, bool half_tiles, int grid, hipStream_t s);
hipError_t launch_append_f32(const AppendArgs& a, int head_dim, int grid, hipStream_t s);
hipError_t launch_kv_write(const void* k_new, const void* v_new, const int32_t* q_lens, const int32_t* q_offsets,
                           void* k_pages, void* v_pages, const int32_t* page_table, const int32_t* ctx_lens,
                           float* k_scale, float* v_scale, int32_t batch, int32_t hkv, int32_t max_pages,
                           int32_t max_q_len, int head_dim, int src_bytes, bool fp8, hipStream_t s);
hipError_t launch_shared_prep(const int32_t* ctx_lens, const int32_t* shared_lens, const int32_t* page_table, int32_t batch,
                              int32_t group_size, int32_t max_pages, int32_t* grp_ctx, int32_t* grp_qlens, int32_t* grp_qoff,
                              int32_t* sfx_ctx, int32_t* sfx_table, hipStream_t s);
hipError_t launch_merge_states(const void* o1, const float* d1, const void* o2, const float* d2, void* out, float* d_out,
                               long rows, int head_dim, bool f32, hipStream_t s);
hipError_t launch_check_inputs(const int32_t* page_table, const int32_t* ctx_lens, const int32_t* q_lens,
                               const int32_t* q_offsets, int32_t batch, int32_t max_pages, int64_t num_pages,
                               int32_t* counts, hipStream_t s);
hipError_t launch_gather(const void* pages, const int32_t* page_table, const int32_t* ctx_lens, int32_t b,
                         int32_t kv_head, int32_t hkv, int32_t max_pages, int32_t row_bytes, void* dst,
                         hipStream_t s);

}  // namespace rollattn
