// Internal declarations shared by the host entry points and the HIP kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "rollattn.h"

namespace rollattn {

constexpr int kPageSize = 16;
constexpr int kNumCUs = 256;          // MI355X
constexpr int kItemBudget = 16384;    // target upper bound on (piece, kv head) work items per decode call
constexpr int kMinChunk = 256;        // smallest KV piece, tokens
constexpr int kMaxDoublings = 8;      // largest piece = kMinChunk << kMaxDoublings before "one piece per row"
constexpr int kAppendTileRows = 256;  // query rows (token, head-in-group pairs) per append workgroup

// Header words of the plan, at the start of the workspace.
enum PlanWord { kPlanChunk = 0, kPlanItems = 1, kPlanCounter = 2, kPlanTiles = 3, kPlanWords = 64 };

// Byte offsets of the workspace regions (all multiples of 256).
struct WorkspaceLayout {
  int32_t cap;            // capacity in pieces (decode) or query tiles (append)
  size_t header;          // int32[kPlanWords]
  size_t item_b;          // int32[cap]   trajectory of a piece / tile
  size_t item_start;      // int32[cap]   first token of a piece / first chunk row of a tile
  size_t row_first;       // int32[B + 1] first piece of every trajectory (exclusive scan)
  size_t partial_ml;      // float[cap * Hkv][G][2]   (max in log2 units, sum)
  size_t partial_o;       // float[cap * Hkv][G][D]   un-normalised
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
  int32_t* header;
  const int32_t* item_b;
  const int32_t* item_start;
  const int32_t* row_first;
  float* partial_ml;
  float* partial_o;
  int32_t batch, hq, hkv, group, max_pages;
  float scale_log2;     // sm_scale * log2(e)
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
  const int32_t* tile_b;
  const int32_t* tile_q0;
  int32_t batch, hq, hkv, group, max_pages, tile_tokens, total_q;
  float scale_log2;
};

// Launchers (defined in the .hip files).  Each returns the hipError_t of its launch.
hipError_t launch_plan_decode(const int32_t* ctx_lens, int32_t batch, int32_t cap, int32_t* header,
                              int32_t* item_b, int32_t* item_start, int32_t* row_first, hipStream_t s);
hipError_t launch_plan_append(const int32_t* q_lens, int32_t batch, int32_t tile_tokens, int32_t cap,
                              int32_t* header, int32_t* tile_b, int32_t* tile_q0, hipStream_t s);
hipError_t launch_decode_f32(const DecodeArgs& a, int head_dim, int grid, hipStream_t s);
hipError_t launch_decode_mfma(const DecodeArgs& a, int head_dim, bool fp8, int grid, hipStream_t s);
hipError_t launch_combine(const DecodeArgs& a, int head_dim, bool out_bf16, hipStream_t s);
hipError_t launch_append_mfma(const AppendArgs& a, int head_dim, bool fp8, int grid, hipStream_t s);
hipError_t launch_append_f32(const AppendArgs& a, int head_dim, int grid, hipStream_t s);
hipError_t launch_gather(const void* pages, const int32_t* page_table, const int32_t* ctx_lens, int32_t b,
                         int32_t kv_head, int32_t hkv, int32_t max_pages, int32_t row_bytes, void* dst,
                         hipStream_t s);

}  // namespace rollattn
