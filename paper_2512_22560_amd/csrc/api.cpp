// Host side of librollattn: argument checks, workspace layout, the host twin of the
// partition rule, and the launch sequence of each entry point.  Nothing here touches the
// GPU before every argument check has passed.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "host_plan.h"
#include "rollattn_internal.h"

// Scratch memory of attn_decode_static, the decode call for callers that cannot allocate: one array per GPU,
// part of the library's code object, alive until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it stands for is looked up once per device (static_scratch_ptr).
constexpr size_t kStaticScratchBytes = (size_t)36 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
// Profiling only: what the append kernel adds up while profiling is on (shader-clock cycles, constant-rate ticks).
static __device__ unsigned long long clock_sums[2];

namespace rollattn {

namespace {

std::mutex g_mu;
std::string g_hip_error;
bool g_profile = false;
struct EventPair {
  hipEvent_t a, b;
};
constexpr size_t kMaxEvents = 1024;

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

int fail_hip(hipError_t e) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_hip_error = hipGetErrorString(e);
  return ROLLATTN_EHIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int dtype_bytes(int dt) { return dt == ROLLATTN_F32 ? 4 : dt == ROLLATTN_BF16 ? 2 : 1; }

// Descriptor checks shared by every entry point.
int check_desc(const rollattn_desc* d, bool need_scales = true) {
  if (!d) return ROLLATTN_EINVAL;
  if (d->batch < 0 || d->num_pages < 0 || d->max_pages_per_seq < 1) return ROLLATTN_EINVAL;
  if (d->num_q_heads < 1 || d->num_kv_heads < 1 || d->num_q_heads % d->num_kv_heads) return ROLLATTN_ESHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return ROLLATTN_ESHAPE;
  if (d->page_size != kPageSize) return ROLLATTN_ESHAPE;
  if (d->num_pages * (int64_t)d->num_kv_heads > INT32_MAX) return ROLLATTN_ESHAPE;   // (page, head) tiles are counted in 32 bits
  const bool f32 = d->q_dtype == ROLLATTN_F32 && d->kv_dtype == ROLLATTN_F32;
  const bool bf = d->q_dtype == ROLLATTN_BF16 && (d->kv_dtype == ROLLATTN_BF16 || d->kv_dtype == ROLLATTN_FP8_E4M3);
  if (!f32 && !bf) return ROLLATTN_EDTYPE;
  if (d->kv_dtype == ROLLATTN_FP8_E4M3 && need_scales) {
    if (!d->k_scale || !d->v_scale) return ROLLATTN_EDTYPE;
    if (!aligned16(d->k_scale) || !aligned16(d->v_scale)) return ROLLATTN_EALIGN;
  }
  if (!(d->sm_scale == d->sm_scale) || std::isinf(d->sm_scale)) return ROLLATTN_EINVAL;
  return ROLLATTN_OK;
}

// Timing events are created when profiling is switched on, never inside an attention call: a call only
// records a pair from the pool, and records nothing on a stream that is being captured into a graph
// (events recorded during capture cannot be read back).
std::vector<EventPair> g_pool;
size_t g_used = 0;
int32_t g_debug_workers = 0;                  // testing: decode plans are cut for this many workers (0: all of them)
unsigned long long* g_clock_sums = nullptr;   // device address of clock_sums on the device profiling was switched on for
int g_clock_dev = -1;                         // ... and that device: launches on other devices do not count

struct ProfileScope {
  hipStream_t s;
  bool on = false;
  EventPair ev{};
  explicit ProfileScope(hipStream_t stream) : s(stream) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_profile || g_used >= g_pool.size()) return;
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &st) != hipSuccess || st != hipStreamCaptureStatusNone) return;
    ev = g_pool[g_used++];
    on = true;
    (void)hipEventRecord(ev.a, s);
  }
  void stop() {
    if (!on) return;
    (void)hipEventRecord(ev.b, s);
    on = false;
  }
};

}  // namespace

WorkspaceLayout decode_layout(const rollattn_desc& d) {
  WorkspaceLayout w{};
  const int group = d.num_q_heads / d.num_kv_heads;
  const bool f32 = d.q_dtype == ROLLATTN_F32;
  w.head_tile = f32 ? kF32HeadTile : kMfmaHeadTile;
  w.rows_per_b = d.num_kv_heads * ((group + w.head_tile - 1) / w.head_tile);
  w.workers = f32 ? kF32DecodeWgs : kMfmaDecodeWgs * 4;
  size_t off = 0;
  w.header = off;      off += align256(sizeof(int32_t) * kPlanWords);
  w.prefix = off;      off += align256(sizeof(int32_t) * ((size_t)d.batch + 1));
  w.wstart = off;      off += align256(sizeof(int32_t) * 4 * (size_t)w.workers);
  w.partial_ml = off;  off += align256(sizeof(float) * 2 * (size_t)w.workers * w.head_tile * 2);
  w.partial_o = off;   off += align256(sizeof(float) * 2 * (size_t)w.workers * w.head_tile * d.head_dim);
  w.total = off;
  return w;
}

// Workers the decode partition is cut for: all of them, unless rollattn_debug_set_decode_workers says fewer.
static int32_t plan_workers(const WorkspaceLayout& w) {
  std::lock_guard<std::mutex> lk(g_mu);
  return (g_debug_workers > 0 && g_debug_workers < w.workers) ? g_debug_workers : w.workers;
}

WorkspaceLayout append_layout(const rollattn_desc& d, int32_t total_q) {
  WorkspaceLayout w{};
  const int group = d.num_q_heads / d.num_kv_heads;
  // room for the list of half-size tiles too (a call whose chunks are all short chooses them)
  const int tile_tokens = std::max(1, kAppendTileRows / 2 / group);
  w.workers = (int32_t)std::min<int64_t>((int64_t)total_q / tile_tokens + d.batch + 1, INT32_MAX);
  size_t off = 0;
  w.header = off;      off += align256(sizeof(int32_t) * kPlanWords);
  w.wstart = off;      off += align256(sizeof(int32_t) * kTileRecWords * (size_t)w.workers);
  w.prefix = off;
  w.partial_ml = off;
  w.partial_o = off;
  w.total = off;
  return w;
}

}  // namespace rollattn

using namespace rollattn;

static_assert(kPlanBlockTokens == kBlockTokens, "the host twin and the kernels cut rows into the same blocks");

extern "C" {

size_t rollattn_workspace_bytes(const rollattn_desc* desc, int32_t total_q) {
  if (check_desc(desc) != ROLLATTN_OK || total_q < 0) return 0;
  return std::max(decode_layout(*desc).total, append_layout(*desc, total_q).total);
}

int32_t rollattn_plan_capacity(const rollattn_desc* desc) {
  if (check_desc(desc, false) != ROLLATTN_OK) return 0;
  const WorkspaceLayout w = decode_layout(*desc);
  // every worker boundary and every row end closes one segment
  const int64_t cap = (int64_t)w.workers + (int64_t)desc->batch * w.rows_per_b;
  return (int32_t)std::min<int64_t>(cap, INT32_MAX);
}

int rollattn_debug_plan(const rollattn_desc* desc, const int32_t* ctx_lens_host, int32_t* per_out,
                        int32_t* total_out, int32_t* segments_out, int32_t* n_segments) {
  int rc = check_desc(desc, false);
  if (rc) return rc;
  if ((!ctx_lens_host && desc->batch > 0) || !per_out || !total_out || !n_segments) return ROLLATTN_EINVAL;
  const WorkspaceLayout w = decode_layout(*desc);
  const int32_t workers = plan_workers(w);
  const HostPlan p = host_plan(ctx_lens_host, desc->batch, w.rows_per_b, workers);
  *per_out = p.per;
  *total_out = p.total;
  *n_segments = expand_segments(p, desc->batch, w.rows_per_b, workers, segments_out, rollattn_plan_capacity(desc));
  return ROLLATTN_OK;
}

int rollattn_debug_read_plan(const rollattn_desc* desc, const void* workspace, int32_t* per_out,
                             int32_t* total_out, int32_t* starts_out, void* hip_stream) {
  int rc = check_desc(desc, false);
  if (rc) return rc;
  if (!workspace || !per_out || !total_out || !starts_out) return ROLLATTN_EINVAL;
  const WorkspaceLayout w = decode_layout(*desc);
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(e);
  const char* base = (const char*)workspace;
  int32_t header[kPlanWords];
  e = hipMemcpy(header, base + w.header, sizeof(header), hipMemcpyDeviceToHost);
  if (e == hipSuccess)
    e = hipMemcpy(starts_out, base + w.wstart, sizeof(int32_t) * 4 * (size_t)plan_workers(w), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(e);
  *per_out = header[kPlanPer];
  *total_out = header[kPlanTotal];
  return ROLLATTN_OK;
}

int32_t rollattn_append_plan_capacity(const rollattn_desc* desc, int32_t total_q) {
  if (check_desc(desc, false) != ROLLATTN_OK || total_q < 0) return 0;
  return append_layout(*desc, total_q).workers;
}

int rollattn_debug_read_append_plan(const rollattn_desc* desc, const void* workspace, int32_t total_q, int32_t* n_tiles_out,
                                    int32_t* tiles_out, void* hip_stream) {
  int rc = check_desc(desc, false);
  if (rc) return rc;
  if (!workspace || !n_tiles_out || !tiles_out || total_q < 0) return ROLLATTN_EINVAL;
  const WorkspaceLayout w = append_layout(*desc, total_q);
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(e);
  const char* base = (const char*)workspace;
  int32_t header[kPlanWords];
  std::vector<int32_t> rec((size_t)w.workers * kTileRecWords);
  e = hipMemcpy(header, base + w.header, sizeof(header), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(rec.data(), base + w.wstart, sizeof(int32_t) * rec.size(), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(e);
  const int32_t n = std::max(0, std::min(header[kPlanTiles], w.workers));
  *n_tiles_out = n;
  for (int32_t i = 0; i < n; ++i) {
    tiles_out[2 * i] = rec[(size_t)i * kTileRecWords];
    tiles_out[2 * i + 1] = rec[(size_t)i * kTileRecWords + 1];
  }
  return ROLLATTN_OK;
}

int32_t rollattn_plan_workers(const rollattn_desc* desc) {
  if (check_desc(desc, false) != ROLLATTN_OK) return 0;
  return plan_workers(decode_layout(*desc));
}

int32_t rollattn_debug_set_decode_workers(int32_t workers) {
  std::lock_guard<std::mutex> lk(g_mu);
  const int32_t before = g_debug_workers;
  g_debug_workers = workers > 0 ? workers : 0;
  return before;
}

// Shape limits of the decode path and of the append path beyond the descriptor checks; the entry points that
// chain several launches check both before the first one.
static int decode_limits(const rollattn_desc& d) {
  const WorkspaceLayout w = decode_layout(d);
  // the block sequence is indexed with 32-bit integers
  if ((int64_t)d.batch * w.rows_per_b * ((int64_t)d.max_pages_per_seq / 2 + 1) > INT32_MAX) return ROLLATTN_ESHAPE;
  // a worker's start record packs the row index into 11 bits and the block index into 20
  if (w.rows_per_b > 2047 || d.max_pages_per_seq / 2 + 1 > (1 << 20)) return ROLLATTN_ESHAPE;
  return ROLLATTN_OK;
}
static int append_limits(const rollattn_desc& d) {
  if (d.q_dtype != ROLLATTN_F32 && d.num_q_heads / d.num_kv_heads > kAppendTileRows) return ROLLATTN_ESHAPE;
  return ROLLATTN_OK;
}

// attn_decode proper; lse (optional, device [B][Hq]) receives log2 of every row's softmax denominator.
// q_lens / q_offsets (both or neither): the mixed step, see DecodeArgs.
static int decode_impl(const rollattn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                       const int32_t* page_table, const int32_t* ctx_lens, void* out, void* workspace,
                       size_t workspace_bytes, void* hip_stream, float* lse, const int32_t* q_lens = nullptr,
                       const int32_t* q_offsets = nullptr) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (desc->batch == 0) return ROLLATTN_OK;
  if (!q || !k_pages || !v_pages || !page_table || !ctx_lens || !out || !workspace) return ROLLATTN_EINVAL;
  if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(page_table) ||
      !aligned16(ctx_lens) || !aligned16(out) || !aligned16(workspace))
    return ROLLATTN_EALIGN;
  const WorkspaceLayout w = decode_layout(*desc);
  if (workspace_bytes < w.total) return ROLLATTN_EWORKSPACE;
  rc = decode_limits(*desc);
  if (rc) return rc;

  hipStream_t s = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  DecodeArgs a{};
  a.q = q; a.k_pages = k_pages; a.v_pages = v_pages; a.page_table = page_table; a.ctx_lens = ctx_lens;
  a.out = out; a.k_scale = desc->k_scale; a.v_scale = desc->v_scale;
  a.header = (const int32_t*)(base + w.header);
  a.prefix = (const int32_t*)(base + w.prefix);
  a.wstart = (const int32_t*)(base + w.wstart);
  a.partial_ml = (float*)(base + w.partial_ml);
  a.partial_o = (float*)(base + w.partial_o);
  a.batch = desc->batch; a.hq = desc->num_q_heads; a.hkv = desc->num_kv_heads;
  a.group = desc->num_q_heads / desc->num_kv_heads; a.max_pages = desc->max_pages_per_seq;
  a.head_tile = w.head_tile; a.rows_per_b = w.rows_per_b;
  a.scale_log2 = desc->sm_scale * 1.4426950408889634f;
  a.lse = lse;
  a.q_lens = q_lens;
  a.q_offsets = q_offsets;

  // (the launch has w.workers workers whatever the partition is cut for: the others get a record without blocks)
  hipError_t e = launch_plan_decode(ctx_lens, q_lens, desc->batch, w.rows_per_b, plan_workers(w), w.workers,
                                    (int32_t*)(base + w.header), (int32_t*)(base + w.prefix), (int32_t*)(base + w.wstart), s);
  if (e != hipSuccess) return fail_hip(e);
  const bool f32 = desc->q_dtype == ROLLATTN_F32;
  {
    ProfileScope prof(s);
    if (f32) {
      e = launch_decode_f32(a, desc->head_dim, kF32DecodeWgs, s);
    } else {
      e = launch_decode_mfma(a, desc->head_dim, desc->kv_dtype == ROLLATTN_FP8_E4M3, kMfmaDecodeWgs, s);
    }
    prof.stop();
  }
  if (e != hipSuccess) return fail_hip(e);
  e = launch_combine(a, desc->head_dim, !f32, s);
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int attn_decode(const rollattn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                const int32_t* page_table, const int32_t* ctx_lens, void* out, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  return decode_impl(desc, q, k_pages, v_pages, page_table, ctx_lens, out, workspace, workspace_bytes, hip_stream, nullptr);
}

namespace {
constexpr int kMaxDevices = 64;
void* g_static_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, null until looked up

// Address of the current device's copy of `scratch`; the lookup runs once per device, with that device current.
int static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e);
  if (dev < 0 || dev >= kMaxDevices) return fail_hip(hipErrorInvalidDevice);
  {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_static_ptr[dev]) {
      *out = g_static_ptr[dev];
      return ROLLATTN_OK;
    }
  }
  void* p = nullptr;
  e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return fail_hip(e);
  if (!p) return fail_hip(hipErrorInvalidSymbol);
  std::lock_guard<std::mutex> lk(g_mu);
  g_static_ptr[dev] = p;
  *out = p;
  return ROLLATTN_OK;
}
}  // namespace

size_t rollattn_static_scratch_bytes(void) { return kStaticScratchBytes; }

int rollattn_static_init(void) {
  void* p = nullptr;
  return static_scratch_ptr(&p);
}

int attn_decode_static(const rollattn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                       const int32_t* page_table, const int32_t* ctx_lens, void* out, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (desc->batch == 0) return ROLLATTN_OK;
  if (decode_layout(*desc).total > kStaticScratchBytes) return ROLLATTN_ELIMIT;
  void* ws = nullptr;
  rc = static_scratch_ptr(&ws);
  if (rc) return rc;
  return decode_impl(desc, q, k_pages, v_pages, page_table, ctx_lens, out, ws, kStaticScratchBytes, hip_stream, nullptr);
}

// attn_append proper.  table_stride: int32 entries between the page-table rows of consecutive
// trajectories; noncausal: every row sees all of [0, L_b) (then n_b <= L_b is not required);
// lse as in decode_impl, [total_q][Hq].  table_stride and noncausal are for the bf16 kernels only.
static int append_impl(const rollattn_desc* desc, const void* q_chunk, const int32_t* q_lens, const int32_t* q_offsets,
                       int32_t total_q, int32_t max_q_len, const void* k_pages, const void* v_pages,
                       const int32_t* page_table, const int32_t* ctx_lens, void* out, void* workspace,
                       size_t workspace_bytes, void* hip_stream, int32_t table_stride, bool noncausal, float* lse,
                       bool skip_unit_chunks = false) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (total_q < 0 || max_q_len < 0) return ROLLATTN_EINVAL;
  rc = append_limits(*desc);
  if (rc) return rc;
  if (desc->batch == 0 || total_q == 0) return ROLLATTN_OK;
  if (!q_chunk || !q_lens || !q_offsets || !k_pages || !v_pages || !page_table || !ctx_lens || !out || !workspace)
    return ROLLATTN_EINVAL;
  if (!aligned16(q_chunk) || !aligned16(q_lens) || !aligned16(q_offsets) || !aligned16(k_pages) ||
      !aligned16(v_pages) || !aligned16(page_table) || !aligned16(ctx_lens) || !aligned16(out) ||
      !aligned16(workspace))
    return ROLLATTN_EALIGN;
  const WorkspaceLayout w = append_layout(*desc, total_q);
  if (workspace_bytes < w.total) return ROLLATTN_EWORKSPACE;

  hipStream_t s = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  AppendArgs a{};
  a.q = q_chunk; a.k_pages = k_pages; a.v_pages = v_pages; a.page_table = page_table; a.ctx_lens = ctx_lens;
  a.q_lens = q_lens; a.q_offsets = q_offsets; a.out = out; a.k_scale = desc->k_scale; a.v_scale = desc->v_scale;
  a.header = (int32_t*)(base + w.header);
  a.tile_rec = (const int32_t*)(base + w.wstart);
  a.batch = desc->batch; a.hq = desc->num_q_heads; a.hkv = desc->num_kv_heads;
  a.group = desc->num_q_heads / desc->num_kv_heads; a.max_pages = table_stride;
  a.tile_tokens = std::max(1, kAppendTileRows / a.group);
  // No chunk longer than half a tile (a few new tokens per trajectory; the members of a group in attn_decode_shared):
  // half tiles, whose blocks the two waves of a SIMD share
  const bool half_tiles = desc->q_dtype != ROLLATTN_F32 && (int64_t)max_q_len * a.group <= kAppendTileRows / 2;
  if (half_tiles) a.tile_tokens = std::max(1, kAppendTileRows / 2 / a.group);
  // tiles this call can have at most (<= the capacity of the workspace, which is laid out for half tiles)
  const int32_t tile_cap = (int32_t)std::min<int64_t>((int64_t)total_q / a.tile_tokens + desc->batch + 1, w.workers);
  a.tile_cap = tile_cap;
  a.total_q = total_q;
  a.scale_log2 = desc->sm_scale * 1.4426950408889634f;
  a.lse = lse;
  a.noncausal = noncausal ? 1 : 0;
  a.clock_sums = nullptr;

  hipError_t e;
  if (desc->q_dtype == ROLLATTN_F32) {
    const int tiles = (a.group + 3) / 4;
    const int grid = (int)std::min<int64_t>((int64_t)total_q * a.hkv * tiles, 1 << 20);
    ProfileScope prof(s);
    e = launch_append_f32(a, desc->head_dim, grid, s);
    prof.stop();
    if (e != hipSuccess) return fail_hip(e);
    return ROLLATTN_OK;
  }
  e = launch_plan_append(q_lens, q_offsets, ctx_lens, desc->batch, a.tile_tokens, tile_cap, skip_unit_chunks, a.header,
                         (int32_t*)(base + w.wstart), s);
  if (e != hipSuccess) return fail_hip(e);
  {
    ProfileScope prof(s);
    // one workgroup per (tile, KV head); with fewer than 8 heads the kernel deals runs of tiles to the XCDs
    // of a head, which needs up to one run of slack per XCD (see the kernel's index mapping)
    int64_t grid64 = (int64_t)tile_cap * a.hkv;
    if (a.hkv < kXcds && kXcds % a.hkv == 0) {
      const int64_t parts = kXcds / a.hkv;
      grid64 = kXcds * (((int64_t)tile_cap + parts - 1) / parts + kAppendXcdRun);
    }
    const int grid = (int)std::min<int64_t>(grid64, INT32_MAX);
    int dev = -1;
    if (prof.on && hipGetDevice(&dev) == hipSuccess && dev == g_clock_dev) a.clock_sums = g_clock_sums;
    e = launch_append_mfma(a, desc->head_dim, desc->kv_dtype == ROLLATTN_FP8_E4M3, half_tiles, grid, s);
    prof.stop();
  }
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int attn_append(const rollattn_desc* desc, const void* q_chunk, const int32_t* q_lens, const int32_t* q_offsets,
                int32_t total_q, int32_t max_q_len, const void* k_pages, const void* v_pages,
                const int32_t* page_table, const int32_t* ctx_lens, void* out, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  if (!desc) return ROLLATTN_EINVAL;
  return append_impl(desc, q_chunk, q_lens, q_offsets, total_q, max_q_len, k_pages, v_pages, page_table, ctx_lens, out,
                     workspace, workspace_bytes, hip_stream, desc->max_pages_per_seq, false, nullptr);
}

int attn_decode_lse(const rollattn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                    const int32_t* page_table, const int32_t* ctx_lens, void* out, float* lse, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (desc && desc->batch > 0 && !lse) return ROLLATTN_EINVAL;
  if (lse && !aligned16(lse)) return ROLLATTN_EALIGN;
  return decode_impl(desc, q, k_pages, v_pages, page_table, ctx_lens, out, workspace, workspace_bytes, hip_stream, lse);
}

int attn_append_lse(const rollattn_desc* desc, const void* q_chunk, const int32_t* q_lens, const int32_t* q_offsets,
                    int32_t total_q, int32_t max_q_len, const void* k_pages, const void* v_pages,
                    const int32_t* page_table, const int32_t* ctx_lens, void* out, float* lse, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (!desc) return ROLLATTN_EINVAL;
  if (desc->batch > 0 && total_q > 0 && !lse) return ROLLATTN_EINVAL;
  if (lse && !aligned16(lse)) return ROLLATTN_EALIGN;
  return append_impl(desc, q_chunk, q_lens, q_offsets, total_q, max_q_len, k_pages, v_pages, page_table, ctx_lens, out,
                     workspace, workspace_bytes, hip_stream, desc->max_pages_per_seq, false, lse);
}

int attn_merge(const rollattn_desc* desc, int64_t rows, const void* o1, const float* lse1, const void* o2,
               const float* lse2, void* out, float* lse_out, void* hip_stream) {
  int rc = check_desc(desc, /*need_scales=*/false);
  if (rc) return rc;
  if (rows < 0) return ROLLATTN_EINVAL;
  if (rows == 0) return ROLLATTN_OK;
  if (!o1 || !lse1 || !o2 || !lse2 || !out) return ROLLATTN_EINVAL;
  if (!aligned16(o1) || !aligned16(lse1) || !aligned16(o2) || !aligned16(lse2) || !aligned16(out) ||
      (lse_out && !aligned16(lse_out)))
    return ROLLATTN_EALIGN;
  if (rows * (int64_t)desc->num_q_heads > (int64_t)INT32_MAX * 4) return ROLLATTN_ESHAPE;   // one wave per (row, head), four per workgroup
  const hipError_t e = launch_merge_states(o1, lse1, o2, lse2, out, lse_out, (long)rows * desc->num_q_heads, desc->head_dim,
                                           desc->q_dtype == ROLLATTN_F32, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

size_t rollattn_step_workspace_bytes(const rollattn_desc* desc, int32_t total_q) {
  if (check_desc(desc) != ROLLATTN_OK || total_q < 0) return 0;
  return align256(decode_layout(*desc).total) + append_layout(*desc, total_q).total;
}

size_t rollattn_step_append_offset(const rollattn_desc* desc) {
  if (check_desc(desc, false) != ROLLATTN_OK) return 0;
  return align256(decode_layout(*desc).total);
}

int attn_step(const rollattn_desc* desc, const void* q, const int32_t* q_lens, const int32_t* q_offsets, int32_t total_q,
              int32_t max_q_len, const void* k_pages, const void* v_pages, const int32_t* page_table,
              const int32_t* ctx_lens, void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (total_q < 0 || max_q_len < 0) return ROLLATTN_EINVAL;
  if (desc->batch == 0 || total_q == 0) return ROLLATTN_OK;
  if (!workspace) return ROLLATTN_EINVAL;
  if (!aligned16(workspace)) return ROLLATTN_EALIGN;
  if (workspace_bytes < rollattn_step_workspace_bytes(desc, total_q)) return ROLLATTN_EWORKSPACE;
  if (desc->q_dtype == ROLLATTN_F32) {
    // the float32 path has one kernel for chunks of any length, one token included
    return append_impl(desc, q, q_lens, q_offsets, total_q, max_q_len, k_pages, v_pages, page_table, ctx_lens, out,
                       workspace, workspace_bytes, hip_stream, desc->max_pages_per_seq, false, nullptr);
  }
  if (!q || !q_lens || !q_offsets || !k_pages || !v_pages || !page_table || !ctx_lens || !out) return ROLLATTN_EINVAL;
  if (!aligned16(q) || !aligned16(q_lens) || !aligned16(q_offsets) || !aligned16(k_pages) || !aligned16(v_pages) ||
      !aligned16(page_table) || !aligned16(ctx_lens) || !aligned16(out))
    return ROLLATTN_EALIGN;
  rc = append_limits(*desc);                       // everything either half could object to, before the first launch
  if (!rc) rc = decode_limits(*desc);
  if (rc) return rc;
  const size_t dec_bytes = align256(decode_layout(*desc).total);
  // the long tiles of the chunks first, then the decode rows and their merge; all on one stream, disjoint output rows
  rc = append_impl(desc, q, q_lens, q_offsets, total_q, max_q_len, k_pages, v_pages, page_table, ctx_lens, out,
                   (char*)workspace + dec_bytes, workspace_bytes - dec_bytes, hip_stream, desc->max_pages_per_seq, false,
                   nullptr, /*skip_unit_chunks=*/true);
  if (rc) return rc;
  return decode_impl(desc, q, k_pages, v_pages, page_table, ctx_lens, out, workspace, dec_bytes, hip_stream, nullptr, q_lens,
                     q_offsets);
}

namespace {
// Workspace of attn_decode_shared: the two inner workspaces, the two halves' rows and denominators,
// the group "chunk" description and the shifted private tables.
struct SharedLayout {
  rollattn_desc grp;      // descriptor of the shared half: one "trajectory" per group
  size_t dec_ws, app_ws, o1, o2, d1, d2, grp_ctx, grp_qlens, grp_qoff, sfx_ctx, sfx_table, total;
  size_t dec_bytes, app_bytes;
};
SharedLayout shared_layout(const rollattn_desc& d, int32_t group_size) {
  SharedLayout L{};
  L.grp = d;
  L.grp.batch = d.batch / group_size;
  const size_t rows = (size_t)d.batch * d.num_q_heads;
  const size_t groups = (size_t)L.grp.batch;
  L.dec_bytes = decode_layout(d).total;
  L.app_bytes = append_layout(L.grp, d.batch).total;
  size_t off = 0;
  L.dec_ws = off;    off += align256(L.dec_bytes);
  L.app_ws = off;    off += align256(L.app_bytes);
  L.o1 = off;        off += align256(rows * d.head_dim * 2);
  L.o2 = off;        off += align256(rows * d.head_dim * 2);
  L.d1 = off;        off += align256(rows * sizeof(float));
  L.d2 = off;        off += align256(rows * sizeof(float));
  L.grp_ctx = off;   off += align256(groups * sizeof(int32_t));
  L.grp_qlens = off; off += align256(groups * sizeof(int32_t));
  L.grp_qoff = off;  off += align256((groups + 1) * sizeof(int32_t));
  L.sfx_ctx = off;   off += align256((size_t)d.batch * sizeof(int32_t));
  L.sfx_table = off; off += align256((size_t)d.batch * d.max_pages_per_seq * sizeof(int32_t));
  L.total = off;
  return L;
}
int check_shared(const rollattn_desc* desc, int32_t group_size) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (desc->q_dtype != ROLLATTN_BF16) return ROLLATTN_EDTYPE;
  if (group_size < 1 || desc->batch % group_size) return ROLLATTN_EINVAL;
  if ((int64_t)group_size * desc->max_pages_per_seq > INT32_MAX) return ROLLATTN_ESHAPE;
  return ROLLATTN_OK;
}
}  // namespace

size_t rollattn_shared_workspace_bytes(const rollattn_desc* desc, int32_t group_size) {
  if (check_shared(desc, group_size) != ROLLATTN_OK) return 0;
  return shared_layout(*desc, group_size).total;
}

int attn_decode_shared(const rollattn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                       const int32_t* page_table, const int32_t* ctx_lens, int32_t group_size, const int32_t* shared_lens,
                       void* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shared(desc, group_size);
  if (rc) return rc;
  if (desc->batch == 0) return ROLLATTN_OK;
  if (!q || !k_pages || !v_pages || !page_table || !ctx_lens || !shared_lens || !out || !workspace) return ROLLATTN_EINVAL;
  if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(page_table) || !aligned16(ctx_lens) ||
      !aligned16(shared_lens) || !aligned16(out) || !aligned16(workspace))
    return ROLLATTN_EALIGN;
  const SharedLayout L = shared_layout(*desc, group_size);
  if (workspace_bytes < L.total) return ROLLATTN_EWORKSPACE;
  rc = append_limits(L.grp);                       // everything either half could object to, before the first launch
  if (!rc) rc = decode_limits(*desc);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  int32_t* grp_ctx = (int32_t*)(base + L.grp_ctx);
  int32_t* grp_qlens = (int32_t*)(base + L.grp_qlens);
  int32_t* grp_qoff = (int32_t*)(base + L.grp_qoff);
  int32_t* sfx_ctx = (int32_t*)(base + L.sfx_ctx);
  int32_t* sfx_table = (int32_t*)(base + L.sfx_table);
  hipError_t e = launch_shared_prep(ctx_lens, shared_lens, page_table, desc->batch, group_size, desc->max_pages_per_seq,
                                    grp_ctx, grp_qlens, grp_qoff, sfx_ctx, sfx_table, s);
  if (e != hipSuccess) return fail_hip(e);
  // shared half: the members' query rows of a group as one chunk over the group's first S tokens
  rc = append_impl(&L.grp, q, grp_qlens, grp_qoff, desc->batch, group_size, k_pages, v_pages, page_table, grp_ctx,
                   base + L.o1, base + L.app_ws, L.app_bytes, hip_stream, group_size * desc->max_pages_per_seq, true,
                   (float*)(base + L.d1));
  if (rc) return rc;
  // private half: every trajectory from token S on
  rc = decode_impl(desc, q, k_pages, v_pages, sfx_table, sfx_ctx, base + L.o2, base + L.dec_ws, L.dec_bytes, hip_stream,
                   (float*)(base + L.d2));
  if (rc) return rc;
  e = launch_merge_states(base + L.o1, (const float*)(base + L.d1), base + L.o2, (const float*)(base + L.d2), out, nullptr,
                          (long)desc->batch * desc->num_q_heads, desc->head_dim, /*f32=*/false, s);
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int kv_write(const rollattn_desc* desc, const void* k_new, const void* v_new, const int32_t* q_lens,
             const int32_t* q_offsets, int32_t total_q, int32_t max_q_len, void* k_pages, void* v_pages,
             const int32_t* page_table, const int32_t* ctx_lens, float* k_scale, float* v_scale, void* hip_stream) {
  int rc = check_desc(desc, /*need_scales=*/false);
  if (rc) return rc;
  if (total_q < 0 || max_q_len < 0) return ROLLATTN_EINVAL;
  if (desc->batch == 0 || total_q == 0) return ROLLATTN_OK;
  const bool fp8 = desc->kv_dtype == ROLLATTN_FP8_E4M3;
  if (!k_new || !v_new || !q_lens || !q_offsets || !k_pages || !v_pages || !page_table || !ctx_lens) return ROLLATTN_EINVAL;
  if (fp8 && (!k_scale || !v_scale)) return ROLLATTN_EDTYPE;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(q_lens) || !aligned16(q_offsets) || !aligned16(k_pages) ||
      !aligned16(v_pages) || !aligned16(page_table) || !aligned16(ctx_lens) || (fp8 && (!aligned16(k_scale) || !aligned16(v_scale))))
    return ROLLATTN_EALIGN;
  if (desc->batch > 65535) return ROLLATTN_ESHAPE;     // one grid row per trajectory
  hipStream_t s = (hipStream_t)hip_stream;
  ProfileScope prof(s);
  const hipError_t e = launch_kv_write(k_new, v_new, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, k_scale,
                                       v_scale, desc->batch, desc->num_kv_heads, desc->max_pages_per_seq, max_q_len,
                                       desc->head_dim, desc->q_dtype == ROLLATTN_F32 ? 4 : 2, fp8, s);
  prof.stop();
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int rollattn_debug_gather(const rollattn_desc* desc, const void* pages, const int32_t* page_table,
                          const int32_t* ctx_lens, int32_t b, int32_t kv_head, void* dst, void* hip_stream) {
  int rc = check_desc(desc, /*need_scales=*/false);
  if (rc) return rc;
  if (!pages || !page_table || !ctx_lens || !dst) return ROLLATTN_EINVAL;
  if (b < 0 || b >= desc->batch || kv_head < 0 || kv_head >= desc->num_kv_heads) return ROLLATTN_EINVAL;
  if (!aligned16(pages) || !aligned16(page_table) || !aligned16(dst)) return ROLLATTN_EALIGN;
  hipError_t e = launch_gather(pages, page_table, ctx_lens, b, kv_head, desc->num_kv_heads, desc->max_pages_per_seq,
                               desc->head_dim * dtype_bytes(desc->kv_dtype), dst, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int rollattn_debug_check_inputs(const rollattn_desc* desc, const int32_t* page_table, const int32_t* ctx_lens,
                                const int32_t* q_lens, const int32_t* q_offsets, int32_t* counts_dev,
                                int32_t* counts_out, void* hip_stream) {
  int rc = check_desc(desc, /*need_scales=*/false);
  if (rc) return rc;
  if (!counts_out) return ROLLATTN_EINVAL;
  for (int i = 0; i < 4; ++i) counts_out[i] = 0;
  if (desc->batch == 0) return ROLLATTN_OK;
  if (!page_table || !ctx_lens || !counts_dev) return ROLLATTN_EINVAL;
  if (!aligned16(page_table) || !aligned16(ctx_lens) || !aligned16(counts_dev) || (q_lens && !aligned16(q_lens)) ||
      (q_offsets && !aligned16(q_offsets)))
    return ROLLATTN_EALIGN;
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = launch_check_inputs(page_table, ctx_lens, q_lens, q_offsets, desc->batch, desc->max_pages_per_seq,
                                     desc->num_pages, counts_dev, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess) e = hipMemcpy(counts_out, counts_dev, 4 * sizeof(int32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int rollattn_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (on && g_pool.empty()) {
    g_pool.reserve(kMaxEvents);
    for (size_t i = 0; i < kMaxEvents; ++i) {
      EventPair ev{};
      hipError_t e = hipEventCreate(&ev.a);
      if (e == hipSuccess) {
        e = hipEventCreate(&ev.b);
        if (e != hipSuccess) (void)hipEventDestroy(ev.a);
      }
      if (e != hipSuccess) {
        g_hip_error = hipGetErrorString(e);
        for (auto& p : g_pool) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
        g_pool.clear();
        return ROLLATTN_EHIP;
      }
      g_pool.push_back(ev);
    }
  }
  if (on && !g_clock_sums) {
    void* p = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(clock_sums));
    if (e == hipSuccess) e = hipMemset(p, 0, 2 * sizeof(unsigned long long));
    if (e != hipSuccess) {
      g_hip_error = hipGetErrorString(e);
      return ROLLATTN_EHIP;
    }
    g_clock_sums = (unsigned long long*)p;
    g_clock_dev = dev;
  }
  g_profile = on != 0;
  return ROLLATTN_OK;
}

int rollattn_profile_append_clock(double* mhz_out) {
  if (!mhz_out) return ROLLATTN_EINVAL;
  *mhz_out = 0.0;
  unsigned long long* p;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    p = g_clock_sums;
  }
  if (!p) return ROLLATTN_OK;
  unsigned long long sums[2] = {0, 0};
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpy(sums, p, sizeof(sums), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemset(p, 0, sizeof(sums));
  if (e != hipSuccess) return fail_hip(e);
  if (sums[1]) *mhz_out = 100.0 * (double)sums[0] / (double)sums[1];
  return ROLLATTN_OK;
}

int rollattn_profile_read(float* ms_out, int cap) {
  std::vector<EventPair> evs;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    evs.assign(g_pool.begin(), g_pool.begin() + g_used);
    g_used = 0;
  }
  int n = 0;
  for (auto& ev : evs) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(ev.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
    if (e == hipSuccess && ms_out && n < cap) ms_out[n++] = ms;
  }
  return n;
}

const char* rollattn_status_string(int status) {
  switch (status) {
    case ROLLATTN_OK: return "ok";
    case ROLLATTN_EINVAL: return "invalid argument (null pointer or negative size)";
    case ROLLATTN_ESHAPE: return "unsupported shape (Hq % Hkv != 0, head_dim not 64/128, page_size not 16)";
    case ROLLATTN_EDTYPE: return "unsupported q/kv dtype pair, or FP8 pools without scales";
    case ROLLATTN_EALIGN: return "device pointer not 16-byte aligned";
    case ROLLATTN_EWORKSPACE: return "workspace smaller than rollattn_workspace_bytes()";
    case ROLLATTN_EHIP: return "HIP call failed (see rollattn_last_hip_error)";
    case ROLLATTN_ELIMIT: return "the call needs more scratch memory than the library's built-in array holds (rollattn_static_scratch_bytes)";
    default: return "unknown status";
  }
}

const char* rollattn_last_hip_error(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  static thread_local std::string copy;
  copy = g_hip_error;
  return copy.c_str();
}

int rollattn_version(void) { return 101; }

}  // extern "C"
