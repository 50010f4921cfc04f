// Host side of librollattn: argument checks, workspace layout, the host twin of the
// partition rule, and the launch sequence of each entry point.  Nothing here touches the
// GPU before every argument check has passed.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "rollattn_internal.h"

namespace rollattn {

namespace {

std::mutex g_mu;
std::string g_hip_error;
bool g_profile = false;
struct EventPair {
  hipEvent_t a, b;
};
std::vector<EventPair> g_events;
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

int32_t plan_cap(const rollattn_desc& d) { return std::max<int32_t>(std::max(d.batch, 1), kItemBudget / d.num_kv_heads); }

struct ProfileScope {
  hipStream_t s;
  bool on = false;
  EventPair ev{};
  explicit ProfileScope(hipStream_t stream) : s(stream) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_profile && g_events.size() < kMaxEvents) {
      if (hipEventCreate(&ev.a) == hipSuccess && hipEventCreate(&ev.b) == hipSuccess) {
        on = true;
        (void)hipEventRecord(ev.a, s);
      }
    }
  }
  void stop() {
    if (!on) return;
    (void)hipEventRecord(ev.b, s);
    std::lock_guard<std::mutex> lk(g_mu);
    g_events.push_back(ev);
    on = false;
  }
};

}  // namespace

WorkspaceLayout decode_layout(const rollattn_desc& d) {
  WorkspaceLayout w{};
  const size_t group = d.num_q_heads / d.num_kv_heads;
  w.cap = plan_cap(d);
  size_t off = 0;
  w.header = off;      off += align256(sizeof(int32_t) * kPlanWords);
  w.item_b = off;      off += align256(sizeof(int32_t) * (size_t)w.cap);
  w.item_start = off;  off += align256(sizeof(int32_t) * (size_t)w.cap);
  w.row_first = off;   off += align256(sizeof(int32_t) * ((size_t)d.batch + 1));
  w.partial_ml = off;  off += align256(sizeof(float) * (size_t)w.cap * d.num_kv_heads * group * 2);
  w.partial_o = off;   off += align256(sizeof(float) * (size_t)w.cap * d.num_kv_heads * group * d.head_dim);
  w.total = off;
  return w;
}

WorkspaceLayout append_layout(const rollattn_desc& d, int32_t total_q) {
  WorkspaceLayout w{};
  const int group = d.num_q_heads / d.num_kv_heads;
  const int tile_tokens = std::max(1, kAppendTileRows / group);
  w.cap = (int32_t)std::min<int64_t>((int64_t)total_q / tile_tokens + d.batch + 1, INT32_MAX);
  size_t off = 0;
  w.header = off;      off += align256(sizeof(int32_t) * kPlanWords);
  w.item_b = off;      off += align256(sizeof(int32_t) * (size_t)w.cap);
  w.item_start = off;  off += align256(sizeof(int32_t) * (size_t)w.cap);
  w.row_first = off;
  w.partial_ml = off;
  w.partial_o = off;
  w.total = off;
  return w;
}

}  // namespace rollattn

using namespace rollattn;

extern "C" {

size_t rollattn_workspace_bytes(const rollattn_desc* desc, int32_t total_q) {
  if (check_desc(desc) != ROLLATTN_OK || total_q < 0) return 0;
  return std::max(decode_layout(*desc).total, append_layout(*desc, total_q).total);
}

int32_t rollattn_plan_capacity(const rollattn_desc* desc) {
  if (check_desc(desc) != ROLLATTN_OK) return 0;
  return plan_cap(*desc);
}

int rollattn_debug_plan(const rollattn_desc* desc, const int32_t* ctx_lens_host, int32_t* chunk_out,
                        int32_t* items_out, int32_t* n_items) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if ((!ctx_lens_host && desc->batch > 0) || !chunk_out || !n_items) return ROLLATTN_EINVAL;
  const int32_t cap = plan_cap(*desc);
  int32_t chunk = 0;
  for (int k = 0; k <= kMaxDoublings; ++k) {
    const int32_t c = kMinChunk << k;
    int64_t pieces = 0;
    for (int32_t b = 0; b < desc->batch; ++b) pieces += (ctx_lens_host[b] + c - 1) / c;
    if (pieces <= cap) {
      chunk = c;
      break;
    }
  }
  int32_t n = 0;
  for (int32_t b = 0; b < desc->batch; ++b) {
    const int32_t len = ctx_lens_host[b];
    const int32_t count = chunk ? (len + chunk - 1) / chunk : (len > 0 ? 1 : 0);
    for (int32_t s = 0; s < count; ++s, ++n) {
      if (items_out) {
        items_out[4 * n + 0] = b;
        items_out[4 * n + 1] = s * chunk;
        items_out[4 * n + 2] = chunk ? std::min(chunk, len - s * chunk) : len;
        items_out[4 * n + 3] = s;
      }
    }
  }
  *chunk_out = chunk;
  *n_items = n;
  return ROLLATTN_OK;
}

int rollattn_debug_read_plan(const rollattn_desc* desc, const void* workspace, const int32_t* ctx_lens,
                             int32_t* chunk_out, int32_t* items_out, int32_t* n_items, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!workspace || !ctx_lens || !chunk_out || !n_items) return ROLLATTN_EINVAL;
  const WorkspaceLayout w = decode_layout(*desc);
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail_hip(e);
  const char* base = (const char*)workspace;
  int32_t header[kPlanWords];
  e = hipMemcpy(header, base + w.header, sizeof(header), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(e);
  const int32_t n = header[kPlanItems], chunk = header[kPlanChunk];
  *chunk_out = chunk;
  *n_items = n;
  if (!items_out || n <= 0) return ROLLATTN_OK;
  std::vector<int32_t> ib(n), is(n), rf((size_t)desc->batch + 1), lens((size_t)desc->batch);
  e = hipMemcpy(lens.data(), ctx_lens, sizeof(int32_t) * lens.size(), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(ib.data(), base + w.item_b, sizeof(int32_t) * n, hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(is.data(), base + w.item_start, sizeof(int32_t) * n, hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(rf.data(), base + w.row_first, sizeof(int32_t) * rf.size(), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(e);
  for (int32_t i = 0; i < n; ++i) {
    const int32_t b = ib[i];
    items_out[4 * i + 0] = b;
    items_out[4 * i + 1] = is[i];
    items_out[4 * i + 2] = chunk ? std::min(chunk, lens[b] - is[i]) : lens[b];
    items_out[4 * i + 3] = i - rf[b];
  }
  return ROLLATTN_OK;
}

int attn_decode(const rollattn_desc* desc, const void* q, const void* k_pages, const void* v_pages,
                const int32_t* page_table, const int32_t* ctx_lens, void* out, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (desc->batch == 0) return ROLLATTN_OK;
  if (!q || !k_pages || !v_pages || !page_table || !ctx_lens || !out || !workspace) return ROLLATTN_EINVAL;
  if (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(page_table) ||
      !aligned16(ctx_lens) || !aligned16(out) || !aligned16(workspace))
    return ROLLATTN_EALIGN;
  const WorkspaceLayout w = decode_layout(*desc);
  if (workspace_bytes < w.total) return ROLLATTN_EWORKSPACE;

  hipStream_t s = (hipStream_t)hip_stream;
  char* base = (char*)workspace;
  DecodeArgs a{};
  a.q = q; a.k_pages = k_pages; a.v_pages = v_pages; a.page_table = page_table; a.ctx_lens = ctx_lens;
  a.out = out; a.k_scale = desc->k_scale; a.v_scale = desc->v_scale;
  a.header = (int32_t*)(base + w.header);
  a.item_b = (const int32_t*)(base + w.item_b);
  a.item_start = (const int32_t*)(base + w.item_start);
  a.row_first = (const int32_t*)(base + w.row_first);
  a.partial_ml = (float*)(base + w.partial_ml);
  a.partial_o = (float*)(base + w.partial_o);
  a.batch = desc->batch; a.hq = desc->num_q_heads; a.hkv = desc->num_kv_heads;
  a.group = desc->num_q_heads / desc->num_kv_heads; a.max_pages = desc->max_pages_per_seq;
  a.scale_log2 = desc->sm_scale * 1.4426950408889634f;

  hipError_t e = launch_plan_decode(ctx_lens, desc->batch, w.cap, a.header, (int32_t*)(base + w.item_b),
                                    (int32_t*)(base + w.item_start), (int32_t*)(base + w.row_first), s);
  if (e != hipSuccess) return fail_hip(e);
  const bool f32 = desc->q_dtype == ROLLATTN_F32;
  {
    ProfileScope prof(s);
    if (f32) {
      const int tiles = (a.group + 3) / 4;
      const int grid = (int)std::min<int64_t>((int64_t)w.cap * a.hkv * tiles, kNumCUs * 4);
      e = launch_decode_f32(a, desc->head_dim, grid, s);
    } else {
      const int tiles = (a.group + 15) / 16;
      const int grid = (int)std::min<int64_t>((int64_t)w.cap * a.hkv * tiles, kNumCUs * 2);
      e = launch_decode_mfma(a, desc->head_dim, desc->kv_dtype == ROLLATTN_FP8_E4M3, grid, s);
    }
    prof.stop();
  }
  if (e != hipSuccess) return fail_hip(e);
  e = launch_combine(a, desc->head_dim, !f32, s);
  if (e != hipSuccess) return fail_hip(e);
  return ROLLATTN_OK;
}

int attn_append(const rollattn_desc* desc, const void* q_chunk, const int32_t* q_lens, const int32_t* q_offsets,
                int32_t total_q, int32_t max_q_len, const void* k_pages, const void* v_pages,
                const int32_t* page_table, const int32_t* ctx_lens, void* out, void* workspace,
                size_t workspace_bytes, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (total_q < 0 || max_q_len < 0) return ROLLATTN_EINVAL;
  if (desc->q_dtype != ROLLATTN_F32 && desc->num_q_heads / desc->num_kv_heads > kAppendTileRows) return ROLLATTN_ESHAPE;
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
  a.tile_b = (const int32_t*)(base + w.item_b);
  a.tile_q0 = (const int32_t*)(base + w.item_start);
  a.batch = desc->batch; a.hq = desc->num_q_heads; a.hkv = desc->num_kv_heads;
  a.group = desc->num_q_heads / desc->num_kv_heads; a.max_pages = desc->max_pages_per_seq;
  a.tile_tokens = std::max(1, kAppendTileRows / a.group);
  a.total_q = total_q;
  a.scale_log2 = desc->sm_scale * 1.4426950408889634f;

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
  e = launch_plan_append(q_lens, desc->batch, a.tile_tokens, w.cap, a.header, (int32_t*)(base + w.item_b),
                         (int32_t*)(base + w.item_start), s);
  if (e != hipSuccess) return fail_hip(e);
  {
    ProfileScope prof(s);
    const int grid = (int)std::min<int64_t>((int64_t)w.cap * a.hkv, INT32_MAX);
    e = launch_append_mfma(a, desc->head_dim, desc->kv_dtype == ROLLATTN_FP8_E4M3, grid, s);
    prof.stop();
  }
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

int rollattn_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_profile = on != 0;
  return ROLLATTN_OK;
}

int rollattn_profile_read(float* ms_out, int cap) {
  std::vector<EventPair> evs;
  {
    std::lock_guard<std::mutex> lk(g_mu);
    evs.swap(g_events);
  }
  int n = 0;
  for (auto& ev : evs) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(ev.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
    (void)hipEventDestroy(ev.a);
    (void)hipEventDestroy(ev.b);
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
    default: return "unknown status";
  }
}

const char* rollattn_last_hip_error(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  static thread_local std::string copy;
  copy = g_hip_error;
  return copy.c_str();
}

int rollattn_version(void) { return 100; }

}  // extern "C"
