// float32 attention on the vector ALUs: decode pieces and (row-at-a-time) append.
//
// One workgroup handles one (KV piece, KV head, tile of up to 4 query heads).  Each token row
// is read by D/4 adjacent lanes with one 16-byte load each; the partial dot products are
// summed across those lanes with wavefront xor-shuffles; every lane group keeps its own
// online-softmax state (max, sum, weighted values) and the groups are merged through LDS
// with the log-sum-exp rule at the end.
#include "rollattn_internal.h"

namespace rollattn {

namespace {

constexpr int kThreads = 256;
constexpr int kHT = kF32HeadTile;   // query heads per row

template <int D>
struct F32Geo {
  static constexpr int kLanesPerTok = D / 4;
  static constexpr int kTokPerWave = 64 / kLanesPerTok;
  static constexpr int kGroups = (kThreads / 64) * kTokPerWave;   // independent softmax states
};

// Attention of up to kHT query rows (same KV head) over tokens [0, len) of a paged range whose
// page ids start at table[0].  Leaves un-normalised o in o_out[h][D] (LDS), and max (log2
// units) / sum in ml_out[h][2].  All 256 threads must call it.
template <int D>
__device__ void attend_f32(const float* const* qrows, int n_heads, const float* k_pages, const float* v_pages,
                           const int32_t* table, int len, int hkv, int g, float scale_log2,
                           float (*o_part)[kHT][D], float (*ml_part)[kHT][2], float (*o_out)[D],
                           float (*ml_out)[2]) {
  using G_ = F32Geo<D>;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int sub = lane / G_::kLanesPerTok;          // token slot within the wave
  const int dl = lane % G_::kLanesPerTok;           // which 4 dims
  const int grp = (tid >> 6) * G_::kTokPerWave + sub;

  float4 q[kHT];
#pragma unroll
  for (int h = 0; h < kHT; ++h) q[h] = (h < n_heads) ? *(const float4*)(qrows[h] + dl * 4) : make_float4(0, 0, 0, 0);
  float4 acc[kHT];
  float m[kHT], l[kHT];
#pragma unroll
  for (int h = 0; h < kHT; ++h) {
    acc[h] = make_float4(0, 0, 0, 0);
    m[h] = -INFINITY;
    l[h] = 0.f;
  }
  for (int t = grp; t < len; t += G_::kGroups) {
    const int pid = table[t / kPageSize];
    const size_t off = (((size_t)pid * hkv + g) * kPageSize + (t % kPageSize)) * D + dl * 4;
    const float4 kv = *(const float4*)(k_pages + off);
    const float4 vv = *(const float4*)(v_pages + off);
#pragma unroll
    for (int h = 0; h < kHT; ++h) {
      float s = q[h].x * kv.x + q[h].y * kv.y + q[h].z * kv.z + q[h].w * kv.w;
#pragma unroll
      for (int off2 = 1; off2 < G_::kLanesPerTok; off2 <<= 1) s += __shfl_xor(s, off2, 64);
      s *= scale_log2;
      const float m_new = fmaxf(m[h], s);
      const float alpha = __builtin_amdgcn_exp2f(m[h] - m_new);
      const float p = __builtin_amdgcn_exp2f(s - m_new);
      l[h] = l[h] * alpha + p;
      acc[h].x = acc[h].x * alpha + p * vv.x;
      acc[h].y = acc[h].y * alpha + p * vv.y;
      acc[h].z = acc[h].z * alpha + p * vv.z;
      acc[h].w = acc[h].w * alpha + p * vv.w;
      m[h] = m_new;
    }
  }
#pragma unroll
  for (int h = 0; h < kHT; ++h) {
    *(float4*)(&o_part[grp][h][dl * 4]) = acc[h];
    if (dl == 0) {
      ml_part[grp][h][0] = m[h];
      ml_part[grp][h][1] = l[h];
    }
  }
  __syncthreads();
  for (int e = tid; e < kHT * D; e += kThreads) {
    const int h = e / D, d = e % D;
    float mmax = -INFINITY;
    for (int gi = 0; gi < G_::kGroups; ++gi) mmax = fmaxf(mmax, ml_part[gi][h][0]);
    float o = 0.f, ls = 0.f;
    for (int gi = 0; gi < G_::kGroups; ++gi) {
      const float mg = ml_part[gi][h][0];
      const float f = (mg == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mg - mmax);
      o += f * o_part[gi][h][d];
      ls += f * ml_part[gi][h][1];
    }
    o_out[h][d] = o;
    if (d == 0) {
      ml_out[h][0] = mmax;
      ml_out[h][1] = ls;
    }
  }
  __syncthreads();
}

// Decode in float32: every workgroup is one worker of the block partition (see plan.hip) and walks
// its run of 32-token blocks one row segment at a time.
template <int D>
__global__ __launch_bounds__(kThreads) void decode_f32_kernel(const DecodeArgs a) {
  using G_ = F32Geo<D>;
  __shared__ __attribute__((aligned(16))) float o_part[G_::kGroups][kHT][D];
  __shared__ float ml_part[G_::kGroups][kHT][2];
  __shared__ __attribute__((aligned(16))) float o_out[kHT][D];
  __shared__ float ml_out[kHT][2];
  const int tid = threadIdx.x;
  const int group = a.group, hkv = a.hkv, rows_per_b = a.rows_per_b;
  const int n_ht = rows_per_b / hkv;
  const int worker = blockIdx.x;
  const int4 st = *(const int4*)(a.wstart + 4 * worker);   // (b, r << 20 | block, L_b, run length)
  if (st.x < 0) return;
  int left = st.w;
  int b = st.x, r = st.y >> 20, blk = st.y & 0xFFFFF, n = (st.z + kBlockTokens - 1) / kBlockTokens;
  bool first_segment = true;
  while (left > 0) {
    const int cnt = min(left, n - blk);                 // blocks of this row that are ours
    const int ctx = a.ctx_lens[b];
    const int tok0 = blk * kBlockTokens;
    const int len = min(ctx, (blk + cnt) * kBlockTokens) - tok0;
    const int g = r / n_ht;
    const int h0 = (r - g * n_ht) * kHT;
    const int n_heads = min(kHT, group - h0);
    const float* qrows[kHT];
#pragma unroll
    for (int h = 0; h < kHT; ++h)
      qrows[h] = (const float*)a.q + ((size_t)b * a.hq + (size_t)g * group + h0 + min(h, n_heads - 1)) * D;
    attend_f32<D>(qrows, n_heads, (const float*)a.k_pages, (const float*)a.v_pages,
                  a.page_table + (size_t)b * a.max_pages + tok0 / kPageSize, len, hkv, g, a.scale_log2, o_part,
                  ml_part, o_out, ml_out);
    const bool whole = (blk == 0 && cnt == n);
    for (int e = tid; e < n_heads * D; e += kThreads) {
      const int h = e / D, d = e % D;
      if (whole) {
        const size_t orow = (size_t)b * a.hq + (size_t)g * group + h0 + h;
        ((float*)a.out)[orow * D + d] = o_out[h][d] / ml_out[h][1];
        if (a.lse && d == 0) a.lse[orow] = ml_out[h][0] + __builtin_amdgcn_logf(ml_out[h][1]);
      } else {
        const size_t slot = (size_t)worker * 2 + (first_segment ? 0 : 1);
        a.partial_o[(slot * kHT + h) * D + d] = o_out[h][d];
        if (d == 0) {
          a.partial_ml[(slot * kHT + h) * 2 + 0] = ml_out[h][0];
          a.partial_ml[(slot * kHT + h) * 2 + 1] = ml_out[h][1];
        }
      }
    }
    __syncthreads();
    first_segment = false;
    left -= cnt;
    if (left > 0) {                                      // next row of the sequence
      blk = 0;
      if (++r == rows_per_b) {
        r = 0;
        do {
          ++b;
          n = a.prefix[b + 1] - a.prefix[b];
        } while (n == 0);
      }
    }
  }
}

// Append in float32: one workgroup per (query row, KV head, head tile); row i of trajectory b
// sees tokens [0, L_b - n_b + i].
template <int D>
__global__ __launch_bounds__(kThreads) void append_f32_kernel(const AppendArgs a, int total_q) {
  using G_ = F32Geo<D>;
  __shared__ __attribute__((aligned(16))) float o_part[G_::kGroups][kHT][D];
  __shared__ float ml_part[G_::kGroups][kHT][2];
  __shared__ __attribute__((aligned(16))) float o_out[kHT][D];
  __shared__ float ml_out[kHT][2];
  const int tid = threadIdx.x;
  const int group = a.group, hkv = a.hkv;
  const int n_ht = (group + kHT - 1) / kHT;
  const long n_work = (long)total_q * hkv * n_ht;
  for (long work = blockIdx.x; work < n_work; work += gridDim.x) {
    const int row = (int)(work / (hkv * n_ht));
    const int g = (int)((work - (long)row * hkv * n_ht) / n_ht);
    const int h0 = (int)(work % n_ht) * kHT;
    const int n_heads = min(kHT, group - h0);
    // trajectory of this packed row: largest b with q_offsets[b] <= row
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (a.q_offsets[mid] <= row) lo = mid; else hi = mid;
    }
    const int b = lo;
    const int i = row - a.q_offsets[b];
    const int len = a.ctx_lens[b] - a.q_lens[b] + i + 1;
    const float* qrows[kHT];
#pragma unroll
    for (int h = 0; h < kHT; ++h)
      qrows[h] = (const float*)a.q + ((size_t)row * a.hq + (size_t)g * group + h0 + min(h, n_heads - 1)) * D;
    attend_f32<D>(qrows, n_heads, (const float*)a.k_pages, (const float*)a.v_pages,
                  a.page_table + (size_t)b * a.max_pages, len, hkv, g, a.scale_log2, o_part, ml_part, o_out,
                  ml_out);
    for (int e = tid; e < n_heads * D; e += kThreads) {
      const int h = e / D, d = e % D;
      const size_t orow = (size_t)row * a.hq + (size_t)g * group + h0 + h;
      ((float*)a.out)[orow * D + d] = o_out[h][d] / ml_out[h][1];
      if (a.lse && d == 0) a.lse[orow] = ml_out[h][0] + __builtin_amdgcn_logf(ml_out[h][1]);
    }
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_decode_f32(const DecodeArgs& a, int head_dim, int grid, hipStream_t s) {
  if (head_dim == 64) {
    hipLaunchKernelGGL((decode_f32_kernel<64>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128) {
    hipLaunchKernelGGL((decode_f32_kernel<128>), dim3(grid), dim3(kThreads), 0, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_append_f32(const AppendArgs& a, int head_dim, int grid, hipStream_t s) {
  const int total_q = a.total_q;   // rows are enumerated directly, no tile list
  if (head_dim == 64) {
    hipLaunchKernelGGL((append_f32_kernel<64>), dim3(grid), dim3(kThreads), 0, s, a, total_q);
  } else if (head_dim == 128) {
    hipLaunchKernelGGL((append_f32_kernel<128>), dim3(grid), dim3(kThreads), 0, s, a, total_q);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rollattn
