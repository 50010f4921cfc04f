// Decode step for groups of trajectories that share a prompt (their page tables alias the same
// physical pages for the first tokens): the shared range is read once per group, for all the
// group's query heads, instead of once per trajectory.
//
//   prep:   per group, the shared length actually used: S = floor32(min(shared_lens[group],
//           min over the group of L_b - 1)), so that every trajectory keeps at least its current
//           token for itself and the private part starts on a block boundary; then the inputs of
//           the two halves: for the shared half one "chunk" per group (its members' query rows) on
//           a KV range of S tokens behind the first member's table; for the private half every
//           trajectory's table shifted left by S / 16 entries and its length reduced by S.
//   merge:  each half returns its own softmax-normalised rows o1, o2 and the log2 of its
//           denominators d1, d2; the row over the whole context is
//           (2^d1 o1 + 2^d2 o2) / (2^d1 + 2^d2), taken relative to max(d1, d2).
#include "rollattn_internal.h"

namespace rollattn {

namespace {

constexpr int kThreads = 256;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(kThreads) void shared_prep_kernel(const int32_t* __restrict__ ctx_lens,
                                                               const int32_t* __restrict__ shared_lens,
                                                               const int32_t* __restrict__ page_table, int32_t batch,
                                                               int32_t group_size, int32_t max_pages,
                                                               int32_t* __restrict__ grp_ctx, int32_t* __restrict__ grp_qlens,
                                                               int32_t* __restrict__ grp_qoff, int32_t* __restrict__ sfx_ctx,
                                                               int32_t* __restrict__ sfx_table) {
  const int b = blockIdx.x;
  const int grp = b / group_size;
  int s = shared_lens[grp];
  for (int m = 0; m < group_size; ++m) s = min(s, ctx_lens[grp * group_size + m] - 1);
  s = max(s, 0) & ~(kBlockTokens - 1);
  if (threadIdx.x == 0) {
    sfx_ctx[b] = ctx_lens[b] - s;
    if (b == grp * group_size) {
      grp_ctx[grp] = s;
      grp_qlens[grp] = group_size;
      grp_qoff[grp] = grp * group_size;
      if (grp == batch / group_size - 1) grp_qoff[grp + 1] = batch;
    }
  }
  const int shift = s / kPageSize;
  const int live = (ctx_lens[b] + kPageSize - 1) / kPageSize;
  for (int p = threadIdx.x; p < max_pages; p += kThreads)
    sfx_table[(size_t)b * max_pages + p] = (p + shift < live) ? page_table[(size_t)b * max_pages + p + shift] : -1;
}

// Attention over the union of two disjoint token ranges from the results over each (one wave per row): weights
// 2^d1 and 2^d2 on the two outputs, log2(2^d1 + 2^d2) as the new denominator's logarithm.  A side that saw nothing
// (d = -inf) has weight 0; when both saw nothing the row is zero and its logarithm -inf.
template <int D, typename T>
__global__ __launch_bounds__(kThreads) void merge_states_kernel(const T* o1, const float* __restrict__ d1, const T* o2,
                                                                const float* __restrict__ d2, T* out, float* d_out, long rows) {
  constexpr int kPer = D / 64;                            // consecutive elements per lane, moved as one vector
  typedef T vec_t __attribute__((ext_vector_type(kPer)));
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const size_t off = (size_t)row * D + lane * kPer;
  const vec_t v1 = *(const vec_t*)(o1 + off), v2 = *(const vec_t*)(o2 + off);   // out may be o1 or o2: read first
  const float a = d1[row], b = d2[row];
  const float top = fmaxf(a, b);
  const float m = (top == -INFINITY) ? 0.f : top;
  const float wa = __builtin_amdgcn_exp2f(a - m), wb = __builtin_amdgcn_exp2f(b - m);   // 2^-inf = 0
  const float tot = wa + wb;
  const float inv = tot > 0.f ? 1.f / tot : 0.f;
  vec_t r;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    // an empty side may hold anything (zeros by this library's calls): its weight is an exact zero, but keep
    // non-finite leftovers of other producers out of the sum
    const float x1 = wa > 0.f ? (float)v1[e] : 0.f, x2 = wb > 0.f ? (float)v2[e] : 0.f;
    r[e] = (T)((wa * x1 + wb * x2) * inv);
  }
  *(vec_t*)(out + off) = r;
  if (d_out && lane == 0) d_out[row] = tot > 0.f ? m + __builtin_amdgcn_logf(tot) : -INFINITY;
}

}  // namespace

hipError_t launch_shared_prep(const int32_t* ctx_lens, const int32_t* shared_lens, const int32_t* page_table, int32_t batch,
                              int32_t group_size, int32_t max_pages, int32_t* grp_ctx, int32_t* grp_qlens, int32_t* grp_qoff,
                              int32_t* sfx_ctx, int32_t* sfx_table, hipStream_t s) {
  hipLaunchKernelGGL(shared_prep_kernel, dim3(batch), dim3(kThreads), 0, s, ctx_lens, shared_lens, page_table, batch, group_size,
                     max_pages, grp_ctx, grp_qlens, grp_qoff, sfx_ctx, sfx_table);
  return hipGetLastError();
}

hipError_t launch_merge_states(const void* o1, const float* d1, const void* o2, const float* d2, void* out, float* d_out,
                               long rows, int head_dim, bool f32, hipStream_t s) {
  const int grid = (int)((rows + kThreads / 64 - 1) / (kThreads / 64));
  if (grid == 0) return hipSuccess;
  if (head_dim == 128 && !f32) {
    hipLaunchKernelGGL((merge_states_kernel<128, __bf16>), dim3(grid), dim3(kThreads), 0, s, (const __bf16*)o1, d1, (const __bf16*)o2, d2, (__bf16*)out, d_out, rows);
  } else if (head_dim == 64 && !f32) {
    hipLaunchKernelGGL((merge_states_kernel<64, __bf16>), dim3(grid), dim3(kThreads), 0, s, (const __bf16*)o1, d1, (const __bf16*)o2, d2, (__bf16*)out, d_out, rows);
  } else if (head_dim == 128) {
    hipLaunchKernelGGL((merge_states_kernel<128, float>), dim3(grid), dim3(kThreads), 0, s, (const float*)o1, d1, (const float*)o2, d2, (float*)out, d_out, rows);
  } else if (head_dim == 64) {
    hipLaunchKernelGGL((merge_states_kernel<64, float>), dim3(grid), dim3(kThreads), 0, s, (const float*)o1, d1, (const float*)o2, d2, (float*)out, d_out, rows);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rollattn
