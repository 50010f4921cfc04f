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

template <int D>
__global__ __launch_bounds__(kThreads) void shared_merge_kernel(const __bf16* __restrict__ o1, const float* __restrict__ d1,
                                                                const __bf16* __restrict__ o2, const float* __restrict__ d2,
                                                                __bf16* __restrict__ out, long rows) {
  constexpr int kPer = D / 64;
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float a = d1[row], b = d2[row];
  const float m = fmaxf(a, b);                        // the private half is never empty, so m is finite
  const float wa = __builtin_amdgcn_exp2f(a - m), wb = __builtin_amdgcn_exp2f(b - m);
  const float inv = 1.f / (wa + wb);
  const size_t off = (size_t)row * D + lane * kPer;
#pragma unroll
  for (int e = 0; e < kPer; ++e) out[off + e] = (__bf16)((wa * (float)o1[off + e] + wb * (float)o2[off + e]) * inv);
}

}  // namespace

hipError_t launch_shared_prep(const int32_t* ctx_lens, const int32_t* shared_lens, const int32_t* page_table, int32_t batch,
                              int32_t group_size, int32_t max_pages, int32_t* grp_ctx, int32_t* grp_qlens, int32_t* grp_qoff,
                              int32_t* sfx_ctx, int32_t* sfx_table, hipStream_t s) {
  hipLaunchKernelGGL(shared_prep_kernel, dim3(batch), dim3(kThreads), 0, s, ctx_lens, shared_lens, page_table, batch, group_size,
                     max_pages, grp_ctx, grp_qlens, grp_qoff, sfx_ctx, sfx_table);
  return hipGetLastError();
}

hipError_t launch_shared_merge(const void* o1, const float* d1, const void* o2, const float* d2, void* out, long rows,
                               int head_dim, hipStream_t s) {
  const int grid = (int)((rows + kThreads / 64 - 1) / (kThreads / 64));
  if (grid == 0) return hipSuccess;
  if (head_dim == 128) {
    hipLaunchKernelGGL((shared_merge_kernel<128>), dim3(grid), dim3(kThreads), 0, s, (const __bf16*)o1, d1, (const __bf16*)o2, d2, (__bf16*)out, rows);
  } else if (head_dim == 64) {
    hipLaunchKernelGGL((shared_merge_kernel<64>), dim3(grid), dim3(kThreads), 0, s, (const __bf16*)o1, d1, (const __bf16*)o2, d2, (__bf16*)out, rows);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rollattn
