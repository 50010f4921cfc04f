// Split-K merge: one wave per (trajectory, query head) folds the partial results that the
// decode workers left for rows they did not cover alone (max m_s in log2 units, sum l_s,
// un-normalised o_s) into the final row:
//   M = max_s m_s ;  out = sum_s 2^(m_s - M) o_s / sum_s 2^(m_s - M) l_s
// which equals the softmax over the whole context.  Which workers touched a row follows from
// the plan alone: the row occupies blocks [R0, R1) of the global sequence and worker w owns
// [w * per, (w + 1) * per).  A worker keeps at most two partials, slot 0 for the first row
// segment of its run and slot 1 for the last; the only segment that lands in slot 1 is the one
// of the worker whose run began before this row.  Rows covered by a single worker were already
// written by it; rows without tokens are zero-filled here.
#include "rollattn_internal.h"

namespace rollattn {

namespace {

constexpr int kThreads = 256;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <int D, bool OUT_BF16>
__global__ __launch_bounds__(kThreads) void combine_kernel(const DecodeArgs a) {
  constexpr int kPer = D / 64;   // consecutive output elements per lane
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);   // b * Hq + h
  if (row >= (long)a.batch * a.hq) return;
  const int b = (int)(row / a.hq);
  const int h = (int)(row % a.hq);
  if (a.q_lens && a.q_lens[b] != 1) return;                 // mixed step: not a decode row, nothing of ours to write
  const size_t orow = (size_t)(a.q_offsets ? a.q_offsets[b] : b) * a.hq + h;   // where this row's output goes
  const int ht = a.head_tile;
  const int n_ht = a.rows_per_b / a.hkv;
  const int g = h / a.group, j = h % a.group;
  const int r = g * n_ht + j / ht, jj = j % ht;
  const int per = a.header[kPlanPer];
  const int first = a.prefix[b];
  const int n = a.prefix[b + 1] - first;
  const long r0 = (long)a.rows_per_b * first + (long)r * n;
  const int wf = n ? (int)(r0 / per) : 0;
  const int wl = n ? (int)((r0 + n - 1) / per) : 0;
  if (n && wf == wl) return;      // one worker had the whole row
  float o[kPer];
#pragma unroll
  for (int e = 0; e < kPer; ++e) o[e] = 0.f;
  float inv = 0.f;
  if (n) {
    const int first_slot = ((long)wf * per < r0) ? 1 : 0;
    const int pieces = wl - wf + 1;
    float mmax = -INFINITY;
    for (int s = lane; s < pieces; s += 64) {
      const size_t slot = (size_t)(wf + s) * 2 + (s == 0 ? first_slot : 0);
      mmax = fmaxf(mmax, a.partial_ml[(slot * ht + jj) * 2]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mmax = fmaxf(mmax, __shfl_xor(mmax, off, 64));
    float lsum = 0.f;
#pragma unroll 4
    for (int s = 0; s < pieces; ++s) {
      const size_t slot = (size_t)(wf + s) * 2 + (s == 0 ? first_slot : 0);
      const float* ml = a.partial_ml + (slot * ht + jj) * 2;
      const float f = __builtin_amdgcn_exp2f(ml[0] - mmax);
      lsum += f * ml[1];
      const float* src = a.partial_o + (slot * ht + jj) * D + lane * kPer;
#pragma unroll
      for (int e = 0; e < kPer; ++e) o[e] += f * src[e];
    }
    inv = 1.f / lsum;
    if (a.lse && lane == 0) a.lse[orow] = mmax + __builtin_amdgcn_logf(lsum);
  } else if (a.lse && lane == 0) {
    a.lse[orow] = -INFINITY;
  }
  if (OUT_BF16) {
    __bf16* dst = (__bf16*)a.out + orow * D + lane * kPer;
    if (kPer == 2) {
      bf16x2 pr;
      pr[0] = (__bf16)(o[0] * inv);
      pr[1] = (__bf16)(o[kPer - 1] * inv);
      *(bf16x2*)dst = pr;
    } else {
      dst[0] = (__bf16)(o[0] * inv);
    }
  } else {
    float* dst = (float*)a.out + orow * D + lane * kPer;
#pragma unroll
    for (int e = 0; e < kPer; ++e) dst[e] = o[e] * inv;
  }
}

// Copies logical tokens of one (trajectory, KV head) out of a pool, byte for byte.
__global__ __launch_bounds__(kThreads) void gather_kernel(const unsigned char* pages, const int32_t* page_table,
                                                          const int32_t* ctx_lens, int32_t b, int32_t kv_head,
                                                          int32_t hkv, int32_t max_pages, int32_t row_bytes,
                                                          unsigned char* dst) {
  const int len = ctx_lens[b];
  const int vec_per_row = row_bytes / 16;
  const long n_vec = (long)len * vec_per_row;
  for (long i = (long)blockIdx.x * kThreads + threadIdx.x; i < n_vec; i += (long)gridDim.x * kThreads) {
    const int t = (int)(i / vec_per_row), c = (int)(i % vec_per_row);
    const int pid = page_table[(size_t)b * max_pages + t / kPageSize];
    const size_t off = (((size_t)pid * hkv + kv_head) * kPageSize + (t % kPageSize)) * row_bytes + c * 16;
    *(uint4*)(dst + (size_t)t * row_bytes + c * 16) = *(const uint4*)(pages + off);
  }
}

// Counts what the entry points take on trust (see rollattn_debug_check_inputs): one workgroup per trajectory.
__global__ __launch_bounds__(kThreads) void check_inputs_kernel(const int32_t* page_table, const int32_t* ctx_lens,
                                                                const int32_t* q_lens, const int32_t* q_offsets,
                                                                int32_t batch, int32_t max_pages, int64_t num_pages,
                                                                int32_t* counts) {
  const int b = blockIdx.x;
  const int len = ctx_lens[b];
  const bool bad_len = len < 0 || (long)len > (long)max_pages * kPageSize;
  const int live = bad_len ? 0 : (len + kPageSize - 1) / kPageSize;
  int bad_ids = 0;
  for (int pg = threadIdx.x; pg < live; pg += kThreads) {
    const int id = page_table[(size_t)b * max_pages + pg];
    bad_ids += (id < 0 || id >= num_pages) ? 1 : 0;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) bad_ids += __shfl_xor(bad_ids, off, 64);
  if ((threadIdx.x & 63) == 0 && bad_ids) atomicAdd(counts + 1, bad_ids);
  if (threadIdx.x == 0) {
    if (bad_len) atomicAdd(counts + 0, 1);
    if (q_lens) {
      const int n = q_lens[b];
      if (n < 0 || (!bad_len && n > len)) atomicAdd(counts + 2, 1);
      if (q_offsets && (q_offsets[b + 1] - q_offsets[b] != n || (b == 0 && q_offsets[0] != 0))) atomicAdd(counts + 3, 1);
    }
  }
}

__global__ void clear4_kernel(int32_t* counts) {
  if (threadIdx.x < 4) counts[threadIdx.x] = 0;
}

}  // namespace

hipError_t launch_check_inputs(const int32_t* page_table, const int32_t* ctx_lens, const int32_t* q_lens,
                               const int32_t* q_offsets, int32_t batch, int32_t max_pages, int64_t num_pages,
                               int32_t* counts, hipStream_t s) {
  hipLaunchKernelGGL(clear4_kernel, dim3(1), dim3(64), 0, s, counts);
  hipLaunchKernelGGL(check_inputs_kernel, dim3(batch), dim3(kThreads), 0, s, page_table, ctx_lens, q_lens, q_offsets, batch,
                     max_pages, num_pages, counts);
  return hipGetLastError();
}

hipError_t launch_combine(const DecodeArgs& a, int head_dim, bool out_bf16, hipStream_t s) {
  const long rows = (long)a.batch * a.hq;
  const int grid = (int)((rows + kThreads / 64 - 1) / (kThreads / 64));
  if (grid == 0) return hipSuccess;
  if (head_dim == 128 && out_bf16) {
    hipLaunchKernelGGL((combine_kernel<128, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128) {
    hipLaunchKernelGGL((combine_kernel<128, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && out_bf16) {
    hipLaunchKernelGGL((combine_kernel<64, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64) {
    hipLaunchKernelGGL((combine_kernel<64, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_gather(const void* pages, const int32_t* page_table, const int32_t* ctx_lens, int32_t b,
                         int32_t kv_head, int32_t hkv, int32_t max_pages, int32_t row_bytes, void* dst,
                         hipStream_t s) {
  hipLaunchKernelGGL(gather_kernel, dim3(64), dim3(kThreads), 0, s, (const unsigned char*)pages, page_table,
                     ctx_lens, b, kv_head, hkv, max_pages, row_bytes, (unsigned char*)dst);
  return hipGetLastError();
}

}  // namespace rollattn
