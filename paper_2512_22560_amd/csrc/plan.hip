// Device-side planning: turns ctx_lens / q_lens into compact work lists without a host
// round trip, so a call never synchronises.  The partition depends on the lengths only,
// never on physical page ids.
#include "rollattn_internal.h"

namespace rollattn {

namespace {

constexpr int kPlanThreads = 1024;

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Exclusive scan of one int per thread across the workgroup; returns this thread's prefix
// and leaves the workgroup total in *total.
__device__ int block_exclusive_scan(int v, int* wave_tot /*[16]*/, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  int base = 0;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  int tot = 0;
  for (int w = 0; w < kPlanThreads / 64; ++w) tot += wave_tot[w];
  *total = tot;
  __syncthreads();
  return base + incl - v;
}

// Decode partition: pieces of C tokens, C the smallest kMinChunk << k (k <= kMaxDoublings)
// whose piece count fits `cap`, else one piece per trajectory (C = 0).
__global__ __launch_bounds__(kPlanThreads) void plan_decode_kernel(
    const int32_t* __restrict__ ctx_lens, int32_t batch, int32_t cap, int32_t* __restrict__ header,
    int32_t* __restrict__ item_b, int32_t* __restrict__ item_start, int32_t* __restrict__ row_first) {
  __shared__ int sums[kMaxDoublings + 1];
  __shared__ int wave_tot[kPlanThreads / 64];
  __shared__ int chunk_s;
  const int tid = threadIdx.x;
  if (tid <= kMaxDoublings) sums[tid] = 0;
  __syncthreads();
  int local[kMaxDoublings + 1];
#pragma unroll
  for (int k = 0; k <= kMaxDoublings; ++k) local[k] = 0;
  for (int b = tid; b < batch; b += kPlanThreads) {
    const int len = ctx_lens[b];
#pragma unroll
    for (int k = 0; k <= kMaxDoublings; ++k) {
      const int c = kMinChunk << k;
      local[k] += (len + c - 1) / c;
    }
  }
#pragma unroll
  for (int k = 0; k <= kMaxDoublings; ++k) {
    const int s = wave_sum(local[k]);
    if ((tid & 63) == 0 && s) atomicAdd(&sums[k], s);
  }
  __syncthreads();
  if (tid == 0) {
    int chosen = 0;
    for (int k = 0; k <= kMaxDoublings; ++k) {
      if (sums[k] <= cap) {
        chosen = kMinChunk << k;
        break;
      }
    }
    chunk_s = chosen;
  }
  __syncthreads();
  const int chunk = chunk_s;
  int running = 0;
  for (int b0 = 0; b0 < batch; b0 += kPlanThreads) {
    const int b = b0 + tid;
    int len = 0, count = 0;
    if (b < batch) {
      len = ctx_lens[b];
      count = chunk ? (len + chunk - 1) / chunk : (len > 0 ? 1 : 0);
    }
    int tile_total;
    const int first = running + block_exclusive_scan(count, wave_tot, &tile_total);
    if (b < batch) {
      row_first[b] = first;
      for (int s = 0; s < count; ++s) {
        item_b[first + s] = b;
        item_start[first + s] = s * chunk;
      }
    }
    running += tile_total;
  }
  if (tid == 0) {
    row_first[batch] = running;
    header[kPlanChunk] = chunk;
    header[kPlanItems] = running;
    header[kPlanCounter] = 0;
  }
}

// Append work list: each chunk cut into tiles of tile_tokens query tokens.
__global__ __launch_bounds__(kPlanThreads) void plan_append_kernel(
    const int32_t* __restrict__ q_lens, int32_t batch, int32_t tile_tokens, int32_t cap,
    int32_t* __restrict__ header, int32_t* __restrict__ tile_b, int32_t* __restrict__ tile_q0) {
  __shared__ int wave_tot[kPlanThreads / 64];
  const int tid = threadIdx.x;
  int running = 0;
  for (int b0 = 0; b0 < batch; b0 += kPlanThreads) {
    const int b = b0 + tid;
    int count = 0;
    if (b < batch) count = (q_lens[b] + tile_tokens - 1) / tile_tokens;
    int tile_total;
    const int first = running + block_exclusive_scan(count, wave_tot, &tile_total);
    for (int s = 0; s < count; ++s) {
      if (first + s < cap) {
        tile_b[first + s] = b;
        tile_q0[first + s] = s * tile_tokens;
      }
    }
    running += tile_total;
  }
  if (tid == 0) {
    header[kPlanTiles] = running < cap ? running : cap;
    header[kPlanCounter] = 0;
  }
}

}  // namespace

hipError_t launch_plan_decode(const int32_t* ctx_lens, int32_t batch, int32_t cap, int32_t* header,
                              int32_t* item_b, int32_t* item_start, int32_t* row_first, hipStream_t s) {
  hipLaunchKernelGGL(plan_decode_kernel, dim3(1), dim3(kPlanThreads), 0, s, ctx_lens, batch, cap, header,
                     item_b, item_start, row_first);
  return hipGetLastError();
}

hipError_t launch_plan_append(const int32_t* q_lens, int32_t batch, int32_t tile_tokens, int32_t cap,
                              int32_t* header, int32_t* tile_b, int32_t* tile_q0, hipStream_t s) {
  hipLaunchKernelGGL(plan_append_kernel, dim3(1), dim3(kPlanThreads), 0, s, q_lens, batch, tile_tokens, cap,
                     header, tile_b, tile_q0);
  return hipGetLastError();
}

}  // namespace rollattn
