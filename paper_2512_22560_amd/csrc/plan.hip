// Device-side planning: turns ctx_lens / q_lens into compact work lists without a host
// round trip, so a call never synchronises.  The partition depends on the lengths only,
// never on physical page ids.
#include "rollattn_internal.h"

namespace rollattn {

namespace {

constexpr int kPlanThreads = 1024;

constexpr int kLdsPrefix = 8192;   // batches up to this size keep the scan in LDS for the searches

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

// Decode partition.  Every trajectory is cut into blocks of kBlockTokens tokens; the rows
// (trajectory b, row r in [0, rows_per_b)) are laid end to end, b outermost, each with
// n_b = ceil(L_b / kBlockTokens) blocks; the resulting sequence of T blocks is dealt to the W
// workers in equal contiguous runs of per = ceil(T / W) blocks.  Written out: the exclusive
// scan of n_b, the run length, T, and for every worker one 16-byte record with all it needs to
// start: (b, r << 20 | block, L_b, blocks in its run), or b = -1 for a worker without blocks.
// With q_lens given (mixed step) only the trajectories with q_lens[b] == 1 take part; the others count as empty.
__global__ __launch_bounds__(kPlanThreads) void plan_decode_kernel(
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ q_lens, int32_t batch, int32_t rows_per_b,
    int32_t workers, int32_t slots, int32_t* __restrict__ header, int32_t* __restrict__ prefix, int32_t* __restrict__ wstart) {
  __shared__ int wave_tot[kPlanThreads / 64];
  __shared__ int prefix_s[kLdsPrefix + 1];
  const int tid = threadIdx.x;
  const bool in_lds = batch <= kLdsPrefix;
  __shared__ int len_s[kLdsPrefix];
  int running = 0;
  for (int b0 = 0; b0 < batch; b0 += kPlanThreads) {
    const int b = b0 + tid;
    const int len = (b < batch && (!q_lens || q_lens[b] == 1)) ? ctx_lens[b] : 0;
    const int count = (len + kBlockTokens - 1) / kBlockTokens;
    int tile_total;
    const int first = running + block_exclusive_scan(count, wave_tot, &tile_total);
    if (b < batch) {
      prefix[b] = first;
      if (in_lds) {
        prefix_s[b] = first;
        len_s[b] = len;
      }
    }
    running += tile_total;
  }
  if (tid == 0) {
    prefix[batch] = running;
    if (in_lds) prefix_s[batch] = running;
  }
  const int total = running * rows_per_b;
  const int per = max(1, (total + workers - 1) / workers);
  if (tid == 0) {
    header[kPlanPer] = per;
    header[kPlanTotal] = total;
    header[kPlanWorkers] = workers;
    header[kPlanRowsPerB] = rows_per_b;
  }
  __threadfence_block();
  __syncthreads();   // prefix[] written above is read below by other threads of this workgroup
  for (int w = tid; w < slots; w += kPlanThreads) {
    const long x = (long)w * per;
    int4 st = make_int4(-1, 0, 0, 0);
    if (w < workers && x < total) {
      // largest b with rows_per_b * prefix[b] <= x (rows without blocks can never be the answer
      // because the next row then starts at the same position)
      const int* pf = in_lds ? prefix_s : prefix;
      int lo = 0, hi = batch;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((long)rows_per_b * pf[mid] <= x) lo = mid; else hi = mid;
      }
      const int n = pf[lo + 1] - pf[lo];
      const int rem = (int)(x - (long)rows_per_b * pf[lo]);
      const int mine = (int)min((long)per, (long)total - x);
      st = make_int4(lo, ((rem / n) << 20) | (rem % n), in_lds ? len_s[lo] : ctx_lens[lo], mine);   // lo has blocks, so it takes part
    }
    *(int4*)(wstart + 4 * w) = st;
  }
}

// Append work list: each chunk cut into tiles of tile_tokens query tokens.  A tile's cost grows
// with its trajectory's context, and workgroups are dispatched in list order, so (for batches that
// fit the ranking in LDS) trajectories are listed longest context first: the long tiles start
// early and the short ones fill the tail.  For the same reason a chunk's tiles are listed last
// tile first.
constexpr int kRankBatch = 4096;
__global__ __launch_bounds__(kPlanThreads) void plan_append_kernel(
    const int32_t* __restrict__ q_lens, const int32_t* __restrict__ q_offsets, const int32_t* __restrict__ ctx_lens,
    int32_t batch, int32_t tile_tokens, int32_t cap, bool skip_unit_chunks, int32_t* __restrict__ header,
    int32_t* __restrict__ tile_rec) {
  __shared__ int wave_tot[kPlanThreads / 64];
  __shared__ int len_s[kRankBatch];
  __shared__ int order_s[kRankBatch];
  const int tid = threadIdx.x;
  const bool ranked = batch <= kRankBatch;
  if (ranked) {
    for (int b = tid; b < batch; b += kPlanThreads) len_s[b] = ctx_lens[b];
    __syncthreads();
    for (int b = tid; b < batch; b += kPlanThreads) {
      const int mine = len_s[b];
      int rank = 0;
      for (int o = 0; o < batch; ++o) {
        const int other = len_s[o];
        rank += (other > mine || (other == mine && o < b)) ? 1 : 0;
      }
      order_s[rank] = b;
    }
    __syncthreads();
  }
  __shared__ int first_s[kPlanThreads], count_s[kPlanThreads], b_s[kPlanThreads], qlen_s[kPlanThreads], ctx_s[kPlanThreads],
      qoff_s[kPlanThreads];
  int running = 0;
  for (int p0 = 0; p0 < batch; p0 += kPlanThreads) {
    const int p = p0 + tid;
    int b = 0, count = 0, q_len = 0;
    if (p < batch) {
      b = ranked ? order_s[p] : p;
      q_len = q_lens[b];
      count = (q_len + tile_tokens - 1) / tile_tokens;
      if (skip_unit_chunks && q_len == 1) count = 0;   // mixed step: the decode kernel takes these
    }
    int tile_total;
    const int first = running + block_exclusive_scan(count, wave_tot, &tile_total);
    first_s[tid] = first;
    count_s[tid] = count;
    b_s[tid] = b;
    qlen_s[tid] = q_len;
    ctx_s[tid] = p < batch ? ctx_lens[b] : 0;
    qoff_s[tid] = p < batch ? q_offsets[b] : 0;
    __syncthreads();
    // One 32-byte record per tile with everything the tile's workgroup needs to start, so that it gets there with
    // one dependent load instead of a chain of them: (b, first row, n_b, L_b, q_offsets[b]).  The tiles of these
    // trajectories are dealt to the threads one by one (a trajectory may have hundreds): a tile finds its
    // trajectory as the last one of the group that starts at or before it (those without tiles start where the
    // next one starts, and are never the last such).
    const int end = min(running + tile_total, cap);
    for (int t = running + tid; t < end; t += kPlanThreads) {
      int lo = 0, hi = kPlanThreads;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (first_s[mid] <= t) lo = mid; else hi = mid;
      }
      const int s = t - first_s[lo];
      int4* rec = (int4*)(tile_rec + (size_t)t * kTileRecWords);
      rec[0] = make_int4(b_s[lo], (count_s[lo] - 1 - s) * tile_tokens, qlen_s[lo], ctx_s[lo]);   // a chunk's last tile sees the most context
      rec[1] = make_int4(qoff_s[lo], 0, 0, 0);
    }
    __syncthreads();
    running += tile_total;
  }
  if (tid == 0) header[kPlanTiles] = running < cap ? running : cap;
}

}  // namespace

hipError_t launch_plan_decode(const int32_t* ctx_lens, const int32_t* q_lens, int32_t batch, int32_t rows_per_b,
                              int32_t workers, int32_t slots, int32_t* header, int32_t* prefix, int32_t* wstart, hipStream_t s) {
  hipLaunchKernelGGL(plan_decode_kernel, dim3(1), dim3(kPlanThreads), 0, s, ctx_lens, q_lens, batch, rows_per_b, workers,
                     slots, header, prefix, wstart);
  return hipGetLastError();
}

hipError_t launch_plan_append(const int32_t* q_lens, const int32_t* q_offsets, const int32_t* ctx_lens, int32_t batch,
                              int32_t tile_tokens, int32_t cap, bool skip_unit_chunks, int32_t* header, int32_t* tile_rec,
                              hipStream_t s) {
  hipLaunchKernelGGL(plan_append_kernel, dim3(1), dim3(kPlanThreads), 0, s, q_lens, q_offsets, ctx_lens, batch, tile_tokens,
                     cap, skip_unit_chunks, header, tile_rec);
  return hipGetLastError();
}

}  // namespace rollattn
