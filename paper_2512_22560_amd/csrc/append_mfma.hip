// Observation-append attention (chunked causal prefill on a cached prefix) for bf16 queries
// over bf16 or FP8-E4M3 paged KV, on the gfx950 matrix cores.
//
// One workgroup = 256 query rows of one (trajectory, KV head): a row is a (chunk token, query
// head of the group) pair, token-major, so the G heads that share the KV head reuse every K/V
// tile.  Eight waves of 32 rows each walk the visible KV range in 64-token blocks (four
// pages) that the workgroup stages once through LDS (double buffered, global loads two
// blocks ahead of the one being consumed).  FP8 pools are widened to bf16
// while staging, so the tiles in LDS always hold bf16; page scales are applied in float to
// S (K scale) and to P (V scale).  Per 32-token sub-block a wave computes
//   S^T = K Q^T        tokens x rows, v_mfma_f32_32x32x16_bf16, K rows as A operand
//   O^T += V^T P^T     dims x rows, V read transposed with ds_read_b64_tr_b16
// The transposed products keep "row" on the lane axis in both accumulators: the softmax
// state is one scalar per lane (shared by two lanes) and P goes from accumulator registers
// straight into the B operand of the second product.
#include <type_traits>

#include "rollattn_internal.h"

namespace rollattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kRowsPerWave = 32;
static_assert(kWaves * kRowsPerWave == kAppendTileRows, "tile rows");
constexpr int kBlockTokens = 64;                   // KV tokens staged per step
constexpr float kSlack = 8.f;                      // log2 of the largest p tolerated before rescaling

// Row t of an S^T tile holds this token of its 16-token group: the middle two quads are
// swapped so that the 8 scores a lane ends up with are 8 consecutive tokens.
__device__ __forceinline__ int tau(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

__device__ __forceinline__ float xor32_max(float x) {
  uintx2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_add(float x) {
  uintx2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ void fp8x16_to_bf16(const uintx4 raw, uintx4& lo, uintx4& hi) {
  const uint32_t w[4] = {raw[0], raw[1], raw[2], raw[3]};
  uint32_t o[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    floatx2 a = __builtin_amdgcn_cvt_pk_f32_fp8(w[i], false);
    floatx2 b = __builtin_amdgcn_cvt_pk_f32_fp8(w[i], true);
    bf16x2 pa, pb;
    pa[0] = (__bf16)a[0]; pa[1] = (__bf16)a[1];
    pb[0] = (__bf16)b[0]; pb[1] = (__bf16)b[1];
    o[2 * i] = __builtin_bit_cast(uint32_t, pa);
    o[2 * i + 1] = __builtin_bit_cast(uint32_t, pb);
  }
  lo = uintx4{o[0], o[1], o[2], o[3]};
  hi = uintx4{o[4], o[5], o[6], o[7]};
}

template <int D, bool FP8>
__global__ __launch_bounds__(kThreads) void append_mfma_kernel(const AppendArgs a) {
  constexpr int kRowBytes = D * 2;                 // bf16 rows in LDS
  constexpr int kChunks = kRowBytes / 16;          // 16-byte chunks per LDS row
  constexpr int kTileBytes = kBlockTokens * kRowBytes;
  constexpr int kSrcRowBytes = D * (FP8 ? 1 : 2);  // row bytes in HBM
  constexpr int kSrcChunks = kSrcRowBytes / 16;
  constexpr int kLoads = (kBlockTokens * kSrcChunks + kThreads - 1) / kThreads;   // per pool, per thread
  constexpr int kKK = D / 16;                      // 16-deep steps of the QK product
  constexpr int kDT = D / 32;                      // 32-wide output tiles along D
  static_assert((kBlockTokens * kSrcChunks) % kThreads == 0 || kBlockTokens * kSrcChunks < kThreads, "staging shape");

  __shared__ __attribute__((aligned(16))) unsigned char k_lds[2][kTileBytes];
  __shared__ __attribute__((aligned(16))) unsigned char v_lds[2][kTileBytes];
  __shared__ float kscale_s[2][kBlockTokens / kPageSize];
  __shared__ float vscale_s[2][kBlockTokens / kPageSize];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31;   // row (B column) / K token row (A row) carried by this lane
  const int h2 = lane >> 5;    // half of the contraction this lane feeds

  const int group = a.group;
  const int hkv = a.hkv;
  const int tile_tokens = a.tile_tokens;
  const int n_tiles = a.header[kPlanTiles];
  const int tile = blockIdx.x / hkv;
  const int g = blockIdx.x - tile * hkv;
  if (tile >= n_tiles) return;
  const int b = a.tile_b[tile];
  const int q0 = a.tile_q0[tile];
  const int n_b = a.q_lens[b];
  const int ctx = a.ctx_lens[b];
  const int tokens_here = min(tile_tokens, n_b - q0);
  const int rows_here = tokens_here * group;
  const int pos0 = ctx - n_b + q0;                       // position of the tile's first token
  const int kv_end = pos0 + tokens_here;                 // tokens [0, kv_end) are visible to some row
  const int n_blocks = (kv_end + kBlockTokens - 1) / kBlockTokens;
  const int32_t* table = a.page_table + (size_t)b * a.max_pages;
  const size_t tile_stride = (size_t)kPageSize * kSrcRowBytes;

  // ---- this lane's query row
  const int row = wave * kRowsPerWave + n32;
  const bool row_ok = row < rows_here;
  const int tok_in_tile = row / group;
  const int head = g * group + (row - tok_in_tile * group);
  const int my_pos = row_ok ? pos0 + tok_in_tile : -1;   // last visible token of this row
  // wave-uniform bounds for skipping fully masked sub-blocks
  const int wave_last_row = min(wave * kRowsPerWave + kRowsPerWave - 1, rows_here - 1);
  const int wave_max_pos = (wave * kRowsPerWave < rows_here) ? pos0 + wave_last_row / group : -1;
  const int wave_min_pos = pos0 + (wave * kRowsPerWave) / group;

  bf16x8 qop[kKK];
  {
    const __bf16* qrow = (const __bf16*)a.q + ((size_t)(a.q_offsets[b] + q0 + tok_in_tile) * a.hq + head) * D;
#pragma unroll
    for (int kk = 0; kk < kKK; ++kk) {
      bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row_ok) v = *(const bf16x8*)(qrow + kk * 16 + h2 * 8);
      qop[kk] = v;
    }
  }

  floatx16 acc[kDT];
#pragma unroll
  for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const bool positive_scale = a.scale_log2 > 0.f;   // the usual case; FP8 page scales are positive too

  // ---- staging: thread's share of a 64-token block
  const int live_pages = (ctx + kPageSize - 1) / kPageSize;
  uintx4 kreg[2][kLoads], vreg[2][kLoads];   // two blocks in flight
  float ksc_r[2][kLoads], vsc_r[2][kLoads];  // FP8: scales of the page each wave-wide load came from
  // Branch-free on purpose: with every load in one straight line the hardware counter the K/V loads
  // are tracked with can be waited on partially, which is what keeps two blocks in flight.  Rows at
  // or past L_b (ragged last block, or a block index clamped at the end of the loop) re-read the
  // trajectory's last token instead: finite data that the causal / length mask never lets through.
  // Per thread and load, the byte offset inside a (page, head) tile never changes: only the page
  // does, and that is a scalar.  Two variants, the second with the row clamped to the last live slot
  // for loads that fall in (or past) the trajectory's last page.
  const int last_slot = (ctx - 1) % kPageSize;
  unsigned int goff[kLoads], goff_last[kLoads];
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const int idx = j * kThreads + tid;               // 16-byte chunk index within the block
    const int tslot = (idx / kSrcChunks) % kPageSize; // token slot within its page
    const int c = idx % kSrcChunks;
    goff[j] = tslot * kSrcRowBytes + c * 16;
    goff_last[j] = min(tslot, last_slot) * kSrcRowBytes + c * 16;
  }
  auto issue = [&](int blk, auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      // the 64 chunks a wave fetches with one instruction lie in one page: its id is a scalar
      const int pg = blk * (kBlockTokens / kPageSize) + ((j * kThreads + wave * 64) / kSrcChunks) / kPageSize;
      const int pid = table[min(pg, live_pages - 1)];
      if (FP8) {
        ksc_r[slot][j] = a.k_scale[pid];
        vsc_r[slot][j] = a.v_scale[pid];
      }
      const size_t tile_off = ((size_t)pid * hkv + g) * tile_stride;     // scalar
      const unsigned int off = (pg >= live_pages - 1) ? goff_last[j] : goff[j];
      if (kBlockTokens * kSrcChunks >= kThreads || (j * kThreads + tid) / kSrcChunks < kBlockTokens) {
        kreg[slot][j] = *(const uintx4*)((const unsigned char*)a.k_pages + tile_off + off);
        vreg[slot][j] = *(const uintx4*)((const unsigned char*)a.v_pages + tile_off + off);
      }
    }
  };
  auto commit = [&](int blk, auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;   // register slot and LDS buffer have the same parity
    constexpr int buf = slot;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      const int idx = j * kThreads + tid;
      const int trow = idx / kSrcChunks;
      const int c = idx % kSrcChunks;
      if (trow < kBlockTokens) {
        unsigned char* krow = k_lds[buf] + trow * kRowBytes;
        unsigned char* vrow = v_lds[buf] + trow * kRowBytes;
        const int kkey = trow & 15;
        const int vkey = (trow & 3) << 2;
        if (FP8) {
          uintx4 lo, hi;
          fp8x16_to_bf16(kreg[slot][j], lo, hi);
          *(uintx4*)(krow + (((2 * c) ^ kkey) & (kChunks - 1)) * 16) = lo;
          *(uintx4*)(krow + (((2 * c + 1) ^ kkey) & (kChunks - 1)) * 16) = hi;
          fp8x16_to_bf16(vreg[slot][j], lo, hi);
          *(uintx4*)(vrow + (((2 * c) ^ vkey) & (kChunks - 1)) * 16) = lo;
          *(uintx4*)(vrow + (((2 * c + 1) ^ vkey) & (kChunks - 1)) * 16) = hi;
        } else {
          *(uintx4*)(krow + ((c ^ kkey) & (kChunks - 1)) * 16) = kreg[slot][j];
          *(uintx4*)(vrow + ((c ^ vkey) & (kChunks - 1)) * 16) = vreg[slot][j];
        }
      }
    }
    if (FP8 && lane == 0) {
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const int page = ((j * kThreads + wave * 64) / kSrcChunks) / kPageSize;   // page within the block
        if (page < kBlockTokens / kPageSize) {
          kscale_s[buf][page] = ksc_r[slot][j];
          vscale_s[buf][page] = vsc_r[slot][j];
        }
      }
    }
  };

  // Per-lane LDS byte offsets that do not change over the loop: the K row this lane feeds as an A
  // operand for each 16-dim step, and the V row / column pair it addresses in each transposed
  // read.  Everything else (buffer, sub-block, token group) is a compile-time immediate.
  int koff[kKK], voff[kDT];
  {
    const int t = (n32 & 16) + tau(n32 & 15);
#pragma unroll
    for (int kk = 0; kk < kKK; ++kk) koff[kk] = t * kRowBytes + (((kk * 2 + h2) ^ (t & 15)) & (kChunks - 1)) * 16;
    const int j = lane & 15;
    const int tv = h2 * 8 + (j >> 2);
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt)
      voff[dt] = tv * kRowBytes +
                 (((dt * 4 + ((lane >> 4) & 1) * 2 + ((j & 3) >> 1)) ^ ((tv & 3) << 2)) & (kChunks - 1)) * 16 + (j & 1) * 8;
  }

  auto compute = [&](int blk, auto buf_c) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_c)::value;
#pragma unroll
    for (int sub = 0; sub < kBlockTokens / 32; ++sub) {
      const int tok0 = blk * kBlockTokens + sub * 32;
      if (tok0 > wave_max_pos) continue;                 // nothing visible to this wave (uniform)
      // ---- S^T (32 tokens x 32 rows)
      floatx16 s;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < kKK; ++kk) {
        const bf16x8 kop = *(const bf16x8*)(k_lds[buf] + sub * 32 * kRowBytes + koff[kk]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop, qop[kk], s, 0, 0, 0);
      }
      // register i of this lane is token tok0 + (i/8)*16 + h2*8 + (i%8) of row n32.  Scores stay
      // unscaled in s; the scale (and, for FP8, the K scale of the token's page) is folded into the
      // exponent with one fused multiply-add per element: p = 2^(s * sc - m).
      float sc[2];
      sc[0] = FP8 ? a.scale_log2 * kscale_s[buf][sub * 2] : a.scale_log2;
      sc[1] = FP8 ? a.scale_log2 * kscale_s[buf][sub * 2 + 1] : a.scale_log2;
      if (!positive_scale) {                             // rare: scale the scores themselves instead
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] *= sc[i >> 3];
        sc[0] = sc[1] = 1.f;
      }
      if (tok0 + 31 > wave_min_pos) {                    // causal edge or ragged end inside this sub-block
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = tok0 + (i >> 3) * 16 + h2 * 8 + (i & 7);
          if (tok > my_pos) s[i] = -INFINITY;
        }
      }
      // sc > 0 here, so the row maximum can be taken on the unscaled scores of each page
      float m0 = fmaxf(fmaxf(s[0], s[1]), s[2]), m1 = fmaxf(fmaxf(s[8], s[9]), s[10]);
      m0 = fmaxf(fmaxf(m0, s[3]), s[4]); m1 = fmaxf(fmaxf(m1, s[11]), s[12]);
      m0 = fmaxf(fmaxf(m0, s[5]), s[6]); m1 = fmaxf(fmaxf(m1, s[13]), s[14]);
      m0 = fmaxf(m0, s[7]); m1 = fmaxf(m1, s[15]);
      const float mx = xor32_max(fmaxf(m0 * sc[0], m1 * sc[1]));
      // The reference maximum only moves when a row's scores exceed it by more than 2^kSlack: until
      // then p may be as large as 2^kSlack, which float sums and bf16 P hold without loss, and the
      // accumulators are left alone.
      const bool bump = mx > m_run + kSlack;             // also true for the first live block (-inf)
      const float m_new = bump ? mx : m_run;
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;   // rows that see nothing yet
      if (__builtin_amdgcn_ballot_w64(bump)) {
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[dt][i] *= alpha;
        m_run = m_new;
      }
      float psum = 0.f;
      bf16x8 pop[2];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], sc[i >> 3], -m_safe));
        psum += p;
        pop[i >> 3][i & 7] = (__bf16)(FP8 ? p * vscale_s[buf][sub * 2 + (i >> 3)] : p);
      }
      l_run += psum;
      // ---- O^T += V^T P^T
      typedef __attribute__((address_space(3))) shortx4 lds_s4;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int dt = 0; dt < kDT; ++dt) {
          bf16x8 vop;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            const shortx4 raw = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_s4*)(v_lds[buf] + (sub * 32 + ks * 16 + hf * 4) * kRowBytes + voff[dt]));
            const bf16x4 h4 = __builtin_bit_cast(bf16x4, raw);
            vop[hf * 4 + 0] = h4[0]; vop[hf * 4 + 1] = h4[1]; vop[hf * 4 + 2] = h4[2]; vop[hf * 4 + 3] = h4[3];
          }
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop, pop[ks], acc[dt], 0, 0, 0);
        }
      }
    }
  };

  // ---- main loop: block j sits in LDS buffer j & 1; its global loads were issued two iterations
  // before it is consumed and land in register slot j & 1 in between
  constexpr std::integral_constant<int, 0> even{};
  constexpr std::integral_constant<int, 1> odd{};
  // (block indices past the end are clamped: the redundant copy lands in the buffer nobody reads)
  const int last_blk = n_blocks - 1;
  issue(0, even);
  issue(min(1, last_blk), odd);
  commit(0, even);
  __syncthreads();
  for (int blk = 0; blk < n_blocks; blk += 2) {
    issue(min(blk + 2, last_blk), even);
    compute(blk, even);
    commit(min(blk + 1, last_blk), odd);
    __syncthreads();
    if (blk + 1 < n_blocks) {
      issue(min(blk + 3, last_blk), odd);
      compute(blk + 1, odd);
      commit(min(blk + 2, last_blk), even);
      __syncthreads();
    }
  }

  // ---- normalise and store: lane (row n32, half h2) owns dims dt*32 + (i/4)*8 + h2*4 + i%4
  l_run = xor32_add(l_run);
  if (row_ok) {
    const float inv = 1.f / l_run;
    __bf16* orow = (__bf16*)a.out + ((size_t)(a.q_offsets[b] + q0 + tok_in_tile) * a.hq + head) * D;
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(acc[dt][i4 * 4 + e] * inv);
        *(bf16x4*)(orow + dt * 32 + i4 * 8 + h2 * 4) = pk;
      }
    }
  }
}

}  // namespace

hipError_t launch_append_mfma(const AppendArgs& a, int head_dim, bool fp8, int grid, hipStream_t s) {
  if (head_dim == 128 && !fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<128, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128 && fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<128, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && !fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<64, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<64, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rollattn
