// Decode attention for bf16 queries over bf16 or FP8-E4M3 paged KV (gfx950).
//
// A row is (trajectory, KV head, tile of up to 16 query heads of its group): the heads ride
// along as the 16 columns of an MFMA tile, so K and V are read from HBM exactly once per
// row.  Rows are cut into 32-token blocks (two pages), laid end to end, and every wave of
// the launch is a worker that owns one equal, contiguous run of that block sequence (the
// plan kernel tells it where its run starts).  A wave streams its run without any
// workgroup-level synchronisation: it prefetches blocks from HBM with 16-byte loads into
// registers several blocks ahead, drops each into its private LDS tile, and consumes it with
//   S^T = K Q^T          (tokens x heads, v_mfma_f32_16x16x32_bf16, K rows as A)
//   O^T += V^T P^T       (dims x heads, V read back transposed with ds_read_b64_tr_*)
// A run that covers a whole row writes the row's output itself; a run that starts or ends
// inside a row leaves an un-normalised partial (max, sum, O) for the merge kernel.
// The transposed products keep "head" on the lane axis in both results, so the online
// softmax state (running max, running sum, rescale factor) is one scalar per lane and P
// feeds the second product straight from the first one's accumulator registers.
#include "rollattn_internal.h"

namespace rollattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef int intx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

template <int D, bool FP8>
struct Geo {
  static constexpr int kRowBytes = D * (FP8 ? 1 : 2);
  static constexpr int kChunks = kRowBytes / 16;          // 16-byte chunks per token row
  static constexpr int kRowsPerLoad = 64 / kChunks;        // token rows one wave-wide load covers
  static constexpr int kLoads = kBlockTokens / kRowsPerLoad;  // loads per block, per pool
  static constexpr int kTileBytes = kBlockTokens * kRowBytes; // LDS bytes per block, per pool
  static constexpr int kStages = FP8 ? 4 : 2;              // blocks in flight per wave
  static constexpr int kDT = D / 16;                       // 16-wide output tiles along D
  static constexpr int kKK = D / 32;                       // 32-deep steps of the QK product
  static_assert(kRowsPerLoad <= 16 && 16 % kRowsPerLoad == 0, "a load must stay inside one page");
};

// Swizzle keys: which 16-byte column a logical chunk of token row t lands in.  K rows are
// read 16 rows at a time (rows {0-3, 8-11, 16-19, 24-27} + 4*tile), V rows 4 or 8 at a time.
__device__ __forceinline__ int key_k(int t) { return (t & 3) | (((t >> 3) & 3) << 2); }
__device__ __forceinline__ int key_v16(int t) { return ((t & 3) << 1) | (((t >> 3) & 1) << 3); }
__device__ __forceinline__ int key_v8(int t) { return t & 7; }

__device__ __forceinline__ float xor16_max(float x) {
  uintx2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_max(float x) {
  uintx2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor16_add(float x) {
  uintx2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float xor32_add(float x) {
  uintx2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Eight E4M3 codes to bf16, exactly: the scaled conversion with a scale of one, two codes per instruction.
__device__ __forceinline__ bf16x8 fp8x8_to_bf16(uint32_t lo, uint32_t hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
  const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
  const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
  bf16x8 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
  return r;
}

struct Cursor {
  int b, r, blk;   // trajectory, row within it, block within the row
  int n, len;      // blocks in the row, context length of the trajectory
};

template <int D, bool FP8>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(const DecodeArgs a) {
  using G_ = Geo<D, FP8>;
  // Per wave: one K tile and one V tile.
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWaves][2 * G_::kTileBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r16 = lane & 15;   // MFMA row / column index carried by this lane
  const int q4 = lane >> 4;    // which quarter of the contraction this lane feeds
  unsigned char* const k_lds = lds[wave];
  unsigned char* const v_lds = lds[wave] + G_::kTileBytes;

  const int worker = blockIdx.x * kWaves + wave;
  const int4 start = *(const int4*)(a.wstart + 4 * worker);   // (b, r << 20 | block, L_b, run length)
  if (start.x < 0) return;
  const int n_mine = __builtin_amdgcn_readfirstlane(start.w);
  const int group = a.group, hkv = a.hkv, rows_per_b = a.rows_per_b;
  const int n_ht = rows_per_b / hkv;
  const size_t tile_stride = (size_t)kPageSize * G_::kRowBytes;   // bytes of one (page, head) tile

  Cursor pc;   // producer: next block to request from HBM
  pc.b = __builtin_amdgcn_readfirstlane(start.x);
  pc.r = __builtin_amdgcn_readfirstlane(start.y) >> 20;
  pc.blk = __builtin_amdgcn_readfirstlane(start.y) & 0xFFFFF;
  pc.len = __builtin_amdgcn_readfirstlane(start.z);
  pc.n = (pc.len + kBlockTokens - 1) / kBlockTokens;
  Cursor cc = pc;   // consumer: block being computed
  auto advance = [&](Cursor& c) {
    if (++c.blk < c.n) return;
    c.blk = 0;
    if (++c.r < rows_per_b) return;
    c.r = 0;
    do {
      ++c.b;
      c.len = (!a.q_lens || a.q_lens[c.b] == 1) ? a.ctx_lens[c.b] : 0;   // mixed step: chunk rows are not ours
    } while (c.len == 0);
    c.n = (c.len + kBlockTokens - 1) / kBlockTokens;
  };
  // query / output row of a trajectory: its index, or in a mixed step where its one token sits in the packed rows
  auto row_of = [&](int b) { return (size_t)(a.q_offsets ? a.q_offsets[b] : b); };

  // ---- producer state: a window of 64 page ids (32 blocks) of the current row, one per lane
  int pwin = -1, pid_vec = 0, pid_next = 0;
  int issued = 0;
  uint4 kreg[G_::kStages][G_::kLoads];
  uint4 vreg[G_::kStages][G_::kLoads];
  float ksc[G_::kStages], vsc[G_::kStages];   // FP8: page scales of this lane's 8 tokens
  auto load_window = [&](int k) {
    const int pg = k * 64 + lane;
    return (pg < ((pc.len + kPageSize - 1) >> 4)) ? a.page_table[(size_t)pc.b * a.max_pages + pg] : 0;
  };
  auto issue = [&](int stage) {
    const int k = pc.blk >> 5;
    if (k != pwin) {
      pid_vec = (pwin >= 0 && k == pwin + 1) ? pid_next : load_window(k);
      pid_next = load_window(k + 1);
      pwin = k;
    }
    const int g = pc.r / n_ht;
    const int tok0 = pc.blk * kBlockTokens;
    const int p0 = __builtin_amdgcn_readlane(pid_vec, ((pc.blk & 31) << 1));
    const int p1 = __builtin_amdgcn_readlane(pid_vec, ((pc.blk & 31) << 1) + 1);
    if (FP8) {
      const int pid = (q4 < 2) ? p0 : p1;        // tokens 0-15 of the block sit in its first page
      ksc[stage] = a.k_scale[pid];
      vsc[stage] = a.v_scale[pid];
    }
    const unsigned char* kt0 = (const unsigned char*)a.k_pages + ((size_t)p0 * hkv + g) * tile_stride;
    const unsigned char* kt1 = (const unsigned char*)a.k_pages + ((size_t)p1 * hkv + g) * tile_stride;
    const unsigned char* vt0 = (const unsigned char*)a.v_pages + ((size_t)p0 * hkv + g) * tile_stride;
    const unsigned char* vt1 = (const unsigned char*)a.v_pages + ((size_t)p1 * hkv + g) * tile_stride;
    if (tok0 + kBlockTokens <= pc.len) {
      // whole block live: plain 16-byte loads, 1 KB per wave-wide instruction
#pragma unroll
      for (int j = 0; j < G_::kLoads; ++j) {
        const int row0 = j * G_::kRowsPerLoad;
        const int off = (row0 % kPageSize) * G_::kRowBytes + lane * 16;
        kreg[stage][j] = *(const uint4*)((row0 < kPageSize ? kt0 : kt1) + off);
        vreg[stage][j] = *(const uint4*)((row0 < kPageSize ? vt0 : vt1) + off);
      }
    } else {
      // ragged last block of a row: rows at or past L_b are neither read nor left undefined
#pragma unroll
      for (int j = 0; j < G_::kLoads; ++j) {
        const int row0 = j * G_::kRowsPerLoad;
        const int off = (row0 % kPageSize) * G_::kRowBytes + lane * 16;
        const int row = row0 + lane / G_::kChunks;
        uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (tok0 + row < pc.len) {
          kv = *(const uint4*)((row0 < kPageSize ? kt0 : kt1) + off);
          vv = *(const uint4*)((row0 < kPageSize ? vt0 : vt1) + off);
        }
        kreg[stage][j] = kv;
        vreg[stage][j] = vv;
      }
    }
    // step to the next block of the run (never past its end: the rows after the last block need
    // not exist); a new row starts with a fresh page-id window
    if (++issued < n_mine) {
      const int row_before = pc.b * rows_per_b + pc.r;
      advance(pc);
      if (pc.b * rows_per_b + pc.r != row_before) pwin = -1;
    }
  };
  auto commit = [&](int stage) {
#pragma unroll
    for (int j = 0; j < G_::kLoads; ++j) {
      const int row = j * G_::kRowsPerLoad + lane / G_::kChunks;
      const int c = lane % G_::kChunks;
      const int kc = (c ^ key_k(row)) & (G_::kChunks - 1);
      const int vc = (c ^ (FP8 ? key_v8(row) : key_v16(row))) & (G_::kChunks - 1);
      *(uint4*)(k_lds + row * G_::kRowBytes + kc * 16) = kreg[stage][j];
      *(uint4*)(v_lds + row * G_::kRowBytes + vc * 16) = vreg[stage][j];
    }
  };

  // ---- consumer state
  bf16x8 qop[G_::kKK];       // Q^T as the B operand: lane (head r16, quarter q4), 8 dims per step
  floatx4 acc[G_::kDT];      // O^T: lane (head r16, quarter q4) holds dims dt*16 + q4*4 + (0..3)
  float m_run = -INFINITY;   // running max (log2 units) of this lane's head
  float l_run = 0.f;         // this lane's share of the running sum
  int seg_first_blk = 0;     // block of the row at which the current segment started
  bool first_segment = true;

  auto begin_segment = [&]() {
    const int g = cc.r / n_ht;
    const int h0 = (cc.r - g * n_ht) * kMfmaHeadTile;
    const __bf16* qrow = (const __bf16*)a.q + (row_of(cc.b) * a.hq + (size_t)g * group + h0 + r16) * D;
#pragma unroll
    for (int kk = 0; kk < G_::kKK; ++kk) {
      bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (h0 + r16 < group) {
        if (FP8) {
          // 16-byte K chunks hold 16 dims; step 2p+e uses bytes e*8.. of chunk p*4+q4
          v = *(const bf16x8*)(qrow + ((kk >> 1) * 4 + q4) * 16 + (kk & 1) * 8);
        } else {
          v = *(const bf16x8*)(qrow + (kk * 4 + q4) * 8);
        }
      }
      qop[kk] = v;
    }
#pragma unroll
    for (int dt = 0; dt < G_::kDT; ++dt) acc[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    m_run = -INFINITY;
    l_run = 0.f;
    seg_first_blk = cc.blk;
  };
  auto end_segment = [&]() {
    const int g = cc.r / n_ht;
    const int h0 = (cc.r - g * n_ht) * kMfmaHeadTile;
    const float l_tot = xor32_add(xor16_add(l_run));
    const bool head_ok = h0 + r16 < group;
    if (seg_first_blk == 0 && cc.blk == cc.n - 1) {
      // the whole row was ours: normalise and store
      const float inv = 1.f / l_tot;
      const size_t orow = row_of(cc.b) * a.hq + (size_t)g * group + h0 + r16;
      __bf16* dst = (__bf16*)a.out + orow * D + q4 * 4;
      if (a.lse && head_ok && q4 == 0) a.lse[orow] = m_run + __builtin_amdgcn_logf(l_tot);
      if (head_ok) {
#pragma unroll
        for (int dt = 0; dt < G_::kDT; ++dt) {
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(acc[dt][e] * inv);
          *(bf16x4*)(dst + dt * 16) = pk;
        }
      }
    } else {
      const size_t slot = (size_t)worker * 2 + (first_segment ? 0 : 1);
      if (head_ok) {
        float* dst = a.partial_o + (slot * kMfmaHeadTile + r16) * D + q4 * 4;
#pragma unroll
        for (int dt = 0; dt < G_::kDT; ++dt) *(floatx4*)(dst + dt * 16) = acc[dt];
        if (q4 == 0) {
          a.partial_ml[(slot * kMfmaHeadTile + r16) * 2 + 0] = m_run;
          a.partial_ml[(slot * kMfmaHeadTile + r16) * 2 + 1] = l_tot;
        }
      }
    }
    first_segment = false;
  };
  auto compute = [&](float kscale, float vscale) {
    const int tok0 = cc.blk * kBlockTokens;
    const int len = cc.len;
    // ---- S^T = K Q^T for the two 16-row tiles; tile e row r is token (r/4)*8 + e*4 + r%4
    floatx4 s[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      s[e] = floatx4{0.f, 0.f, 0.f, 0.f};
      const int t = ((r16 >> 2) << 3) + e * 4 + (r16 & 3);
      const unsigned char* rowp = k_lds + t * G_::kRowBytes;
      const int key = key_k(t);
      if (FP8) {
#pragma unroll
        for (int p = 0; p < G_::kChunks / 4; ++p) {
          const int c = ((p * 4 + q4) ^ key) & (G_::kChunks - 1);
          const uint4 raw = *(const uint4*)(rowp + c * 16);
          s[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp8x8_to_bf16(raw.x, raw.y), qop[2 * p], s[e], 0, 0, 0);
          s[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp8x8_to_bf16(raw.z, raw.w), qop[2 * p + 1], s[e], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int kk = 0; kk < G_::kKK; ++kk) {
          const int c = ((kk * 4 + q4) ^ key) & (G_::kChunks - 1);
          const bf16x8 kop = *(const bf16x8*)(rowp + c * 16);
          s[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qop[kk], s[e], 0, 0, 0);
        }
      }
    }
    // This lane now holds, for head r16, the scores of tokens tok0 + q4*8 + (0..7):
    // s[0][i] -> +i, s[1][i] -> +4+i.
    const float sc = FP8 ? a.scale_log2 * kscale : a.scale_log2;
    const float vs = FP8 ? vscale : 1.f;
    float x[8];
    const int tbase = tok0 + q4 * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float raw = (j < 4) ? s[0][j] : s[1][j - 4];
      x[j] = (tbase + j < len) ? raw * sc : -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mx = xor32_max(xor16_max(mx));
    const float m_new = fmaxf(m_run, mx);       // finite: the first token of a block is always live
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
    bf16x8 pop;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float p = __builtin_amdgcn_exp2f(x[j] - m_new);
      psum += p;
      pop[j] = (__bf16)(FP8 ? p * vs : p);
    }
    l_run = l_run * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(m_new > m_run)) {
#pragma unroll
      for (int dt = 0; dt < G_::kDT; ++dt) acc[dt] *= alpha;
    }
    m_run = m_new;
    // ---- O^T += V^T P^T : A = V^T tile (16 dims x 32 tokens) read transposed from LDS
#pragma unroll
    for (int dt = 0; dt < G_::kDT; ++dt) {
      bf16x8 vop;
      if (FP8) {
        typedef __attribute__((address_space(3))) intx2 lds_i2;
        const int t = q4 * 8 + (r16 >> 1);
        const int c = (dt ^ key_v8(t)) & (G_::kChunks - 1);
        const intx2 raw = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
            (lds_i2*)(v_lds + t * G_::kRowBytes + c * 16 + (r16 & 1) * 8));
        vop = fp8x8_to_bf16((uint32_t)raw[0], (uint32_t)raw[1]);
      } else {
        typedef __attribute__((address_space(3))) shortx4 lds_s4;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const int t = q4 * 8 + hf * 4 + (r16 >> 2);
          const int c = ((dt * 2 + ((r16 & 3) >> 1)) ^ key_v16(t)) & (G_::kChunks - 1);
          const shortx4 raw = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s4*)(v_lds + t * G_::kRowBytes + c * 16 + (r16 & 1) * 8));
          const bf16x4 h4 = __builtin_bit_cast(bf16x4, raw);
          vop[hf * 4 + 0] = h4[0]; vop[hf * 4 + 1] = h4[1]; vop[hf * 4 + 2] = h4[2]; vop[hf * 4 + 3] = h4[3];
        }
      }
      acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop, acc[dt], 0, 0, 0);
    }
  };

  // ---- software pipeline over this worker's run of n_mine blocks
#pragma unroll
  for (int st = 0; st < G_::kStages; ++st) {
    if (st < n_mine) issue(st);
  }
  for (int i0 = 0; i0 < n_mine; i0 += G_::kStages) {
#pragma unroll
    for (int st = 0; st < G_::kStages; ++st) {
      const int i = i0 + st;
      if (i < n_mine) {
        commit(st);
        const float kscale = FP8 ? ksc[st] : 1.f, vscale = FP8 ? vsc[st] : 1.f;
        if (i + G_::kStages < n_mine) issue(st);   // the registers just drained take the next block
        if (i == 0 || cc.blk == 0) begin_segment();
        compute(kscale, vscale);
        if (cc.blk == cc.n - 1 || i == n_mine - 1) end_segment();
        if (i + 1 < n_mine) advance(cc);
      }
    }
  }
}

}  // namespace

hipError_t launch_decode_mfma(const DecodeArgs& a, int head_dim, bool fp8, int grid, hipStream_t s) {
  if (head_dim == 128 && !fp8) {
    hipLaunchKernelGGL((decode_mfma_kernel<128, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128 && fp8) {
    hipLaunchKernelGGL((decode_mfma_kernel<128, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && !fp8) {
    hipLaunchKernelGGL((decode_mfma_kernel<64, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && fp8) {
    hipLaunchKernelGGL((decode_mfma_kernel<64, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rollattn
