// Observation-append attention (chunked causal prefill on a cached prefix) for bf16 queries
// over bf16 or FP8-E4M3 paged KV, on the gfx950 matrix cores.
//
// One workgroup = 256 query rows of one (trajectory, KV head): a row is a (chunk token, query
// head of the group) pair, token-major, so the G heads that share the KV head reuse every K/V
// tile.  Eight waves of 32 rows each walk the visible KV range in 64-token blocks (four pages)
// that the workgroup stages once in LDS, always as bf16: bf16 pools are copied from HBM into LDS
// directly (no register stop, ring of four tiles per pool), FP8 pools pass through registers to
// be widened (two tiles per pool, loads two blocks ahead of the LDS write).  Per block a wave
// computes
//   S^T = K Q^T        tokens x rows, v_mfma_f32_32x32x16_bf16, K rows as A operand
//   O^T += V^T P^T     dims x rows, V read transposed with ds_read_b64_tr_b16
// The transposed products keep "row" on the lane axis in both accumulators: the softmax
// state is one scalar per lane (shared by two lanes) and P goes from accumulator registers
// straight into the B operand of the second product.
//
// Schedule.  A SIMD holds two of the workgroup's waves (w and w + 4).  Left alone they run in
// step, both in their MFMAs and then both in their softmax, and the matrix and vector pipelines
// take turns.  Here every block is cut into a matrix phase (the second product of the previous
// block, then the first product of this one) and a vector phase (this block's softmax), each
// closed by a workgroup barrier, and waves 4-7 enter the sequence one barrier late: on every SIMD
// one wave feeds the matrix core while the other does the exponentials.  A wave in its matrix
// phase has no partner to hide its latencies, so it reads its LDS operands several steps ahead in
// a fixed source-order schedule and issues as little else as possible: measured with per-phase
// cycle counters, a vector-memory instruction issued between the MFMAs costs the phase 70-90
// cycles (four of them stretched 32 MFMAs from 1270 to 1400 cycles), while the same instruction
// costs the vector phase little more than its issue slot.  All tile loads and the scalar loads of
// page ids and page scales therefore belong to the vector phase; only the widening of FP8 tiles
// (conversions and LDS writes of registers loaded two blocks earlier) stays between the MFMAs,
// where it was measured to cost less than in a vector phase that is bound by its own instruction
// stream.  The vector phase keeps its VALU work short in turn:
//   bf16 pools: the query is multiplied by sm_scale * log2(e) once, when it is loaded (one extra
//     bf16 rounding of q, far below the rounding of P), and the score accumulators start from
//     minus the row's reference instead of zero, so the MFMA result already is the exponent and
//     the softmax is one v_exp_f32 per element with nothing in front of it;
//   FP8 pools: the score needs its page's K scale anyway (one fused multiply-add per element,
//     whose addend carries minus the reference), and the V scale of the page is folded into that
//     addend as log2(vs), so P comes out of the exponential already weighted for the second
//     product; the row sum divides each page's share by vs again (four multiplies per block).
//
// Half tiles.  A call whose chunks all fit into 128 rows gets tiles of 128 rows: waves w and w + 4 then own the
// same 32 rows and split every block, 32 tokens each, and their two running states are merged when the
// tile ends (see the template parameter HALF below).
#include <type_traits>
#include <utility>

#include "rollattn_internal.h"

namespace rollattn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kRowsPerWave = 32;
static_assert(kWaves * kRowsPerWave == kAppendTileRows, "tile rows");
constexpr int kBlockTokens = 64;                   // KV tokens staged per step
constexpr float kSumLimit = 16384.f;               // a lane's 32 probabilities of a block may add up to this much before the row's reference moves

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

// Sixteen E4M3 codes to bf16, exactly (every E4M3 value is a bf16 value): the hardware's scaled
// conversion with a scale of one turns two codes into a packed pair per instruction.
__device__ __forceinline__ void fp8x16_to_bf16(const uintx4 raw, uintx4& lo, uintx4& hi) {
  uint32_t o[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[i], 1.0f, false));
    o[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[i], 1.0f, true));
  }
  lo = uintx4{o[0], o[1], o[2], o[3]};
  hi = uintx4{o[4], o[5], o[6], o[7]};
}

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// HALF: for tiles of at most 128 rows.  With the plain layout such a tile keeps only the leading four waves busy
// and the two pipelines of a SIMD take turns.  Here waves w and w + 4 both own rows 32 (w % 4) .. and split every
// block between them: the leading wave takes its first 32 tokens, the trailing wave the other 32, each with a
// running reference, sum and accumulator of its own, merged through LDS when the tile ends.
template <int D, bool FP8, bool HALF>
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

  // bf16 pools go from HBM straight into LDS (no register stop): a ring of four tiles per pool gives
  // every load a whole block period to land.  FP8 pools pass through registers to be widened: their
  // LDS writes are immediate, two tiles are enough.
  constexpr int kRing = FP8 ? 2 : 4;
  __shared__ __attribute__((aligned(1024))) unsigned char k_lds[kRing][kTileBytes];
  __shared__ __attribute__((aligned(1024))) unsigned char v_lds[kRing][kTileBytes];
  // HALF: where the trailing waves leave their result for the leading ones: per wave pair the accumulators
  // [D / 32][4][64 lanes] as 16-byte quads, and reference and sum.  The accumulators of the four pairs are as large
  // as four bf16 tiles: over bf16 pools they go into the K ring, which nobody reads or loads into any more by
  // then (every wave has waited for its last loads, and the last read of a K tile lies before the trailing
  // waves' last barrier); the two FP8 tiles of the K ring are too small, there the accumulators get LDS of their own.
  constexpr int kMergeAcc = (D / 32) * 16 * 64;      // floats per wave pair
  static_assert(!HALF || FP8 || (size_t)kRing * kTileBytes >= (size_t)(kWaves / 2) * kMergeAcc * sizeof(float), "K ring holds the accumulators");
  __shared__ __attribute__((aligned(16))) float merge_acc_s[HALF && FP8 ? kWaves / 2 : 1][HALF && FP8 ? kMergeAcc : 4];
  __shared__ float merge_ml_s[HALF ? kWaves / 2 : 1][HALF ? 128 : 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31;   // row (B column) / K token row (A row) carried by this lane
  const int h2 = lane >> 5;    // half of the contraction this lane feeds

  const int group = a.group;
  const int hkv = a.hkv;
  const int tile_tokens = a.tile_tokens;
  const int n_tiles = a.header[kPlanTiles];
  // Workgroup -> (tile, KV head).  Workgroups go to the 8 XCDs round-robin and every XCD has an L2 of its
  // own; tiles of one trajectory and KV head walk the same K/V stream and should share one L2.  With the
  // plain order (head fastest) that holds when the head count is a multiple of 8: XCD x then only ever sees
  // heads x, x + 8, ...  With 1, 2 or 4 KV heads a head's tiles would be dealt to 8, 4 or 2 XCDs and each of
  // them would fetch the whole stream; there the 8 / Hkv XCDs that serve a head take turns by runs of
  // kAppendXcdRun consecutive tiles of the list (the list keeps a trajectory's tiles together).
  int tile, g;
  if (hkv < kXcds && kXcds % hkv == 0) {
    const int x = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int parts = kXcds / hkv;
    g = x % hkv;
    tile = (slot / kAppendXcdRun) * (parts * kAppendXcdRun) + (x / hkv) * kAppendXcdRun + slot % kAppendXcdRun;
  } else {
    tile = blockIdx.x / hkv;
    g = blockIdx.x - tile * hkv;
  }
  // The tile's record does not wait for the tile count (the index is clamped to the list's capacity): both loads
  // leave together, and everything else the workgroup needs to start hangs off the record alone.
  typedef const __attribute__((address_space(4))) int32_t* const_rec_p;
  const const_rec_p rec = (const_rec_p)(a.tile_rec + (size_t)min(tile, a.tile_cap - 1) * kTileRecWords);
  const int b = rec[0], q0 = rec[1], n_b = rec[2], ctx = rec[3], q_off = rec[4];
  if (tile >= n_tiles) return;
  __shared__ long clock_s[2];
  if (a.clock_sums && threadIdx.x == 0) {
    clock_s[0] = __builtin_amdgcn_s_memtime();
    clock_s[1] = __builtin_amdgcn_s_memrealtime();
  }
  const int tokens_here = min(tile_tokens, n_b - q0);
  const int rows_here = tokens_here * group;
  // Causal mode: row i of the chunk sits at position L_b - n_b + i and sees tokens up to itself.
  // Non-causal mode (the shared part of a decode step for a group of trajectories): every row sees
  // all of [0, L_b), the rows' own tokens lie outside this range.
  const bool causal = a.noncausal == 0;
  const int pos0 = causal ? ctx - n_b + q0 : ctx - 1;    // position of the tile's first token
  const int kv_end = causal ? pos0 + tokens_here : ctx;  // tokens [0, kv_end) are visible to some row
  const int n_blocks = (kv_end + kBlockTokens - 1) / kBlockTokens;
  // Page ids and page scales are inputs nobody writes during the call: reading them through the
  // constant address space lets every such load (all uniform) take the scalar path.
  typedef const __attribute__((address_space(4))) int32_t* const_i32_p;
  typedef const __attribute__((address_space(4))) float* const_f32_p;
  const const_i32_p table = (const_i32_p)(a.page_table + (size_t)b * a.max_pages);
  const const_f32_p k_scale_c = (const_f32_p)a.k_scale;
  const const_f32_p v_scale_c = (const_f32_p)a.v_scale;
  const size_t tile_stride = (size_t)kPageSize * kSrcRowBytes;

  // ---- this lane's query row
  const int grp = wave >> 2;   // 0: leading half of the workgroup, 1: the half that runs one phase behind (waves w and w + 4 share a SIMD)
  const int row_wave = HALF ? (wave & 3) : wave;         // which 32 rows of the tile this wave owns
  const int sub0 = HALF ? grp : 0;                       // HALF: which 32 tokens of every block
  const int row = row_wave * kRowsPerWave + n32;
  const bool row_ok = row < rows_here;
  const int tok_in_tile = row / group;
  const int head = g * group + (row - tok_in_tile * group);
  const int my_pos = row_ok ? (causal ? pos0 + tok_in_tile : pos0) : -1;   // last visible token of this row
  // blocks that end at or before this position are fully visible to every row of the wave
  const bool wave_active = row_wave * kRowsPerWave < rows_here;
  const int wave_min_pos = wave_active ? (causal ? pos0 + (row_wave * kRowsPerWave) / group : pos0) : -1;

  if (n_blocks <= 0) {                                   // nothing to attend to (non-causal mode with L_b = 0): zero rows
    if (row_ok) {
      __bf16* orow = (__bf16*)a.out + ((size_t)(q_off + q0 + tok_in_tile) * a.hq + head) * D;
#pragma unroll
      for (int d0 = h2 * (D / 2); d0 < (h2 + 1) * (D / 2); d0 += 4) *(bf16x4*)(orow + d0) = bf16x4{0, 0, 0, 0};
      if (a.lse && h2 == 0) a.lse[(size_t)(q_off + q0 + tok_in_tile) * a.hq + head] = -INFINITY;
    }
    return;
  }

  bf16x8 qop[kKK];
  {
    const __bf16* qrow = (const __bf16*)a.q + ((size_t)(q_off + q0 + tok_in_tile) * a.hq + head) * D;
#pragma unroll
    for (int kk = 0; kk < kKK; ++kk) {
      bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (row_ok) v = *(const bf16x8*)(qrow + kk * 16 + h2 * 8);
      qop[kk] = v;                                 // bf16 pools: scaled further down, once the first tiles are on their way
    }
  }

  floatx16 acc[kDT];
#pragma unroll
  for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  floatx16 negm;            // bf16 pools: minus the row's reference in every element, the value the score accumulators start from
#pragma unroll
  for (int i = 0; i < 16; ++i) negm[i] = 0.f;
  const bool positive_scale = a.scale_log2 > 0.f;   // the usual case; FP8 page scales are positive too

  // ---- staging.  Unit u = (K block u + 1, V block u): the two tiles that the matrix phase of
  // block u + 1 reads; block j lives in ring slot j % kRing of its pool.  Per thread and load, the
  // byte offset inside a (page, head) tile never changes: only the page does, and that is a scalar.
  // Every wave stages its share of a unit in its vector phase; branch-free on purpose (loads can
  // then be waited on by count).  Rows at or past L_b (ragged
  // last block, or a block index clamped at the end of the loop) re-read the trajectory's last
  // token instead: finite data that the causal / length mask never lets through.
  const int live_pages = (ctx + kPageSize - 1) / kPageSize;
  const int last_blk = n_blocks - 1;
  const int last_slot = (ctx - 1) % kPageSize;
  constexpr int kPagesPerBlock = kBlockTokens / kPageSize;
  constexpr bool kAllThreadsLoad = kBlockTokens * kSrcChunks >= kThreads;
  // Chunk idx = j * kThreads + tid of a block sits in LDS row idx / kChunks at chunk position
  // (idx % kChunks), holding the row's chunk (position ^ key): key = row & 15 for K, (row & 3) << 2
  // for V.  The register path (FP8) applies the swizzle when it writes LDS; the direct path has to
  // apply it on the global side, because there the LDS position of a lane's chunk is fixed.
  unsigned int goff[kLoads][2], goff_last[kLoads][2];   // [][0]: K, [][1]: V
  int woff[kLoads][2];
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const int idx = j * kThreads + tid;
    const int trow = idx / kSrcChunks;
    const int tslot = trow % kPageSize;               // token slot within its page
    const int c = idx % kSrcChunks;
    const int kkey = trow & 15, vkey = (trow & 3) << 2;
    const int ck = FP8 ? c : ((c ^ kkey) & (kChunks - 1)), cv = FP8 ? c : ((c ^ vkey) & (kChunks - 1));
    goff[j][0] = tslot * kSrcRowBytes + ck * 16;
    goff[j][1] = tslot * kSrcRowBytes + cv * 16;
    goff_last[j][0] = min(tslot, last_slot) * kSrcRowBytes + ck * 16;
    goff_last[j][1] = min(tslot, last_slot) * kSrcRowBytes + cv * 16;
    woff[j][0] = trow * kRowBytes + (((2 * c) ^ kkey) & (kChunks - 1)) * 16;   // FP8 only
    woff[j][1] = trow * kRowBytes + (((2 * c) ^ vkey) & (kChunks - 1)) * 16;
  }
  // The 64 chunks a wave fetches with one instruction lie in one page, so its id is a scalar.
  // fetch_pids: the page ids behind this wave's kLoads loads of one block (block index clamped to
  // the last block, page index to the last live page).
  int pj[kLoads], lim[kLoads];
  const_i32_p table_j[kLoads];
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    pj[j] = ((j * kThreads + wave * 64) / kSrcChunks) / kPageSize;
    lim[j] = live_pages - 1 - pj[j];                  // first page of a block >= lim: the load touches the last live page
    table_j[j] = table + pj[j];
  }
  auto fetch_pids = [&](int blk, int* dst) __attribute__((always_inline)) {
    const int b4 = min(blk, last_blk) * kPagesPerBlock;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) dst[j] = table_j[j][min(b4, lim[j])];
  };
  // byte offset of the (page, KV head) tile in either pool
  auto tile_off_of = [&](int pid) __attribute__((always_inline)) -> size_t {
    return (size_t)(unsigned int)(pid * hkv + g) * tile_stride;
  };
  // one wave-wide 16-byte load of block blk: scalar tile base, per-lane offset
  struct TileAddr { const unsigned char* base; unsigned int off; };
  auto tile_addr = [&](const void* pool, int pool_i, int blk, size_t toff, int j) __attribute__((always_inline)) -> TileAddr {
    const int b4 = min(blk, last_blk) * kPagesPerBlock;
    return TileAddr{(const unsigned char*)pool + toff, (b4 >= lim[j]) ? goff_last[j][pool_i] : goff[j][pool_i]};
  };
  // -- register path (FP8)
  uintx4 kreg[2][kLoads], vreg[2][kLoads];   // two units in flight
  auto issue = [&](int u, const int* pk, const int* pv, auto slot_c) __attribute__((always_inline)) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      if (kAllThreadsLoad || (j * kThreads + tid) / kSrcChunks < kBlockTokens) {
        const TileAddr ka = tile_addr(a.k_pages, 0, u + 1, tile_off_of(pk[j]), j), va = tile_addr(a.v_pages, 1, u, tile_off_of(pv[j]), j);
        kreg[slot][j] = *(const uintx4*)(ka.base + ka.off);
        vreg[slot][j] = *(const uintx4*)(va.base + va.off);
      }
    }
  };
  auto put = [&](unsigned char* tile, int off, const uintx4 raw) __attribute__((always_inline)) {
    // the two 16-byte halves of the widened chunk sit in chunks 2c and 2c + 1: 16 bytes apart after the swizzle
    uintx4 lo, hi;
    fp8x16_to_bf16(raw, lo, hi);
    *(uintx4*)(tile + off) = lo;
    *(uintx4*)(tile + (off ^ 16)) = hi;
  };
  // -- direct path (bf16): HBM -> LDS without a register stop.  Lane l's 16 bytes land at
  // M0 + 16 l.  The compiler does not see these loads as loads: completion is awaited by count
  // below, which is sound only as long as nothing else in the loop uses the vector-memory counter,
  // register spills to scratch memory included (the build checks that this kernel has none).  M0 is
  // a reserved register for this compiler (it refuses it in a clobber list) and is never live
  // across statements in the code it generates, so it is simply overwritten.
  auto dma = [&](const TileAddr& t, unsigned char* lds_dst) __attribute__((always_inline)) {
    const unsigned int m0 = __builtin_amdgcn_readfirstlane((unsigned int)(uintptr_t)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m0), "v"(t.off), "s"(t.base) : "memory");
  };
#define DMA_WAIT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n))

  // FP8: scales of the pages of a block that this wave's tokens lie in (all four; HALF: two), by scalar loads,
  // folded with the softmax scale; the page ids behind them are fetched one vector phase before the scales,
  // the scales one vector phase before use
  constexpr int kPg = HALF ? kPagesPerBlock / 2 : kPagesPerBlock;
  float ksc_cur[kPg], lvs_cur[kPg], ivs_cur[kPg];   // per page: K scale times softmax scale, log2 of the V scale, its reciprocal
  int spid[kPg];
  auto fetch_spids = [&](int blk) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < kPg; ++p)
      spid[p] = FP8 ? table[min(min(blk, last_blk) * kPagesPerBlock + sub0 * kPg + p, live_pages - 1)] : 0;
  };
  auto load_scales = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < kPg; ++p) {
      if (FP8) {
        const float vs = v_scale_c[spid[p]];
        ksc_cur[p] = k_scale_c[spid[p]] * a.scale_log2;
        lvs_cur[p] = __builtin_amdgcn_logf(vs);
        ivs_cur[p] = __builtin_amdgcn_rcpf(vs);
      } else {
        ksc_cur[p] = 1.f;
        lvs_cur[p] = 0.f;
        ivs_cur[p] = 1.f;
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

  constexpr int kSubs = HALF ? 1 : kBlockTokens / 32;   // 32-token sub-blocks of a block that this wave works on
  constexpr int kPvSteps = 8 * kSubs, kSteps = 16 * kSubs;
  const int sub_bytes = sub0 * 32 * kRowBytes;           // HALF: where this wave's tokens start in a K or V tile
  floatx16 s[kSubs];        // scores of the block between its two phases
  bf16x8 pop[kSubs][2];     // its probabilities, as B operands of the second product

  // ---- matrix phase: up to kSteps (32; HALF: 16) MFMA steps, O^T += V^T P^T for the previous block (the
  // first kPvSteps, V buffer at vbo) and S^T = K Q^T for this one (the others, K buffer at kbo).  Every step
  // needs one 32x16 operand from LDS; the reads run kAhead steps in front of the MFMAs that consume them,
  // because during this phase no second wave hides the LDS latency.  The phase has 32 schedule positions
  // spread evenly over its steps; after a step the caller's piece(pos) runs for the positions that belong to
  // it: the FP8 path threads its LDS writes between the MFMAs there.
  constexpr int kAhead = 4;
  // bf16 pools: the operands of the first kAhead steps of a phase that starts with the second product are
  // read at the end of the vector phase before it, in front of the barrier (the V tile they come from was
  // complete one phase earlier), so that the phase does not open with an LDS round trip.
  constexpr bool kEarly = !FP8;
  bf16x8 early[kAhead];
  typedef __attribute__((address_space(3))) shortx4 lds_s4;
  auto read_v_operand = [&](const unsigned char* vbuf, auto t_c, bf16x8& dst) __attribute__((always_inline)) {
    constexpr int t = decltype(t_c)::value;
    constexpr int sub = t >> 3, ks = (t >> 2) & 1, dt = t & 3;
    if constexpr (dt < kDT) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const shortx4 raw = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (lds_s4*)(vbuf + (sub * 32 + ks * 16 + hf * 4) * kRowBytes + voff[dt]));
        const bf16x4 h4 = __builtin_bit_cast(bf16x4, raw);
        dst[hf * 4 + 0] = h4[0]; dst[hf * 4 + 1] = h4[1]; dst[hf * 4 + 2] = h4[2]; dst[hf * 4 + 3] = h4[3];
      }
    }
  };
  auto read_early = [&](int vbo) __attribute__((always_inline)) {
    static_for<kAhead>([&](auto t_c) __attribute__((always_inline)) { read_v_operand(v_lds[0] + vbo + sub_bytes, t_c, early[decltype(t_c)::value]); });
  };
  auto matrix_phase = [&](auto first_c, auto last_c, int kbo, int vbo, auto&& piece) __attribute__((always_inline)) {
    constexpr int T0 = decltype(first_c)::value, T1 = decltype(last_c)::value;
    const unsigned char* kbuf = k_lds[0] + kbo + sub_bytes;    // byte offsets of the ring slots
    const unsigned char* vbuf = v_lds[0] + vbo + sub_bytes;
    bf16x8 ops[kSteps];
    auto fetch = [&](auto t_c) __attribute__((always_inline)) {
      constexpr int t = decltype(t_c)::value;
      if constexpr (t < kPvSteps) {
        read_v_operand(vbuf, t_c, ops[t]);
      } else {
        constexpr int u = t - kPvSteps, kk = u / kSubs, sub = u % kSubs;
        if constexpr (kk < kKK) ops[t] = *(const bf16x8*)(kbuf + sub * 32 * kRowBytes + koff[kk]);
      }
    };
    auto fire = [&](auto t_c) __attribute__((always_inline)) {
      constexpr int t = decltype(t_c)::value;
      if constexpr (t < kPvSteps) {
        constexpr int sub = t >> 3, ks = (t >> 2) & 1, dt = t & 3;
        if constexpr (dt < kDT) acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ops[t], pop[sub][ks], acc[dt], 0, 0, 0);
      } else {
        constexpr int u = t - kPvSteps, kk = u / kSubs, sub = u % kSubs;
        if constexpr (kk < kKK) {
          if constexpr (kk == 0) {
            if constexpr (FP8) {
#pragma unroll
              for (int i = 0; i < 16; ++i) s[sub][i] = 0.f;
              s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ops[t], qop[kk], s[sub], 0, 0, 0);
            } else {
              s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ops[t], qop[kk], negm, 0, 0, 0);
            }
          } else {
            s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ops[t], qop[kk], s[sub], 0, 0, 0);
          }
        }
      }
    };
    static_for<kAhead>([&](auto d_c) __attribute__((always_inline)) {
      constexpr int t = T0 + decltype(d_c)::value;
      if constexpr (kEarly && T0 == 0) ops[t] = early[t];
      else if constexpr (t < T1) fetch(std::integral_constant<int, t>{});
    });
    __builtin_amdgcn_sched_barrier(0);
    static_for<kSteps>([&](auto t_c) __attribute__((always_inline)) {
      constexpr int t = decltype(t_c)::value;
      if constexpr (t >= T0 && t < T1) {
        if constexpr (t + kAhead < T1) fetch(std::integral_constant<int, t + kAhead>{});
        fire(t_c);
        constexpr int P0 = (t - T0) * 32 / (T1 - T0), P1 = (t + 1 - T0) * 32 / (T1 - T0);
        static_for<P1 - P0>([&](auto d_c) __attribute__((always_inline)) { piece(std::integral_constant<int, P0 + decltype(d_c)::value>{}); });
        __builtin_amdgcn_sched_barrier(0);           // the source order of the steps is the schedule
      }
    });
  };
  constexpr std::integral_constant<int, 0> c0{};
  // ---- vector phase: online softmax of block blk.  Register i of s[sub] is token
  // blk*64 + sub*32 + (i/8)*16 + h2*8 + (i%8) of row n32.
  //   bf16 pools: s already is the exponent (scaled query, accumulators started from minus the reference).
  //   FP8 pools:  s is the raw product with the codes; per page sc = K scale times the softmax scale and
  //               ad = log2(V scale) - reference, so p' = 2^(s * sc + ad) = p * vs is the weight the second
  //               product needs, and the row sum takes each page's share divided by vs again.
  // The reference m_run of a row only moves when it has to.  The exponentials are taken against the
  // reference as it stands, without looking for the block's maximum first, and may exceed one: float
  // sums and bf16 P hold large values with the same relative precision as small ones.  Only when the p
  // of one lane add up to more than kSumLimit (so that no single p ever exceeds it), or when a row has no
  // reference yet, does the wave find the true maxima, move the references there, rescale the
  // accumulators and redo the block's exponentials.  In all other blocks the maximum, a chain of
  // dependent steps across the row, is never computed.
  static_assert(kPg == 2 * kSubs, "two pages per 32-token sub-block");
  auto softmax = [&](int blk) __attribute__((always_inline)) {
    float sc[kPg], lvs[kPg], ivs[kPg];                 // this wave's pages: K scale times softmax scale, log2 of the V scale, its reciprocal
    if constexpr (FP8) {
#pragma unroll
      for (int p = 0; p < kPg; ++p) { sc[p] = ksc_cur[p]; lvs[p] = lvs_cur[p]; ivs[p] = ivs_cur[p]; }
      if (!positive_scale) {                           // rare: scale the scores themselves instead
#pragma unroll
        for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[sub][i] *= sc[sub * 2 + (i >> 3)];
#pragma unroll
        for (int p = 0; p < kPg; ++p) sc[p] = 1.f;
      }
    }
    const int tok0 = blk * kBlockTokens + sub0 * 32;     // first token of this wave's share of the block
    if (tok0 + kSubs * 32 - 1 > wave_min_pos) {        // causal edge or ragged end inside this block
#pragma unroll
      for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = tok0 + sub * 32 + (i >> 3) * 16 + h2 * 8 + (i & 7);
          if (tok > my_pos) s[sub][i] = -INFINITY;
        }
    }
    const float m_old = (m_run == -INFINITY) ? 0.f : m_run;   // what the exponents in s (bf16 pools) are relative to
    float p[kSubs][16];
    // exponentials of the block against reference m_old + shift, and this lane's share of the row sums
    auto exponentials = [&](auto first_c, float shift) __attribute__((always_inline)) -> float {
      float ad[kPg], psum[kPg];
      if constexpr (FP8) {
#pragma unroll
        for (int pg = 0; pg < kPg; ++pg) ad[pg] = lvs[pg] - (m_old + shift);
      }
#pragma unroll
      for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int pg = sub * 2 + (i >> 3);
          float x;
          if constexpr (FP8) x = __builtin_fmaf(s[sub][i], sc[pg], ad[pg]);
          else if constexpr (decltype(first_c)::value) x = s[sub][i];
          else x = s[sub][i] - shift;
          p[sub][i] = __builtin_amdgcn_exp2f(x);
          if ((i & 7) == 0) psum[pg] = p[sub][i];
          else psum[pg] += p[sub][i];
        }
      if constexpr (HALF) return FP8 ? psum[0] * ivs[0] + psum[1] * ivs[1] : psum[0] + psum[1];
      else if constexpr (FP8) return (psum[0] * ivs[0] + psum[1] * ivs[1]) + (psum[2] * ivs[2] + psum[3] * ivs[3]);
      else return (psum[0] + psum[1]) + (psum[2] + psum[3]);
    };
    float lane_sum = exponentials(std::true_type{}, 0.f);
    // (an infinite or undefined sum also fails the comparison and takes the slow path)
    const bool bump = row_ok && (m_run == -INFINITY || !(lane_sum <= kSumLimit));
    if (__builtin_amdgcn_ballot_w64(bump)) {
      // largest exponent of the block: FP8 page scales and the softmax scale are positive here, so the maximum
      // can be taken on the raw products of each page
      float pm[kPg];
#pragma unroll
      for (int q = 0; q < kPg; ++q) {
        const int sub = q >> 1, o = (q & 1) * 8;
        float x = fmaxf(fmaxf(s[sub][o], s[sub][o + 1]), s[sub][o + 2]);
        x = fmaxf(fmaxf(x, s[sub][o + 3]), s[sub][o + 4]);
        x = fmaxf(fmaxf(x, s[sub][o + 5]), s[sub][o + 6]);
        pm[q] = fmaxf(x, s[sub][o + 7]);
      }
      float mloc;
      if constexpr (HALF) mloc = FP8 ? fmaxf(pm[0] * sc[0], pm[1] * sc[1]) : fmaxf(pm[0], pm[1]) + m_old;
      else if constexpr (FP8) mloc = fmaxf(fmaxf(pm[0] * sc[0], pm[1] * sc[1]), fmaxf(pm[2] * sc[2], pm[3] * sc[3]));
      else mloc = fmaxf(fmaxf(pm[0], pm[1]), fmaxf(pm[2], pm[3])) + m_old;
      const float m_new = fmaxf(m_run, xor32_max(mloc));           // the same in both lanes of a row
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;     // rows that see nothing yet
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] *= alpha;
      m_run = m_new;
      if constexpr (!FP8) {
#pragma unroll
        for (int i = 0; i < 16; ++i) negm[i] = -m_safe;
      }
      lane_sum = exponentials(std::false_type{}, m_safe - m_old);
    }
    l_run += lane_sum;
#pragma unroll
    for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) pop[sub][i >> 3][i & 7] = (__bf16)p[sub][i];
    // the probabilities are finished here, in this phase, not wherever the compiler would like to sink them
#pragma unroll
    for (int sub = 0; sub < kSubs; ++sub)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        uintx4 t = __builtin_bit_cast(uintx4, pop[sub][ks]);
        asm volatile("" : "+v"(t));
        pop[sub][ks] = __builtin_bit_cast(bf16x8, t);
      }
  };

  // Two phases per block, a matrix phase (O += V P of the previous block, then S = K Q^T of this
  // one: MFMAs and their LDS operand reads, nothing else) and a vector phase (softmax of this block and
  // the wave's share of the staging), each closed by a workgroup barrier.  The trailing half of the
  // waves entered the sequence one barrier late, so on every SIMD one wave is in its matrix phase
  // while the other is in its vector phase and the two pipelines run side by side instead of taking
  // turns.  Phases are numbered by barriers: the leading half has its matrix phase of block i in phase
  // 2i and its vector phase in 2i + 1, the trailing half in 2i + 1 and 2i + 2.  K block i and V block
  // i - 1 are read in phases 2i and 2i + 1 and their ring slots are free from phase 2i + 2 on.
  //   bf16: in its vector phase of block i a wave starts the loads of unit i + 2 (K block i + 3 into
  //         the slot K block i - 1 left in phase 2i - 1 at the latest, V block i + 2 into the slot of
  //         V block i - 2) and then waits until all but those newest loads have landed: unit i + 1,
  //         a whole block period after it was started, and two barriers before phase 2i + 4 reads it.
  //   FP8:  in its matrix phase of block i (phase 2i or 2i + 1) a wave widens its share of unit i
  //         (K block i + 1, V block i; first read in phase 2i + 2) from registers into the tiles that
  //         are not being read, and in the vector phase that follows it reloads those registers
  //         with unit i + 2.
  // FP8: the wave's LDS writes must be complete before the barrier, but its tile loads for later units
  // must stay in flight across it (a full fence would wait for them too).  bf16: a bare barrier; the
  // direct loads are awaited by count where they are issued.
#define BARRIER_RAW() do { if (FP8) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); else asm volatile("s_barrier" ::: "memory"); } while (0)
#define PHASE_END() do { __builtin_amdgcn_sched_barrier(0); BARRIER_RAW(); __builtin_amdgcn_sched_barrier(0); } while (0)
  constexpr std::integral_constant<int, 0> even{};
  constexpr std::integral_constant<int, 1> odd{};
  constexpr std::integral_constant<int, kPvSteps> c_pv{};   // first step of the first product
  constexpr std::integral_constant<int, kSteps> c_end{};     // end of the phase
  // Page ids run ahead of the tile loads, so that no load ever waits for an address: U = i + kLead being
  // the unit whose loads a wave starts in its vector phase of block i, toff holds (on entry to that
  // phase) the tile offsets of block U and pid_new the page ids of block U + 1.
  constexpr int kLead = 2;
  size_t toff[2][kLoads];      // rotated at the start of the staging step: then [0] is K block U + 1, [1] V block U
  int pid_new[kLoads];         // not yet turned into an offset
  // ko[d]: byte offset of the ring slot of block i + d (i = the block whose matrix phase came
  // last); block i - 1 shares the slot of block i + kRing - 1.
  int ko[kRing];
#pragma unroll
  for (int d = 0; d < kRing; ++d) ko[d] = d * kTileBytes;
  unsigned int kraw[kPg], vraw[kPg];
  {
    int h0[kLoads], h1[kLoads], h2[kLoads], h3[kLoads];
    fetch_pids(0, h0); fetch_pids(1, h1); fetch_pids(2, h2); fetch_pids(3, h3);
    fetch_spids(0);
    load_scales();
    fetch_spids(1);
    if constexpr (FP8) {
      // K block 0 goes to LDS here; units 0 and 1 wait in registers
      uintx4 k0[kLoads];
#pragma unroll
      for (int j = 0; j < kLoads; ++j)
        if (kAllThreadsLoad || (j * kThreads + tid) / kSrcChunks < kBlockTokens) {
          const TileAddr ka = tile_addr(a.k_pages, 0, 0, tile_off_of(h0[j]), j);
          k0[j] = *(const uintx4*)(ka.base + ka.off);
        }
      issue(0, h1, h0, even);
      issue(1, h2, h1, odd);
#pragma unroll
      for (int j = 0; j < kLoads; ++j)
        if (kAllThreadsLoad || (j * kThreads + tid) / kSrcChunks < kBlockTokens) put(k_lds[0], woff[j][0], k0[j]);
    } else {
      const int* hh[4] = {h0, h1, h2, h3};
#pragma unroll
      for (int j = 0; j < kLoads; ++j)
        dma(tile_addr(a.k_pages, 0, 0, tile_off_of(h0[j]), j), k_lds[0] + wave * 1024 + j * kThreads * 16);
#pragma unroll
      for (int u0 = 0; u0 < kLead; ++u0)             // units 0 .. kLead - 1
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
          dma(tile_addr(a.k_pages, 0, u0 + 1, tile_off_of(hh[u0 + 1][j]), j), k_lds[0] + (u0 + 1) * kTileBytes + wave * 1024 + j * kThreads * 16);
          dma(tile_addr(a.v_pages, 1, u0, tile_off_of(hh[u0][j]), j), v_lds[0] + u0 * kTileBytes + wave * 1024 + j * kThreads * 16);
        }
      // the query rows have been under way since the top of the kernel; their scaling (bf16 pools: the
      // scores then leave the matrix core as exponents) waits for them here, behind the tile loads
#pragma unroll
      for (int kk = 0; kk < kKK; ++kk)
#pragma unroll
        for (int e = 0; e < 8; ++e) qop[kk][e] = (__bf16)((float)qop[kk][e] * a.scale_log2);
      DMA_WAIT((kLead - 1) * 2 * kLoads);            // K block 0 and unit 0 have landed (unit 0 is read early, one barrier from now)
    }
    PHASE_END();
    if (grp == 1) {                                  // the trailing half starts one phase late
      PHASE_END();
    }
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      pid_new[j] = h3[j];
      toff[0][j] = tile_off_of(h2[j]);
    }
  }
  // Staging.  The tile addresses of the unit whose loads start in this vector phase:
  auto stage_addresses = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < kLoads; ++j) { toff[1][j] = toff[0][j]; toff[0][j] = tile_off_of(pid_new[j]); }
  };
  // ... those loads, in the vector phase of block i (slot: the register slot that the matrix phase of block
  // i has just drained, FP8 only) ...
  auto stage_loads = [&](int i, auto slot_c) __attribute__((always_inline)) {
    const int u = i + kLead;
    if constexpr (FP8) {
      constexpr int slot = decltype(slot_c)::value;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        // (units past the tile's last block are not loaded: what the registers then hold is widened into tiles nobody reads)
        if (u <= last_blk && (kAllThreadsLoad || (j * kThreads + tid) / kSrcChunks < kBlockTokens)) {
          const TileAddr ka = tile_addr(a.k_pages, 0, u + 1, toff[0][j], j), va = tile_addr(a.v_pages, 1, u, toff[1][j], j);
          kreg[slot][j] = *(const uintx4*)(ka.base + ka.off);
          vreg[slot][j] = *(const uintx4*)(va.base + va.off);
        }
      }
    } else if (u <= last_blk) {
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        dma(tile_addr(a.k_pages, 0, u + 1, toff[0][j], j), k_lds[0] + ko[kRing - 1] + wave * 1024 + j * kThreads * 16);
        dma(tile_addr(a.v_pages, 1, u, toff[1][j], j), v_lds[0] + ko[kRing - 2] + wave * 1024 + j * kThreads * 16);
      }
      DMA_WAIT(2 * kLoads);                          // everything but the unit just started has landed
    } else {
      DMA_WAIT(0);                                   // past the tile's last block nothing is started: the units still on their way are real ones
    }
  };
  // ... and, FP8 only, the widening of unit i (K block i + 1, V block i) from registers into LDS during the
  // matrix phase of block i, at two fixed places between its MFMAs.
  auto stage_widen = [&](auto slot_c, auto pos_c) __attribute__((always_inline)) {
    if constexpr (FP8) {
      constexpr int slot = decltype(slot_c)::value, pos = decltype(pos_c)::value;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const bool mine = kAllThreadsLoad || (j * kThreads + tid) / kSrcChunks < kBlockTokens;
        if (pos == 2 + 12 * j / kLoads && mine) put(k_lds[0] + ko[1], woff[j][0], kreg[slot][j]);
        if (pos == 6 + 12 * j / kLoads && mine) put(v_lds[0] + ko[0], woff[j][1], vreg[slot][j]);
      }
    }
  };
  // Scalar loads (page ids of the unit started two vector phases from now, FP8 page scales of the next
  // block) go out before the softmax and are awaited after it.
  auto scalar_issue = [&](int i) __attribute__((always_inline)) {
    fetch_pids(i + kLead + 2, pid_new);
    if constexpr (FP8) {
      // scales of block i + 1: all loads in one statement, so that each keeps a register of its
      // own (the compiler would recycle one register and wait after every load)
      if constexpr (HALF)
        asm volatile(
            "s_load_dword %0, %4, %6\n\ts_load_dword %1, %4, %7\n\ts_load_dword %2, %5, %6\n\ts_load_dword %3, %5, %7"
            : "=&s"(kraw[0]), "=&s"(kraw[1]), "=&s"(vraw[0]), "=&s"(vraw[1])
            : "s"(a.k_scale), "s"(a.v_scale), "s"((unsigned)spid[0] * 4u), "s"((unsigned)spid[1] * 4u));
      else
      asm volatile(
          "s_load_dword %0, %8, %10\n\ts_load_dword %1, %8, %11\n\ts_load_dword %2, %8, %12\n\ts_load_dword %3, %8, %13\n\t"
          "s_load_dword %4, %9, %10\n\ts_load_dword %5, %9, %11\n\ts_load_dword %6, %9, %12\n\ts_load_dword %7, %9, %13"
          : "=&s"(kraw[0]), "=&s"(kraw[1]), "=&s"(kraw[2 % kPg]), "=&s"(kraw[3 % kPg]), "=&s"(vraw[0]), "=&s"(vraw[1]), "=&s"(vraw[2 % kPg]), "=&s"(vraw[3 % kPg])
          : "s"(a.k_scale), "s"(a.v_scale), "s"((unsigned)spid[0] * 4u), "s"((unsigned)spid[1] * 4u), "s"((unsigned)spid[2 % kPg] * 4u),
            "s"((unsigned)spid[3 % kPg] * 4u));
      fetch_spids(i + 2);
    }
  };
  auto scalar_await = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < kLoads; ++j) { pid_new[j] = __builtin_amdgcn_readfirstlane(pid_new[j]); asm volatile("" : "+s"(pid_new[j])); }   // arrived here, not wherever it is used next
    if constexpr (FP8) {
      if constexpr (HALF)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(kraw[0]), "+s"(kraw[1]), "+s"(vraw[0]), "+s"(vraw[1]));
      else
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+s"(kraw[0]), "+s"(kraw[1]), "+s"(kraw[2 % kPg]), "+s"(kraw[3 % kPg]), "+s"(vraw[0]), "+s"(vraw[1]), "+s"(vraw[2 % kPg]), "+s"(vraw[3 % kPg]));
#pragma unroll
      for (int p = 0; p < kPg; ++p) {
        spid[p] = __builtin_amdgcn_readfirstlane(spid[p]);
        asm volatile("" : "+s"(spid[p]));
        ksc_cur[p] = __uint_as_float(kraw[p]) * a.scale_log2;   // the softmax of this block is done with the old ones
        lvs_cur[p] = __builtin_amdgcn_logf(__uint_as_float(vraw[p]));
        ivs_cur[p] = __builtin_amdgcn_rcpf(__uint_as_float(vraw[p]));
      }
    }
  };
  auto next_block = [&]() __attribute__((always_inline)) {
    const int t = ko[0];
#pragma unroll
    for (int d = 0; d + 1 < kRing; ++d) ko[d] = ko[d + 1];
    ko[kRing - 1] = t;
  };
  // A wave whose 32 rows all lie past the tile's last row (ragged last tile of a chunk, or a group
  // call with few rows) keeps its share of the staging and every barrier but skips the products and
  // the softmax: it would only compete with the wave it shares a SIMD with.
  auto run = [&](auto active_c) __attribute__((always_inline)) {
    constexpr bool kActive = decltype(active_c)::value;
    // slot: parity of the block, the register slot of the unit that is widened and reloaded (FP8)
    auto matrix = [&](auto first_c, auto last_c, auto slot_c) __attribute__((always_inline)) {
      auto piece = [&](auto pos_c) __attribute__((always_inline)) { stage_widen(slot_c, pos_c); };
      if constexpr (kActive) {
        __builtin_amdgcn_s_setprio(1);
        matrix_phase(first_c, last_c, ko[0], ko[kRing - 1], piece);
        __builtin_amdgcn_s_setprio(0);
      } else {
        static_for<32>(piece);
      }
      PHASE_END();
    };
    auto vector = [&](int i, auto slot_c) __attribute__((always_inline)) {
      stage_addresses();
      stage_loads(i, slot_c);
      scalar_issue(i);
      if constexpr (kActive) softmax(i);
      scalar_await();
      if constexpr (kEarly && kActive) read_early(ko[0]);   // V block i, for the matrix phase that follows
      PHASE_END();
      next_block();
    };
    matrix(c_pv, c_end, even);                          // block 0 has no predecessor: scores only
    vector(0, even);
    for (int i = 1; i < n_blocks; i += 2) {
      matrix(c0, c_end, odd);
      vector(i, odd);
      if (i + 1 < n_blocks) {
        matrix(c0, c_end, even);
        vector(i + 1, even);
      }
    }
    if constexpr (kActive) {
      __builtin_amdgcn_s_setprio(1);
      matrix_phase(c0, c_pv, 0, ko[kRing - 1], [](auto) {});
      __builtin_amdgcn_s_setprio(0);
    }
  };
  if (wave_active) run(std::true_type{}); else run(std::false_type{});
  float* const mine = !HALF ? nullptr : FP8 ? merge_acc_s[FP8 ? (wave & 3) : 0] : (float*)&k_lds[0][0] + (wave & 3) * kMergeAcc;
  float* const mine_ml = merge_ml_s[HALF ? (wave & 3) : 0];
  if constexpr (HALF) {
    // The trailing wave of a pair hands over its half of the tile: accumulators, reference and (per-lane) sum.
    if (grp == 1 && wave_active) {
#pragma unroll
      for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *(floatx4*)(mine + ((dt * 4 + i4) * 64 + lane) * 4) = floatx4{acc[dt][i4 * 4], acc[dt][i4 * 4 + 1], acc[dt][i4 * 4 + 2], acc[dt][i4 * 4 + 3]};
      mine_ml[lane] = m_run;
      mine_ml[64 + lane] = l_run;
    }
  }
  if (grp == 0) PHASE_END();
  if constexpr (!FP8) DMA_WAIT(0);                   // nothing may still be landing in LDS when the workgroup retires
  if constexpr (HALF) {
    __syncthreads();                                   // the trailing waves' results are in LDS
    if (grp == 1) return;
    if (wave_active) {
      const float* theirs = mine;
      const float m2 = mine_ml[lane], l2 = mine_ml[64 + lane];
      const float m_new = fmaxf(m_run, m2);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float a1 = __builtin_amdgcn_exp2f(m_run - m_safe), a2 = __builtin_amdgcn_exp2f(m2 - m_safe);
      l_run = l_run * a1 + l2 * a2;
      m_run = m_new;
#pragma unroll
      for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const floatx4 o = *(const floatx4*)(theirs + ((dt * 4 + i4) * 64 + lane) * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[dt][i4 * 4 + e] = acc[dt][i4 * 4 + e] * a1 + o[e] * a2;
        }
    }
  }
#undef PHASE_END
#undef BARRIER_RAW
#undef DMA_WAIT

  // ---- normalise and store: lane (row n32, half h2) owns dims dt*32 + (i/4)*8 + h2*4 + i%4, four dims at a
  // time.  The two lanes of a row first trade every other group of four, so that each holds runs of eight dims
  // and stores 16 bytes at a time: half as many store instructions, each of which touches 32 rows.
  l_run = xor32_add(l_run);
  const float inv = 1.f / l_run;
  // log2 of the row's softmax denominator, for callers that merge this result with another range's
  if (row_ok && a.lse && h2 == 0) a.lse[(size_t)(q_off + q0 + tok_in_tile) * a.hq + head] = m_run + __builtin_amdgcn_logf(l_run);
  __bf16* orow = (__bf16*)a.out + ((size_t)(q_off + q0 + tok_in_tile) * a.hq + head) * D;
#pragma unroll
  for (int dt = 0; dt < kDT; ++dt) {
    uintx2 g[4];
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      bf16x4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(acc[dt][i4 * 4 + e] * inv);
      g[i4] = __builtin_bit_cast(uintx2, pk);
    }
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      // h2 = 0 keeps its group 2 pr (dims 8 pr .. + 3 of the 16) and gets the other lane's; h2 = 1 gets this lane's group
      // 2 pr + 1 and keeps its own: lower lane dims 16 pr + 0 .. 7, upper lane dims 16 pr + 8 .. 15
      const uintx2 w0 = __builtin_amdgcn_permlane32_swap(g[2 * pr][0], g[2 * pr + 1][0], false, false);
      const uintx2 w1 = __builtin_amdgcn_permlane32_swap(g[2 * pr][1], g[2 * pr + 1][1], false, false);
      if (row_ok) *(uintx4*)(orow + dt * 32 + pr * 16 + h2 * 8) = uintx4{w0[0], w1[0], w0[1], w1[1]};
    }
  }
  if (a.clock_sums && threadIdx.x == 0) {
    atomicAdd(a.clock_sums, (unsigned long long)(__builtin_amdgcn_s_memtime() - clock_s[0]));
    atomicAdd(a.clock_sums + 1, (unsigned long long)(__builtin_amdgcn_s_memrealtime() - clock_s[1]));
  }
}

}  // namespace

hipError_t launch_append_mfma(const AppendArgs& a, int head_dim, bool fp8, bool half_tiles, int grid, hipStream_t s) {
  if (head_dim == 128 && !fp8 && !half_tiles) {
    hipLaunchKernelGGL((append_mfma_kernel<128, false, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128 && !fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<128, false, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128 && fp8 && !half_tiles) {
    hipLaunchKernelGGL((append_mfma_kernel<128, true, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 128 && fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<128, true, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && !fp8 && !half_tiles) {
    hipLaunchKernelGGL((append_mfma_kernel<64, false, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && !fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<64, false, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && fp8 && !half_tiles) {
    hipLaunchKernelGGL((append_mfma_kernel<64, true, false>), dim3(grid), dim3(kThreads), 0, s, a);
  } else if (head_dim == 64 && fp8) {
    hipLaunchKernelGGL((append_mfma_kernel<64, true, true>), dim3(grid), dim3(kThreads), 0, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace rollattn
