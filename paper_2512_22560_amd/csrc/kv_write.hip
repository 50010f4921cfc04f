// KV write: the new tokens' K and V rows go into the paged cache, the step before attention.
//
// One workgroup per (trajectory, page that receives new tokens, pool); the page belongs to that
// trajectory alone, so nothing here needs an atomic.  Pools that store the source type take the
// rows bit for bit, 16 bytes per lane.  FP8 pools keep one float scale per page and pool: the
// workgroup takes the absolute maximum of the page's new rows (all heads), settles the scale
// (fresh page: amax / 448, or 1 for all zeros; partly filled page: the old scale unless amax / 448
// exceeds it, in which case the codes already there are re-quantised to the new scale), then
// encodes the new rows.  Codes are integers decided by float arithmetic, so every product and
// quotient below is one IEEE float32 operation in a fixed order, with the clamp to [-448, 448]
// before the hardware conversion (round to nearest even onto the E4M3 grid).
#include "rollattn_internal.h"

namespace rollattn {

namespace {

typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr float kE4m3Max = 448.f;

__device__ __forceinline__ float clamp448(float x) { return fminf(fmaxf(x, -kE4m3Max), kE4m3Max); }

// eight floats -> eight E4M3 codes
__device__ __forceinline__ uintx2 encode8(const float* x) {
  uintx2 r;
  int w = 0;
  w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(x[0]), clamp448(x[1]), w, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(x[2]), clamp448(x[3]), w, true);
  r[0] = (unsigned int)w;
  w = 0;
  w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(x[4]), clamp448(x[5]), w, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(x[6]), clamp448(x[7]), w, true);
  r[1] = (unsigned int)w;
  return r;
}

__device__ __forceinline__ void bf16x8_to_float(const uintx4 raw, float* x) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = __uint_as_float(raw[i] << 16);
    x[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
  }
}

__device__ __forceinline__ float block_max(float v, float* lds) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = lds[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, lds[w]);
  __syncthreads();
  return r;
}

struct KvWriteArgs {
  const void* k_new;
  const void* v_new;
  const int32_t* q_lens;
  const int32_t* q_offsets;
  void* k_pages;
  void* v_pages;
  const int32_t* page_table;
  const int32_t* ctx_lens;
  float* k_scale;
  float* v_scale;
  int32_t hkv, max_pages;
};

// SRC_BYTES: 4 (float32) or 2 (bf16); FP8: pool holds E4M3 codes, else the source type
template <int D, int SRC_BYTES, bool FP8>
__global__ __launch_bounds__(kThreads) void kv_write_kernel(const KvWriteArgs a) {
  __shared__ float red[kThreads / 64];
  const int b = blockIdx.y;
  const int n = a.q_lens[b];
  const int len = a.ctx_lens[b];
  const int first = len - n;
  const int page_i = first / kPageSize + blockIdx.x;
  if (n <= 0 || page_i * kPageSize >= len) return;
  const int lo = max(first, page_i * kPageSize), hi = min(len, (page_i + 1) * kPageSize);
  const int s0 = lo - page_i * kPageSize, slots = hi - lo;
  const int64_t phys = a.page_table[(size_t)b * a.max_pages + page_i];
  const int hkv = a.hkv;
  constexpr int kElems = 16 / SRC_BYTES;                 // source elements per 16-byte chunk
  constexpr int kChunksPerRow = D / kElems;
  const int chunks = slots * hkv * kChunksPerRow;        // per pool
  const size_t src_row0 = (size_t)(a.q_offsets[b] + lo - first);

  {
    const int pool = blockIdx.z;                          // 0: K, 1: V -- the two pools have nothing in common
    const unsigned char* src = (const unsigned char*)(pool ? a.v_new : a.k_new) + src_row0 * hkv * D * SRC_BYTES;
    unsigned char* pages = (unsigned char*)(pool ? a.v_pages : a.k_pages);
    if constexpr (!FP8) {
      unsigned char* tile = pages + (size_t)phys * hkv * kPageSize * D * SRC_BYTES;
      // four loads in flight per lane before the first store: the copy is all latency otherwise
      constexpr int kBatch = 4;
      for (int c0 = threadIdx.x; c0 < chunks; c0 += kBatch * kThreads) {
        uintx4 v[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const int c = c0 + i * kThreads;
          if (c < chunks) v[i] = *(const uintx4*)(src + (size_t)c * 16);
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
          const int c = c0 + i * kThreads;
          if (c < chunks) {
            const int col = c % kChunksPerRow, rh = c / kChunksPerRow;   // source order: slot, head, chunk
            const int h = rh % hkv, slot = rh / hkv;
            *(uintx4*)(tile + ((size_t)(h * kPageSize + s0 + slot) * D) * SRC_BYTES + col * 16) = v[i];
          }
        }
      }
    } else {
      static_assert(!FP8 || SRC_BYTES == 2, "FP8 pools are written from bf16 rows");
      float* scale = pool ? a.v_scale : a.k_scale;
      unsigned char* tile = pages + (size_t)phys * hkv * kPageSize * D;
      // The rows are needed twice, for the maximum and for the codes: a page's worth (up to kKeep
      // chunks per thread, which covers 8 KV heads at D = 128) stays in registers in between.
      constexpr int kKeep = 8;
      const bool keep = chunks <= kKeep * kThreads;
      uintx4 held[kKeep];
      float amax = 0.f;
      if (keep) {
#pragma unroll
        for (int i = 0; i < kKeep; ++i) {
          const int c = threadIdx.x + i * kThreads;
          held[i] = c < chunks ? *(const uintx4*)(src + (size_t)c * 16) : uintx4{0, 0, 0, 0};
          float x[8];
          bf16x8_to_float(held[i], x);
#pragma unroll
          for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
        }
      } else {
        for (int c = threadIdx.x; c < chunks; c += kThreads) {
          float x[8];
          bf16x8_to_float(*(const uintx4*)(src + (size_t)c * 16), x);
#pragma unroll
          for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(x[i]));
        }
      }
      amax = block_max(amax, red);
      const float need = amax / kE4m3Max;
      float s_new;
      if (s0 == 0) {
        s_new = amax > 0.f ? need : 1.f;
      } else {
        const float s_old = scale[phys];
        s_new = s_old;
        if (need > s_old) {
          s_new = need;
          // the codes already in slots [0, s0): code <- enc(dec(code) * s_old / s_new), eight at a time
          const int old_chunks = hkv * s0 * (D / 8);
          for (int c = threadIdx.x; c < old_chunks; c += kThreads) {
            const int col = c % (D / 8), rh = c / (D / 8);
            const int slot = rh % s0, h = rh / s0;
            uintx2* p = (uintx2*)(tile + (size_t)(h * kPageSize + slot) * D + col * 8);
            const uintx2 w = *p;
            float x[8];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
              const floatx2 f0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false), f1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
              x[4 * i] = f0[0]; x[4 * i + 1] = f0[1]; x[4 * i + 2] = f1[0]; x[4 * i + 3] = f1[1];
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = (x[i] * s_old) / s_new;
            *p = encode8(x);
          }
        }
      }
      // x / s_new for every new element: ten instructions apiece as the compiler expands an IEEE division.
      // All of them share the divisor, so its refined reciprocal is worked out once and each quotient takes
      // the remaining steps of that same expansion (product, two residual corrections, a last fused step) and
      // the sign of the dividend, which a quotient that rounds to zero would otherwise lose: six
      // instructions, and the same correctly rounded result wherever the expansion's operand scaling would
      // have done nothing, i.e. for a divisor of moderate magnitude and every quotient large enough to
      // matter (one below 2^-10 encodes to zero whatever its last bits).  Divisors outside that range take
      // the plain division.
      const bool fast_div = s_new >= 0x1p-100f && s_new <= 0x1p+100f;
      const float r0 = __builtin_amdgcn_rcpf(s_new);
      const float r1 = __builtin_fmaf(__builtin_fmaf(-s_new, r0, 1.f), r0, r0);
      auto emit = [&](int c, const uintx4 raw) {
        const int col = c % kChunksPerRow, rh = c / kChunksPerRow;
        const int h = rh % hkv, slot = rh / hkv;
        float x[8];
        bf16x8_to_float(raw, x);
        if (fast_div) {
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float q0 = x[i] * r1;
            const float q1 = __builtin_fmaf(__builtin_fmaf(-s_new, q0, x[i]), r1, q0);
            x[i] = __builtin_copysignf(__builtin_fmaf(__builtin_fmaf(-s_new, q1, x[i]), r1, q1), x[i]);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = x[i] / s_new;
        }
        *(uintx2*)(tile + (size_t)(h * kPageSize + s0 + slot) * D + col * 8) = encode8(x);
      };
      if (keep) {
#pragma unroll
        for (int i = 0; i < kKeep; ++i) {
          const int c = threadIdx.x + i * kThreads;
          if (c < chunks) emit(c, held[i]);
        }
      } else {
        for (int c = threadIdx.x; c < chunks; c += kThreads) emit(c, *(const uintx4*)(src + (size_t)c * 16));
      }
      __syncthreads();                                   // every read of the old scale is done
      if (threadIdx.x == 0) scale[phys] = s_new;
    }
  }
}

template <int D>
hipError_t launch_d(const KvWriteArgs& a, int src_bytes, bool fp8, dim3 grid, hipStream_t s) {
  if (fp8) {
    hipLaunchKernelGGL((kv_write_kernel<D, 2, true>), grid, dim3(kThreads), 0, s, a);
  } else if (src_bytes == 2) {
    hipLaunchKernelGGL((kv_write_kernel<D, 2, false>), grid, dim3(kThreads), 0, s, a);
  } else {
    hipLaunchKernelGGL((kv_write_kernel<D, 4, false>), grid, dim3(kThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_write(const void* k_new, const void* v_new, const int32_t* q_lens, const int32_t* q_offsets,
                           void* k_pages, void* v_pages, const int32_t* page_table, const int32_t* ctx_lens,
                           float* k_scale, float* v_scale, int32_t batch, int32_t hkv, int32_t max_pages,
                           int32_t max_q_len, int head_dim, int src_bytes, bool fp8, hipStream_t s) {
  KvWriteArgs a{k_new, v_new, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, hkv, max_pages};
  // a run of max_q_len tokens touches at most this many pages, wherever it starts
  const dim3 grid((unsigned)((max_q_len + kPageSize - 1) / kPageSize + 1), (unsigned)batch, 2);
  if (head_dim == 128) return launch_d<128>(a, src_bytes, fp8, grid, s);
  if (head_dim == 64) return launch_d<64>(a, src_bytes, fp8, grid, s);
  return hipErrorInvalidValue;
}

}  // namespace rollattn
