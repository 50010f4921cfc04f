// Two microbenchmarks that say what this GPU delivers at best, for the fractions the benchmark reports
// next to the nominal peaks: a streaming read of a large buffer (HBM bandwidth) and a register-resident loop
// of the matrix instruction the append kernel uses (bf16 MFMA rate).  Built into a library of its own,
// libbench_peaks.so; nothing of it is part of librollattn.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kReadThreads = 256;
constexpr int kReadUnroll = 8;     // 16-byte loads in flight per thread

// Every thread walks the buffer with a grid stride, kReadUnroll independent 16-byte loads per step.
__global__ __launch_bounds__(kReadThreads) void stream_read_kernel(const uintx4* __restrict__ src, size_t n_vec, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * kReadThreads;
  size_t i = (size_t)blockIdx.x * kReadThreads + threadIdx.x;
  uint32_t acc = 0;
  for (; i + (kReadUnroll - 1) * stride < n_vec; i += kReadUnroll * stride) {
    uintx4 v[kReadUnroll];
#pragma unroll
    for (int u = 0; u < kReadUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < kReadUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n_vec; i += stride) {
    const uintx4 v = __builtin_nontemporal_load(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) *sink = acc;     // practically never: keeps the loads alive
}

constexpr int kMfmaThreads = 512;  // two waves per SIMD
constexpr int kMfmaChains = 4;     // independent accumulators per wave

// Operands and accumulators stay in registers; kMfmaChains independent chains keep the pipe full.
__global__ __launch_bounds__(kMfmaThreads) void mfma_bf16_kernel(int iters, float* sink) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(float)((int)((threadIdx.x * 7 + e * 3) % 13) - 6);
    b[e] = (__bf16)(0.125f * (float)((int)((threadIdx.x * 5 + e) % 11) - 5));
  }
  floatx16 acc[kMfmaChains];
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kMfmaChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  if (s == 12345.678f) *sink = s;
}

}  // namespace

extern "C" {

// Reads `bytes` bytes (a multiple of 16) of device memory `reps` times; *ms_out = average duration of one pass.
// sink: 4 bytes of device memory.  Returns 0, or the HIP error code.
int peaks_stream_read(const void* buf, size_t bytes, int reps, void* sink, float* ms_out, void* hip_stream) {
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) return (int)e;
  const size_t n_vec = bytes / 16;
  const int grid = 256 * 8;
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(kReadThreads), 0, s, (const uintx4*)buf, n_vec, (uint32_t*)sink);   // warm-up
  (void)hipEventRecord(e0, s);
  for (int r = 0; r < reps; ++r)
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(kReadThreads), 0, s, (const uintx4*)buf, n_vec, (uint32_t*)sink);
  (void)hipEventRecord(e1, s);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  *ms_out = ms / (reps > 0 ? reps : 1);
  return (int)hipGetLastError();
}

// Runs iters * 4 MFMAs (32x32x16, bf16) per wave on 256 * 4 * 2 waves; *ms_out = duration, *flops_out = the
// floating-point operations that took.
int peaks_mfma_bf16(int iters, void* sink, float* ms_out, double* flops_out, void* hip_stream) {
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) return (int)e;
  const int grid = 256 * 4;
  hipLaunchKernelGGL(mfma_bf16_kernel, dim3(grid), dim3(kMfmaThreads), 0, s, iters / 8 + 1, (float*)sink);   // warm-up
  (void)hipEventRecord(e0, s);
  hipLaunchKernelGGL(mfma_bf16_kernel, dim3(grid), dim3(kMfmaThreads), 0, s, iters, (float*)sink);
  (void)hipEventRecord(e1, s);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  *ms_out = ms;
  *flops_out = (double)grid * (kMfmaThreads / 64) * (double)iters * kMfmaChains * (2.0 * 32 * 32 * 16);
  return (int)hipGetLastError();
}

}  // extern "C"
