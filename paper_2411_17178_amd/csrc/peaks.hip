// Diagnostics: what this GPU actually delivers, to put next to the published peaks in
// benchmark reports -- a streaming copy (HBM read + write) and a register-only bf16 MFMA loop.
#include "attn_bf16_common.h"

namespace lv {
namespace {

__global__ __launch_bounds__(256) void k_peak_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void k_peak_read(const uint4* __restrict__ src, unsigned* out, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 7 * stride < n; i += 8 * stride) {       // eight loads in flight per thread
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n; i += stride) acc += src[i].x;
  if (acc == 0x12345679u) out[0] = acc;               // practically never: keeps the loads alive
}

// eight independent accumulator tiles per wave, so that the matrix pipe never waits for a result
__global__ __launch_bounds__(256) void k_peak_mfma(int iters, float* out) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)(threadIdx.x & 3); b[e] = (__bf16)1.0f; }
  f32x4 acc[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 8; ++t)   // in place: the builtin form makes the compiler rotate the tiles through copies
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[t]) : "v"(a), "v"(b));
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // inline-assembly results are invisible to the hazard recogniser
  float s = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t) s += acc[t][0] + acc[t][1] + acc[t][2] + acc[t][3];
  if (s == -1.f) out[0] = s;      // never true: keeps the loop alive
}

}  // namespace
}  // namespace lv

using namespace lv;

extern "C" {

litevar_status litevar_peak_copy(const void* d_src, void* d_dst, size_t bytes, void* stream) {
  if (!d_src || !d_dst) return fail(LITEVAR_E_INVALID_ARG, "d_src or d_dst is NULL");
  if (((uintptr_t)d_src | (uintptr_t)d_dst | bytes) & 15) return fail(LITEVAR_E_INVALID_ARG, "pointers and size must be multiples of 16");
  if (bytes == 0) return LITEVAR_OK;
  hipLaunchKernelGGL(k_peak_copy, dim3(65536), dim3(256), 0, (hipStream_t)stream, (const uint4*)d_src, (uint4*)d_dst, bytes / 16);
  return hip_check(hipGetLastError(), "copy probe launch");
}

litevar_status litevar_peak_read(const void* d_src, size_t bytes, void* d_out, void* stream) {
  if (!d_src || !d_out) return fail(LITEVAR_E_INVALID_ARG, "d_src or d_out is NULL");
  if (((uintptr_t)d_src | bytes) & 15) return fail(LITEVAR_E_INVALID_ARG, "pointer and size must be multiples of 16");
  if (bytes == 0) return LITEVAR_OK;
  hipLaunchKernelGGL(k_peak_read, dim3(8192), dim3(256), 0, (hipStream_t)stream, (const uint4*)d_src, (unsigned*)d_out, bytes / 16);
  return hip_check(hipGetLastError(), "read probe launch");
}

litevar_status litevar_peak_mfma_bf16(int32_t iters, void* d_out, double* flops, void* stream) {
  if (iters < 1 || iters > (1 << 24)) return fail(LITEVAR_E_INVALID_ARG, "iters must be in 1..2^24");
  if (!d_out) return fail(LITEVAR_E_INVALID_ARG, "d_out is NULL");
  constexpr int kBlocks = 256 * 8;                                  // eight waves per SIMD of 256 CUs
  hipLaunchKernelGGL(k_peak_mfma, dim3(kBlocks), dim3(256), 0, (hipStream_t)stream, iters, (float*)d_out);
  if (flops) *flops = (double)kBlocks * 4.0 * iters * 8.0 * (2.0 * 16 * 16 * 32);
  return hip_check(hipGetLastError(), "MFMA probe launch");
}

}  // extern "C"
