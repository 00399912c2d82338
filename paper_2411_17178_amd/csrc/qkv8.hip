// QKV8 (paper Section 4, "Quantization Scheme"): 8-bit Q, K, V with dynamic min-max
// parameters computed online, one (scale, zero point) per token row of 64 values.
//   quantise     x_q = rne(clamp((x - z) / s, -128, 127)),  z = (max + min)/2,
//                s = ((max - min)/2) / 127   (the printed scale lacks the integer range and the
//                printed clamp's upper bound is not an 8-bit code; s = 0 for a constant row,
//                whose codes are all 0)
//   dequantise   s x_q + z
// The code is an integer decided in floating point: the decision is taken in binary32 in
// exactly this order of operations (IEEE division, no contraction), so that the codes can be
// compared bit for bit with a CPU statement of the same formula.
//
// The attention entry point hands codes and parameters to the 16-patch attention kernel, which
// converts them on their way into its LDS ring; for plans with smaller groups it dequantises
// K, V and Q into a caller-owned bf16 workspace and runs the bf16 kernels on that copy.
#include "attn_bf16_common.h"

namespace lv {
namespace {

constexpr int kRowLanes = 8;          // lanes per token row: 8 values each

template <typename T> __device__ inline void load8(const T* p, float (&x)[8]);
template <> __device__ inline void load8<__bf16>(const __bf16* p, float (&x)[8]) {
  const bf16x8 v = as_bf16x8(*(const uint4*)p);
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = (float)v[e];
}
template <> __device__ inline void load8<float>(const float* p, float (&x)[8]) {
  const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

// eight lanes per row; a 256-thread block handles 32 rows
template <typename T>
__global__ __launch_bounds__(256) void k_quantize_rows(const T* __restrict__ x, int64_t rows, int64_t row_stride,
                                                       int8_t* __restrict__ xq, float2* __restrict__ sz) {
  const int64_t row = (int64_t)blockIdx.x * 32 + (threadIdx.x >> 3);
  const int part = threadIdx.x & 7;
  if (row >= rows) return;          // (whole eight-lane groups leave together: the shuffles below stay inside a group)
  float v[8];
  load8<T>(x + row * row_stride + 8 * part, v);
  float mx = v[0], mn = v[0];
#pragma unroll
  for (int e = 1; e < 8; ++e) { mx = fmaxf(mx, v[e]); mn = fminf(mn, v[e]); }
#pragma unroll
  for (int d = 1; d < kRowLanes; d <<= 1) {
    mx = fmaxf(mx, __shfl_xor(mx, d));
    mn = fminf(mn, __shfl_xor(mn, d));
  }
  const float z = (mx + mn) * 0.5f;
  const float s = __fdiv_rn((mx - mn) * 0.5f, 127.0f);
  uint32_t lo = 0, hi = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    float t = 0.0f;
    if (s > 0.0f) {
      t = __fdiv_rn(__fsub_rn(v[e], z), s);
      t = fminf(fmaxf(t, -128.0f), 127.0f);
      t = rintf(t);
    }
    const uint32_t byte = (uint32_t)(int)t & 0xffu;
    if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
  }
  *(uint2*)(xq + row * 64 + 8 * part) = make_uint2(lo, hi);
  if (part == 0) sz[row] = make_float2(s, z);
}

// int8 codes + (s, z) -> bf16(s q + z); eight lanes per row
__global__ __launch_bounds__(256) void k_dequantize_rows(const int8_t* __restrict__ xq, const float2* __restrict__ sz,
                                                         int64_t rows, __bf16* __restrict__ out) {
  const int64_t row = (int64_t)blockIdx.x * 32 + (threadIdx.x >> 3);
  const int part = threadIdx.x & 7;
  if (row >= rows) return;
  const uint2 c = *(const uint2*)(xq + row * 64 + 8 * part);
  const float2 p = sz[row];
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int8_t q = (int8_t)(((e < 4 ? c.x : c.y) >> (8 * (e & 3))) & 0xffu);
    r[e] = (__bf16)fmaf(p.x, (float)q, p.y);
  }
  *(bf16x8*)(out + row * 64 + 8 * part) = r;
}

litevar_status check_rows(int64_t rows) {
  if (rows < 0 || rows > ((int64_t)1 << 36)) return fail(LITEVAR_E_INVALID_ARG, "rows out of range");
  return LITEVAR_OK;
}

}  // namespace
}  // namespace lv

using namespace lv;

extern "C" {

litevar_status litevar_qkv8_quantize(const void* d_x, litevar_dtype dt, int64_t rows, int64_t row_stride,
                                     int32_t D, int8_t* d_codes, float* d_scale_zero, void* stream) {
  if (!d_x || !d_codes || !d_scale_zero) return fail(LITEVAR_E_INVALID_ARG, "d_x, d_codes or d_scale_zero is NULL");
  if (D != 64) return fail(LITEVAR_E_UNSUPPORTED, "rows of %d values are not supported (only 64)", D);
  if (dt != LITEVAR_BF16 && dt != LITEVAR_F32) return fail(LITEVAR_E_UNSUPPORTED, "unknown dtype %d", (int)dt);
  if (litevar_status s = check_rows(rows)) return s;
  if (row_stride < D || row_stride % 8) return fail(LITEVAR_E_INVALID_ARG, "row_stride must be a multiple of 8 and at least D");
  if (((uintptr_t)d_x & 15) || ((uintptr_t)d_codes & 7) || ((uintptr_t)d_scale_zero & 7))
    return fail(LITEVAR_E_INVALID_ARG, "d_x must be 16-byte aligned, d_codes and d_scale_zero 8-byte aligned");
  if (rows == 0) return LITEVAR_OK;
  const int64_t blocks = (rows + 31) / 32;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  hipStream_t st = (hipStream_t)stream;
  if (dt == LITEVAR_BF16)
    hipLaunchKernelGGL(k_quantize_rows<__bf16>, dim3((unsigned)blocks), dim3(256), 0, st, (const __bf16*)d_x, rows,
                       row_stride, d_codes, (float2*)d_scale_zero);
  else
    hipLaunchKernelGGL(k_quantize_rows<float>, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)d_x, rows,
                       row_stride, d_codes, (float2*)d_scale_zero);
  return hip_check(hipGetLastError(), "quantiser launch");
}

litevar_status litevar_qkv8_dequantize(const int8_t* d_codes, const float* d_scale_zero, int64_t rows, int32_t D,
                                       void* d_out_bf16, void* stream) {
  if (!d_codes || !d_scale_zero || !d_out_bf16) return fail(LITEVAR_E_INVALID_ARG, "a pointer is NULL");
  if (D != 64) return fail(LITEVAR_E_UNSUPPORTED, "rows of %d values are not supported (only 64)", D);
  if (litevar_status s = check_rows(rows)) return s;
  if (((uintptr_t)d_out_bf16 & 15) || ((uintptr_t)d_codes & 7) || ((uintptr_t)d_scale_zero & 7))
    return fail(LITEVAR_E_INVALID_ARG, "d_out_bf16 must be 16-byte aligned, d_codes and d_scale_zero 8-byte aligned");
  if (rows == 0) return LITEVAR_OK;
  const int64_t blocks = (rows + 31) / 32;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  hipLaunchKernelGGL(k_dequantize_rows, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, d_codes,
                     (const float2*)d_scale_zero, rows, (__bf16*)d_out_bf16);
  return hip_check(hipGetLastError(), "dequantiser launch");
}

// Plans whose groups hold 16 patches can be served by the attention kernel's own 8-bit form,
// which converts every key row once per group that streams it.  That pays while the groups of
// a (batch, head) stream few rows more than once (KV-cache steps: one group; the 680-token
// sequence); once they stream a quarter more rows than the three tensors hold (q_len + 2 kv_len
// per (batch, head)), a single dequantising pass over the tensors is cheaper (measured: both
// cost 35-40 ps per row; 2240 tokens: 9088 rows streamed against 6720, 276 against 262 us).
static bool fused(const litevar_plan* plan) {
  if (plan->waves_per_group != 16) return false;
  const int64_t streamed = plan->n_union_keys / (plan->n_head_groups > 0 ? plan->n_head_groups : 1);
  return 4 * streamed <= 5 * ((int64_t)plan->q_len + 2 * (int64_t)plan->kv_len);
}

litevar_status litevar_windowed_attn_qkv8_workspace_bytes(const litevar_plan* plan, int32_t B, int32_t H,
                                                          size_t* out_bytes) {
  if (!plan || !out_bytes) return fail(LITEVAR_E_INVALID_ARG, "plan or out_bytes is NULL");
  if (B < 1 || H < 1) return fail(LITEVAR_E_INVALID_ARG, "B and H must be positive");
  *out_bytes = fused(plan) ? 0 : (size_t)B * H * ((size_t)plan->q_len + 2 * (size_t)plan->kv_len) * 64 * 2;
  return LITEVAR_OK;
}

litevar_status litevar_windowed_attn_qkv8_fwd(const litevar_plan* plan, const int8_t* d_q, const float* d_q_sz,
                                              const int8_t* d_k, const float* d_k_sz, const int8_t* d_v,
                                              const float* d_v_sz, void* d_o, int32_t B, int32_t H, int32_t D,
                                              float sm_scale, const uint8_t* d_cfg_share, uint32_t flags,
                                              void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!plan) return fail(LITEVAR_E_INVALID_ARG, "plan is NULL");
  if (!d_q || !d_q_sz || !d_k || !d_k_sz || !d_v || !d_v_sz || !d_o)
    return fail(LITEVAR_E_INVALID_ARG, "a pointer is NULL");
  if (B < 1 || H < 1) return fail(LITEVAR_E_INVALID_ARG, "B and H must be positive (got %d, %d)", B, H);
  const bool forced = (flags & LITEVAR_FLAG_QKV8_IN_KERNEL) != 0;
  flags &= ~(uint32_t)LITEVAR_FLAG_QKV8_IN_KERNEL;
  if (forced && plan->waves_per_group != 16)
    return fail(LITEVAR_E_UNSUPPORTED, "in-kernel conversion needs a plan with 16 patches per group (this one has %d)",
                plan->waves_per_group);
  if (forced || fused(plan)) {
    // codes and parameters go straight to the attention kernel: no dequantised copy
    AttnArgs a;
    if (litevar_status s = make_attn_args(plan, B, H, D, sm_scale, d_cfg_share, flags, a)) return s;
    const uintptr_t align = (uintptr_t)d_q | (uintptr_t)d_k | (uintptr_t)d_v | (uintptr_t)d_o;
    if (align & 15) return fail(LITEVAR_E_INVALID_ARG, "q, k, v, o must be 16-byte aligned");
    if (((uintptr_t)d_q_sz | (uintptr_t)d_k_sz | (uintptr_t)d_v_sz) & 7)
      return fail(LITEVAR_E_INVALID_ARG, "the (scale, zero point) arrays must be 8-byte aligned");
    if ((int64_t)plan->kv_len * 64 >= ((int64_t)1 << 31))
      return fail(LITEVAR_E_UNSUPPORTED, "one (batch, head) slab of k/v spans 2 GiB or more");
    a.q = d_q; a.k = d_k; a.v = d_v; a.o = d_o;
    a.qs[2] = 64; a.qs[1] = (int64_t)plan->q_len * 64; a.qs[0] = a.qs[1] * H;
    a.ks[2] = 64; a.ks[1] = (int64_t)plan->kv_len * 64; a.ks[0] = a.ks[1] * H;
    a.os[2] = 64; a.os[1] = (int64_t)plan->q_len * 64; a.os[0] = a.os[1] * H;
    a.q_sz = (const float2*)d_q_sz; a.k_sz = (const float2*)d_k_sz; a.v_sz = (const float2*)d_v_sz;
    return launch_attn_bf16_pair(plan, a, (hipStream_t)stream);
  }
  if (!d_workspace) return fail(LITEVAR_E_INVALID_ARG, "d_workspace is NULL");
  size_t need = 0;
  if (litevar_status s = litevar_windowed_attn_qkv8_workspace_bytes(plan, B, H, &need)) return s;
  if (workspace_bytes < need)
    return fail(LITEVAR_E_INVALID_ARG, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
  if ((uintptr_t)d_workspace & 255) return fail(LITEVAR_E_INVALID_ARG, "d_workspace must be 256-byte aligned");
  const int64_t rows_q = (int64_t)B * H * plan->q_len, rows_kv = (int64_t)B * H * plan->kv_len;
  __bf16* qd = (__bf16*)d_workspace;
  __bf16* kd = qd + rows_q * 64;
  __bf16* vd = kd + rows_kv * 64;
  if (litevar_status s = litevar_qkv8_dequantize(d_q, d_q_sz, rows_q, D, qd, stream)) return s;
  if (litevar_status s = litevar_qkv8_dequantize(d_k, d_k_sz, rows_kv, D, kd, stream)) return s;
  if (litevar_status s = litevar_qkv8_dequantize(d_v, d_v_sz, rows_kv, D, vd, stream)) return s;
  return litevar_windowed_attn_fwd(plan, qd, kd, vd, d_o, B, H, D, LITEVAR_BF16, nullptr, nullptr, nullptr, sm_scale,
                                   d_cfg_share, flags, stream);
}

}  // extern "C"
