// bf16 windowed attention forward for gfx950 (CDNA4), Section 2 of the paper:
// O = softmax(sm_scale * Q K^T over the kept keys) V, with the Section 3 cond ->
// uncond output reuse folded into the store.
//
// One workgroup = one group of up to NW 4x4 query patches (one wave each) of one
// (batch, head).  The workgroup streams the group's key list (K and V rows) from
// HBM/L2 through an LDS ring in chunks of C keys; each wave then runs its own
// 32-key steps, gathering rows from the ring by slot index:
//   S^T (keys x queries) = K_tile (A operand, 16 keys x 64) . Q^T (B operand)
//       -> v_mfma_f32_16x16x32_bf16, two per 16-key tile; a lane ends up holding
//          one query column and four keys, so the softmax state is per lane;
//   mask bits (one per lane and key) -> -inf, online softmax in base 2;
//   O^T (64 x queries) += V^T (A operand, via ds_read_b64_tr_b16) . P^T (B operand,
//          the lane's own eight probabilities rounded to bf16).
// Steps that do not touch a patch's windows are simply absent from its list, so
// fully masked tiles cost nothing.
#include "internal.h"

namespace lv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kRowBytes = 144;   // 128-byte row + 16 bytes so that 16 rows hit distinct banks
constexpr float kFloor = -1.0e30f;  // running-max floor: keeps exp2 arguments finite

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline s16x4 lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(p));
}

template <int NW, int C, int NR>
__global__ __launch_bounds__(NW * 64) void k_attn_bf16(AttnArgs a, float c) {
  constexpr int T = NW * 64;
  constexpr int R = NR * C;
  constexpr int PT = C * 16 / T;           // 16-byte pieces per thread per chunk
  static_assert(PT >= 1 && PT * T == C * 16, "chunk must be a whole number of passes");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* const Kring = smem;
  unsigned char* const Vring = smem + R * kRowBytes;

  // workgroup i runs on XCD i % 8: keep all groups of one (batch, head) on one XCD so
  // its K/V are fetched into a single L2
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int bh = (seq / a.n_groups) * 8 + xcd, grp = seq % a.n_groups;
  if (bh >= a.B * a.H) return;
  const int b = bh / a.H, h = bh % a.H;
  const GroupDesc gd = a.groups[grp];
  const bool shared = a.cfg_share && a.cfg_share[h * a.n_scales + gd.k];
  if (shared && b >= a.B / 2) return;      // the conditional workgroup writes this row

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, n = lane & 15, g4 = lane >> 4;
  const WaveDesc wd = a.waves[grp * NW + wave];

  const __bf16* Kp = (const __bf16*)a.k + b * a.ks[0] + h * a.ks[1];
  const __bf16* Vp = (const __bf16*)a.v + b * a.ks[0] + h * a.ks[1];
  const int32_t* utok = a.union_tok + gd.union_base;

  uint4 stage[PT];
  auto issue = [&](int chunk) {
#pragma unroll
    for (int p = 0; p < PT; ++p) {
      const int id = tid + p * T, kl = id >> 4, part = id & 15;
      const int64_t tok = utok[chunk * C + kl];
      const __bf16* src = (part < 8 ? Kp : Vp) + tok * a.ks[2] + (part & 7) * 8;
      stage[p] = *(const uint4*)src;
    }
  };
  auto commit = [&](int chunk) {
#pragma unroll
    for (int p = 0; p < PT; ++p) {
      const int id = tid + p * T, kl = id >> 4, part = id & 15;
      const int slot = (chunk % NR) * C + kl;
      unsigned char* dst = (part < 8 ? Kring : Vring) + slot * kRowBytes + (part & 7) * 16;
      *(uint4*)dst = stage[p];
    }
  };

  // Q^T as the B operand: lane (n, g4) holds Q[query n][16*g4 .. 16*g4+15]
  const int dy = n >> 2, dx = n & 3;
  const int qrow = (dy < wd.ny && dx < wd.nx) ? wd.q_base + dy * wd.sk + dx : -1;
  bf16x8 qb0, qb1;
  {
    uint4 z = {0, 0, 0, 0}, q0 = z, q1 = z;
    if (qrow >= 0) {
      const __bf16* qp = (const __bf16*)a.q + b * a.qs[0] + h * a.qs[1] + qrow * a.qs[2] + 16 * g4;
      q0 = *(const uint4*)qp; q1 = *(const uint4*)(qp + 8);
    }
    qb0 = as_bf16x8(q0); qb1 = as_bf16x8(q1);
  }

  issue(0);
  commit(0);
  __syncthreads();

  float m = kFloor, l = 0.f;
  f32x4 O[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const uint16_t* pe = a.phase_end + gd.phase_base + wave * gd.n_phases;
  const uint32_t* words = a.step_words + (int64_t)wd.step_begin * 64 + lane;
  int done = 0;
  uint32_t w_next = wd.n_steps > 0 ? words[0] : 0u;

  for (int ph = 0; ph < gd.n_phases; ++ph) {
    const bool more = ph + 1 < gd.n_phases;
    if (more) issue(ph + 1);
    const int end = __builtin_amdgcn_readfirstlane((int)pe[ph]);
    for (; done < end; ++done) {
      const uint32_t w = w_next;
      if (done + 1 < wd.n_steps) w_next = words[(int64_t)(done + 1) * 64];
      const uint32_t bits = w >> 16;
      const int ks0 = __shfl((int)w, n) & 0xffff, ks1 = __shfl((int)w, 16 + n) & 0xffff;
      const int vs0 = __shfl((int)w, 4 * g4 + (n >> 2)) & 0xffff;
      const int vs1 = __shfl((int)w, 16 + 4 * g4 + (n >> 2)) & 0xffff;

      // S^T tiles: keys x queries
      const unsigned char* k0p = Kring + ks0 * kRowBytes + g4 * 32;
      const unsigned char* k1p = Kring + ks1 * kRowBytes + g4 * 32;
      const bf16x8 k00 = as_bf16x8(*(const uint4*)k0p), k01 = as_bf16x8(*(const uint4*)(k0p + 16));
      const bf16x8 k10 = as_bf16x8(*(const uint4*)k1p), k11 = as_bf16x8(*(const uint4*)(k1p + 16));
      f32x4 S0 = {0.f, 0.f, 0.f, 0.f}, S1 = {0.f, 0.f, 0.f, 0.f};
      S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k00, qb0, S0, 0, 0, 0);
      S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k10, qb0, S1, 0, 0, 0);
      S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k01, qb1, S0, 0, 0, 0);
      S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k11, qb1, S1, 0, 0, 0);

      // V^T operand: transposing LDS reads, 4 keys x 16 dims per 16-lane block
      const unsigned char* v0p = Vring + vs0 * kRowBytes + (n & 3) * 8;
      const unsigned char* v1p = Vring + vs1 * kRowBytes + (n & 3) * 8;
      s16x4 va[4][2];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        va[dt][0] = lds_read_tr16(v0p + dt * 32);
        va[dt][1] = lds_read_tr16(v1p + dt * 32);
      }

      float sv[8] = {S0[0], S0[1], S0[2], S0[3], S1[0], S1[1], S1[2], S1[3]};
#pragma unroll
      for (int e = 0; e < 8; ++e) sv[e] = (bits >> e & 1) ? sv[e] : -INFINITY;
      float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                       fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
      const float mc = m_new * c;
      m = m_new;
      float p[8], psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) { p[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], c, -mc)); psum += p[e]; }
      l = fmaf(l, alpha, psum);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) O[dt] *= alpha;

      bf16x8 pb;
#pragma unroll
      for (int e = 0; e < 8; ++e) pb[e] = (__bf16)p[e];
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        s16x8 v8 = {va[dt][0][0], va[dt][0][1], va[dt][0][2], va[dt][0][3],
                    va[dt][1][0], va[dt][1][1], va[dt][1][2], va[dt][1][3]};
        O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v8), pb, O[dt], 0, 0, 0);
      }
    }
    if (more) commit(ph + 1);
    __syncthreads();
  }

  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (qrow < 0) return;
  const float inv = 1.f / l;
  __bf16* op = (__bf16*)a.o + b * a.os[0] + h * a.os[1] + qrow * a.os[2] + 4 * g4;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    bf16x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = (__bf16)(O[dt][i] * inv);
    *(bf16x4*)(op + 16 * dt) = r;
    if (shared) *(bf16x4*)(op + (a.B / 2) * a.os[0] + 16 * dt) = r;
  }
}

template <int NW, int C, int NR>
static litevar_status launch(const AttnArgs& a, hipStream_t st) {
  const size_t smem = (size_t)NR * C * kRowBytes * 2;
  static thread_local bool attr_set = false;
  if (!attr_set) {
    litevar_status rc = hip_check(
        hipFuncSetAttribute((const void*)k_attn_bf16<NW, C, NR>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem),
        "hipFuncSetAttribute(max dynamic LDS)");
    if (rc) return rc;
    attr_set = true;
  }
  const int64_t bh8 = ((int64_t)a.B * a.H + 7) / 8 * 8;
  const int64_t blocks = bh8 * a.n_groups;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  const float c = a.sm_scale * 1.4426950408889634f;
  hipLaunchKernelGGL((k_attn_bf16<NW, C, NR>), dim3((unsigned)blocks), dim3(NW * 64), smem, st, a, c);
  return hip_check(hipGetLastError(), "bf16 attention launch");
}

litevar_status launch_attn_bf16(const litevar_plan* pl, const AttnArgs& a, hipStream_t st) {
  const int nw = pl->waves_per_group, C = pl->chunk_keys, NR = pl->ring_chunks;
  if (nw == 16 && C == 128 && NR == 3) return launch<16, 128, 3>(a, st);
  if (nw == 8 && C == 64 && NR == 3) return launch<8, 64, 3>(a, st);
  if (nw == 4 && C == 64 && NR == 3) return launch<4, 64, 3>(a, st);
  return fail(LITEVAR_E_PLAN_CORRUPT, "no kernel for waves=%d chunk=%d ring=%d", nw, C, NR);
}

}  // namespace lv
