// fp32 windowed attention forward: the accuracy path (1e-5 against the fp64 oracle).
// One 64-lane wave per (batch, head, query patch).  Lane (n, g4) = query column n of
// the patch, head-dim slice [16*g4, 16*g4+16).  It walks the same per-patch steps
// and lane masks as the bf16 MFMA kernel, reading K and V rows straight from global
// memory, with a scalar online softmax (Section 2 of the paper: softmax over the
// kept keys only).
#include "attn_bf16_common.h"

namespace lv {

__global__ __launch_bounds__(64) void k_attn_f32(AttnArgs a, int n_waves) {
  const int wv = blockIdx.x % n_waves, bh = blockIdx.x / n_waves;
  if (!plan_usable(a.hdr)) return;
  const int b = bh / a.H, h = bh % a.H;
  const WaveDesc wd = a.waves[wv + (a.head_map ? a.head_map[h] * n_waves : 0)];   // the head group's patches
  if (wd.ny == 0) return;
  const bool shared = a.cfg_share && a.cfg_share[h * a.n_scales + wd.kq];
  if (shared && b >= a.B / 2) return;

  const int lane = threadIdx.x, n = lane % 16, g4 = lane / 16;
  const int dy = n / 4, dx = n % 4;
  const int qrow = ((wd.valid >> n) & 1u) ? checked_index(a.hdr, wd.q_base + dy * wd.sk + dx, a.q_len) : -1;

  const float* Q = (const float*)a.q + b * a.qs[0] + h * a.qs[1];
  const float* Kp = (const float*)a.k + b * a.ks[0] + h * a.ks[1];
  const float* Vp = (const float*)a.v + b * a.ks[0] + h * a.ks[1];

  float qv[16], acc[16];
  for (int d = 0; d < 16; ++d) {
    qv[d] = qrow >= 0 ? Q[qrow * a.qs[2] + 16 * g4 + d] : 0.f;
    acc[d] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  for (int s = 0; s < wd.n_steps; ++s) {
    const int64_t S = (int64_t)wd.step_begin + s;
    for (int i = 0; i < kStepKeys; ++i) {
      int tok = a.step_tok[S * kStepKeys + i];
      if (tok < 0) continue;                      // padding key (uniform over the wave)
      tok = checked_index(a.hdr, tok, a.kv_len);
      const float* kr = Kp + tok * a.ks[2] + 16 * g4;
      float dot = 0.f;
      for (int d = 0; d < 16; ++d) dot = fmaf(qv[d], kr[d], dot);
      dot += __shfl_xor(dot, 16);
      dot += __shfl_xor(dot, 32);
      const int r = i % 16;
      const bool keep = a.step_mask[S * 8 + 4 * (i / 16) + r % 4] >> ((r / 4) * 16 + n) & 1;
      if (keep) {
        const float z = dot * a.sm_scale;
        const float m_new = fmaxf(m, z);
        const float alpha = expf(m - m_new);      // exp(-inf) = 0 on the first kept key
        const float p = expf(z - m_new);
        const float* vr = Vp + tok * a.ks[2] + 16 * g4;
        l = l * alpha + p;
        for (int d = 0; d < 16; ++d) acc[d] = fmaf(p, vr[d], acc[d] * alpha);
        m = m_new;
      }
    }
  }
  if (qrow < 0) return;
  const float inv = 1.f / l;
  float* O = (float*)a.o + b * a.os[0] + h * a.os[1] + qrow * a.os[2] + 16 * g4;
  for (int d = 0; d < 16; ++d) O[d] = acc[d] * inv;
  if (shared) {
    float* O2 = O + (a.B / 2) * a.os[0];
    for (int d = 0; d < 16; ++d) O2[d] = acc[d] * inv;
  }
}

litevar_status launch_attn_f32(const litevar_plan* pl, const AttnArgs& a, hipStream_t st) {
  const int64_t n_waves = (int64_t)pl->n_groups * pl->waves_per_group;
  const int64_t blocks = n_waves * a.B * a.H;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large for the fp32 path");
  hipLaunchKernelGGL(k_attn_f32, dim3((unsigned)blocks), dim3(64), 0, st, a, (int)n_waves);
  return hip_check(hipGetLastError(), "fp32 attention launch");
}

}  // namespace lv
