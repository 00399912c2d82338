// bf16 windowed attention forward for gfx950 (CDNA4), Section 2 of the paper, for plans
// with 16 patches per group: O = softmax(sm_scale * Q K^T over the kept keys) V, with the
// Section 3 cond -> uncond output reuse folded into the store.
//
// One workgroup = eight waves = one group of up to 16 query patches (16 x 16 queries of
// one scale) of one (batch, head).  Every wave owns two patches (a top and a bottom one,
// so that it has keys in most parts of the stream) and one eighth of the loading.
//
// The group's key list is streamed once through an LDS ring of NRB chunks of 64 keys
// (one 128-byte K row and one 128-byte V row per key, 16-byte pieces XOR-swizzled by
// slot).  Phase c = the steps whose last key lies in chunk c; they read chunks c and c-1.
// At the start of phase c every wave issues, in this order,
//   the descriptor loads of its steps of phase c+1 (register-returning, always six),
//   the token load for its rows of chunk c+3,
//   two global_load_lds_dwordx4 for its eight K rows and eight V rows of chunk c+2
//   (the slot held chunk c-2, which nobody reads after phase c-1),
// then runs its steps of phase c, waits until at most the two youngest of its vector
// memory operations (the two LDS-DMA loads just issued) are outstanding -- vmcnt is
// in-order, so chunk c+1 and everything else has landed -- and joins the barrier.  Two
// chunks (32 KiB) per workgroup are therefore in flight at any time, and a key row is
// moved from HBM/L2 to LDS exactly once per (batch, head, group).
//
// A wave that issues LDS-DMA loads must read LDS through inline assembly: the compiler
// cannot tell which of them a plain LDS read depends on and would wait for all
// (vmcnt(0)), which would serialise the stream.
//
// Step arithmetic is that of the 8-patch kernel: S^T = K_tile . Q^T by
// v_mfma_f32_16x16x32_bf16 (a lane owns one query column and four keys per tile), scalar
// lane masks applied with v_cndmask, base-2 online softmax with a lazily updated
// reference, O^T += V^T . P^T with ds_read_b64_tr_b16 operands, row sums by a fifth MFMA.
#include <type_traits>

#include "attn_bf16_common.h"

namespace lv {

namespace {

constexpr int kPairWaves = 8;         // waves per workgroup
constexpr int kPairChunk = 64;        // keys per chunk

__device__ inline unsigned lds_addr(const void* p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// four 16-byte K pieces (two keys x two halves of the head dimension); waits for them
__device__ inline void lds_read_k(unsigned a0, unsigned a1, uint4& k00, uint4& k01, uint4& k10, uint4& k11) {
  asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\t"
               "ds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
               "s_waitcnt lgkmcnt(0)"
               : "=&v"(k00), "=&v"(k01), "=&v"(k10), "=&v"(k11)
               : "v"(a0), "v"(a0 ^ 16u), "v"(a1), "v"(a1 ^ 16u) : "memory");
}

// transposing reads of the V^T operands of one step (4 head-dim tiles x 2 key halves);
// issued only: lds_wait() must precede the first use
template <int VOFF>
__device__ inline void lds_read_v(unsigned v0, unsigned v1, uint2 (&va)[4][2]) {
  asm volatile("ds_read_b64_tr_b16 %0, %8 offset:%16\n\tds_read_b64_tr_b16 %1, %9 offset:%16\n\t"
               "ds_read_b64_tr_b16 %2, %10 offset:%16\n\tds_read_b64_tr_b16 %3, %11 offset:%16\n\t"
               "ds_read_b64_tr_b16 %4, %12 offset:%16\n\tds_read_b64_tr_b16 %5, %13 offset:%16\n\t"
               "ds_read_b64_tr_b16 %6, %14 offset:%16\n\tds_read_b64_tr_b16 %7, %15 offset:%16"
               : "=&v"(va[0][0]), "=&v"(va[0][1]), "=&v"(va[1][0]), "=&v"(va[1][1]),
                 "=&v"(va[2][0]), "=&v"(va[2][1]), "=&v"(va[3][0]), "=&v"(va[3][1])
               : "v"(v0), "v"(v1), "v"(v0 ^ 32u), "v"(v1 ^ 32u), "v"(v0 ^ 64u), "v"(v1 ^ 64u),
                 "v"(v0 ^ 96u), "v"(v1 ^ 96u), "i"(VOFF) : "memory");
}

// waits for the reads issued by lds_read_v; the operands are tied so that no use is
// scheduled above the wait
__device__ inline void lds_wait(uint2 (&va)[4][2]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(va[0][0]), "+v"(va[0][1]), "+v"(va[1][0]), "+v"(va[1][1]),
                 "+v"(va[2][0]), "+v"(va[2][1]), "+v"(va[3][0]), "+v"(va[3][1]) : : "memory");
}

struct PatchState {       // one query patch of a wave
  bf16x8 qb0, qb1;        // Q^T as the B operand: lane (n, g4) holds Q[query n][16 g4 .. +15]
  f32x4 O[4], Lacc;       // O^T accumulators and row sums
  float m;                // softmax reference
  int qrow;               // local query row of this lane's query column, -1 = none
};

}  // namespace

template <int NRB>
__global__ __launch_bounds__(kPairWaves * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_attn_bf16_pair(AttnArgs a, float c) {
  constexpr int C = kPairChunk;
  constexpr int R = NRB * C;                       // ring slots
  constexpr int VOFF = R * kRingRowBytes;          // V ring follows the K ring
  static_assert(2 * R * kRingRowBytes <= 65536, "static LDS");
  __shared__ __align__(1024) unsigned char smem[2 * R * kRingRowBytes];
  unsigned char* const Kring = smem;
  unsigned char* const Vring = smem + VOFF;

  // workgroup i runs on XCD i % 8: all groups of one (batch, head) share one L2
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int bh = (seq / a.n_groups) * 8 + xcd, grp = seq % a.n_groups;
  if (bh >= a.B * a.H) return;
  const int b = bh / a.H, h = bh % a.H;
  const GroupDesc gd = a.groups[grp];
  const bool shared = a.cfg_share && a.cfg_share[h * a.n_scales + gd.k];
  if (shared && b >= a.B / 2) return;      // the conditional workgroup writes this row

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n = lane & 15, g4 = lane >> 4;
  const int P = __builtin_amdgcn_readfirstlane(gd.n_phases);

  // ---- loading duty: rows [8 wave, 8 wave + 8) of every chunk ----
  const unsigned char* Kp = (const unsigned char*)((const __bf16*)a.k + b * a.ks[0] + h * a.ks[1]);
  const unsigned char* Vp = (const unsigned char*)((const __bf16*)a.v + b * a.ks[0] + h * a.ks[1]);
  const unsigned row_bytes = (unsigned)a.ks[2] * 2u;   // a (batch, head) slab spans < 2 GiB (checked by the API)
  const int32_t* utok = a.union_tok + gd.union_base;
  const int ident = __builtin_amdgcn_readfirstlane(gd.ident);   // union entries [0, ident) are token i at position i
  const int row = 8 * wave + (lane >> 3), pos = lane & 7;
  auto issue_chunk = [&](int t, int tok) {             // chunk t -> ring slots (t % NRB) * 64 ...
    const int slot0 = (t % NRB) * C + 8 * wave;
    const unsigned slot = (unsigned)(slot0 + (lane >> 3));
    const unsigned src = (unsigned)tok * row_bytes + (((unsigned)pos ^ ring_swizzle(slot)) << 4);
    __builtin_amdgcn_global_load_lds((global_void*)(Kp + src), (lds_void*)(Kring + slot0 * kRingRowBytes), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((global_void*)(Vp + src), (lds_void*)(Vring + slot0 * kRingRowBytes), 16, 0, 0);
  };

  // ---- the wave's two patches: p and its partner two patch rows below, columns swapped ----
  const int pa = wave, pb_ = ((wave >> 2) + 2) * 4 + ((wave & 3) ^ 1);
  const WaveDesc wdA = a.waves[grp * 16 + pa], wdB = a.waves[grp * 16 + pb_];
  const int nsA = __builtin_amdgcn_readfirstlane(wdA.n_steps), nsB = __builtin_amdgcn_readfirstlane(wdB.n_steps);
  const int64_t sbA = __builtin_amdgcn_readfirstlane(wdA.step_begin), sbB = __builtin_amdgcn_readfirstlane(wdB.step_begin);
  const const_i32_ptr peA = (const_i32_ptr)(a.phase_end + gd.phase_base + pa * P);
  const const_i32_ptr peB = (const_i32_ptr)(a.phase_end + gd.phase_base + pb_ * P);
  // (an idle patch has no steps of its own: its clamped descriptor loads read step 0 of the plan)
  const uint2* addrA = a.step_addr + (nsA > 0 ? sbA : 0) * 64 + lane;
  const uint2* addrB = a.step_addr + (nsB > 0 ? sbB : 0) * 64 + lane;
  const uint64_t* maskA = a.step_mask + sbA * 8;
  const uint64_t* maskB = a.step_mask + sbB * 8;

  auto init_patch = [&](PatchState& ps, const WaveDesc& wd) {
    const int dy = n >> 2, dx = n & 3;
    ps.qrow = (dy < wd.ny && dx < wd.nx) ? wd.q_base + dy * wd.sk + dx : -1;
    uint4 z = {0, 0, 0, 0}, q0 = z, q1 = z;
    if (ps.qrow >= 0) {
      const __bf16* qp = (const __bf16*)a.q + b * a.qs[0] + h * a.qs[1] + ps.qrow * a.qs[2] + 16 * g4;
      q0 = *(const uint4*)qp; q1 = *(const uint4*)(qp + 8);
    }
    ps.qb0 = as_bf16x8(q0); ps.qb1 = as_bf16x8(q1);
    ps.m = kFloor;
    ps.Lacc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) ps.O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  PatchState A, B;
  init_patch(A, wdA);
  init_patch(B, wdB);

  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  const float slack = kSlack / c;

  // descriptors of the steps of one phase: always kMaxPhaseSteps loads per patch (clamped
  // to the patch's last step), so that the number of loads in flight is static
  auto load_desc = [&](uint2 (&d)[kMaxPhaseSteps], const uint2* addrs, int first, int n_steps) {
#pragma unroll
    for (int i = 0; i < kMaxPhaseSteps; ++i)
      d[i] = addrs[(int64_t)max(min(first + i, n_steps - 1), 0) * 64];
  };
  // this lane's row of chunk t (the load is unconditional so that the number of vector
  // memory operations per phase is static)
  auto load_tok = [&](int t) -> int {
    const int i = t * C + row;
    const int v = utok[i];
    return i < ident ? i : v;
  };

  // ---- prologue: descriptors of phase 0, tokens of chunks 0..2, chunks 0 and 1 ----
  uint2 dA[kMaxPhaseSteps], dB[kMaxPhaseSteps], dAn[kMaxPhaseSteps], dBn[kMaxPhaseSteps];
  load_desc(dA, addrA, 0, nsA);
  load_desc(dB, addrB, 0, nsB);
  int tok_next = load_tok(P > 2 ? 2 : 0);               // token of the chunk issued next
  {
    const int t0 = load_tok(0), t1 = load_tok(P > 1 ? 1 : 0);
    issue_chunk(0, t0);
    if (P > 1) issue_chunk(1, t1);
  }
  if (P > 1) wait_vmcnt<2>(); else wait_vmcnt<0>();     // chunk 0 is in; chunk 1 may be in flight
  asm volatile("s_barrier" ::: "memory");

  // One step: 32 keys against the 16 queries of patch ps.
  auto run_step = [&](PatchState& ps, const uint2 cur, const uint64_t* masks, int s) {
    const const_u64_ptr mk = (const_u64_ptr)(masks + (int64_t)s * 8);
    uint4 k00, k01, k10, k11;
    lds_read_k(lds_addr(Kring + (cur.x & 0xffffu)), lds_addr(Kring + (cur.x >> 16)), k00, k01, k10, k11);
    f32x4 S0 = {0.f, 0.f, 0.f, 0.f}, S1 = {0.f, 0.f, 0.f, 0.f};
    S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k00), ps.qb0, S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k10), ps.qb0, S1, 0, 0, 0);
    S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k01), ps.qb1, S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k11), ps.qb1, S1, 0, 0, 0);

    float sv[8] = {S0[0], S0[1], S0[2], S0[3], S1[0], S1[1], S1[2], S1[3]};
#pragma unroll
    for (int e = 0; e < 8; ++e) sv[e] = mask_select(sv[e], mk[e]);
    float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                     fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    mx = max_across_rows(mx);
    const bool grow = mx > ps.m + slack;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {      // rare after the first steps
      const float m_new = grow ? mx : ps.m;
      const float alpha = __builtin_amdgcn_exp2f((ps.m - m_new) * c);
      ps.m = m_new;
      ps.Lacc *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) ps.O[dt] *= alpha;
    }
    const float mc = ps.m * c;
    // V^T operands: issued here rather than before the softmax, where sixteen more live
    // registers would not fit
    uint2 va[4][2];
    lds_read_v<VOFF>(lds_addr(Kring + (cur.y & 0xffffu)), lds_addr(Kring + (cur.y >> 16)), va);
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], c, -mc));
    bf16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) pb[e] = (__bf16)p[e];

    lds_wait(va);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const uint4 v8 = {va[dt][0].x, va[dt][0].y, va[dt][1].x, va[dt][1].y};
      ps.O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(v8), pb, ps.O[dt], 0, 0, 0);
    }
    ps.Lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb, ps.Lacc, 0, 0, 0);
  };

  // ---- phases ----
  // DMA: chunk ph + 2 exists and is issued; NEXT: phase ph + 1 exists.  All vector memory
  // operations of a phase are unconditional, so the compiler's own waits are exact.
  int doneA = 0, doneB = 0;                             // steps finished so far
  auto run_phase = [&](int ph, auto dma, auto next) {
    constexpr bool DMA = decltype(dma)::value, NEXT = decltype(next)::value;
    const int endA = nsA > 0 ? peA[ph] : 0, endB = nsB > 0 ? peB[ph] : 0;
    if constexpr (NEXT) {                               // descriptors of the next phase
      load_desc(dAn, addrA, endA, nsA);
      load_desc(dBn, addrB, endB, nsB);
    }
    if constexpr (DMA) {
      const int tok = tok_next;
      tok_next = load_tok(min(ph + 3, P - 1));
      issue_chunk(ph + 2, tok);
    }
#pragma unroll
    for (int i = 0; i < kMaxPhaseSteps; ++i)
      if (doneA + i < endA) run_step(A, dA[i], maskA, doneA + i);
#pragma unroll
    for (int i = 0; i < kMaxPhaseSteps; ++i)
      if (doneB + i < endB) run_step(B, dB[i], maskB, doneB + i);
    doneA = endA; doneB = endB;
    if constexpr (NEXT) {
      // everything but the two DMA loads just issued has landed: chunk ph + 1, the next
      // descriptors and tokens.  All LDS reads of this phase have returned (each step
      // waits for its own), so the slot of chunk ph - 1 may be overwritten after the barrier.
      if constexpr (DMA) wait_vmcnt<2>(); else wait_vmcnt<0>();
      asm volatile("s_barrier" ::: "memory");
#pragma unroll
      for (int i = 0; i < kMaxPhaseSteps; ++i) { dA[i] = dAn[i]; dB[i] = dBn[i]; }
    }
  };
  {
    int ph = 0;
    for (; ph + 2 < P; ++ph) run_phase(ph, std::true_type{}, std::true_type{});
    if (ph + 1 < P) { run_phase(ph, std::false_type{}, std::true_type{}); ++ph; }
    run_phase(ph, std::false_type{}, std::false_type{});
  }

  // ---- epilogue ----
  auto store_patch = [&](const PatchState& ps) {
    if (ps.qrow < 0) return;
    const float inv = 1.f / ps.Lacc[0];
    __bf16* op = (__bf16*)a.o + b * a.os[0] + h * a.os[1] + ps.qrow * a.os[2] + 4 * g4;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      bf16x4 r;
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = (__bf16)(ps.O[dt][i] * inv);
      *(bf16x4*)(op + 16 * dt) = r;
      if (shared) *(bf16x4*)(op + (a.B / 2) * a.os[0] + 16 * dt) = r;
    }
  };
  store_patch(A);
  store_patch(B);
}

litevar_status launch_attn_bf16_pair(const litevar_plan* pl, const AttnArgs& a, hipStream_t st) {
  if (pl->waves_per_group != 16 || pl->chunk_keys != kPairChunk || pl->ring_chunks != 4)
    return fail(LITEVAR_E_PLAN_CORRUPT, "no 16-patch kernel for chunk=%d ring=%d", pl->chunk_keys, pl->ring_chunks);
  const int64_t bh8 = ((int64_t)a.B * a.H + 7) / 8 * 8;
  const int64_t blocks = bh8 * a.n_groups;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  const float c = a.sm_scale * 1.4426950408889634f;
  hipLaunchKernelGGL((k_attn_bf16_pair<4>), dim3((unsigned)blocks), dim3(kPairWaves * 64), 0, st, a, c);
  return hip_check(hipGetLastError(), "bf16 attention launch");
}

}  // namespace lv
