// bf16 windowed attention forward for gfx950 (CDNA4), Section 2 of the paper:
// O = softmax(sm_scale * Q K^T over the kept keys) V, with the Section 3 cond ->
// uncond output reuse folded into the store.
//
// One workgroup = one group of up to NW 4x4 query patches of one (batch, head):
// NW compute waves (one patch each) plus one loader wave.
//
// Loader wave: streams the group's key list (K and V rows, 128 B each) from HBM/L2
// into an LDS ring with global_load_lds_dwordx4 (no registers in between), D chunks of
// C keys in flight.  Token indices come from a small LDS token ring that is filled the
// same way, so the loader never waits on a register-returning load (vmcnt is in-order:
// such a wait would drain the whole prefetch queue).
//
// Compute waves: each runs its own list of 32-key steps, gathering rows from the ring
// at pre-swizzled byte offsets stored in the plan:
//   S^T (keys x queries) = K_tile (A operand, 16 keys x 64) . Q^T (B operand)
//       -> v_mfma_f32_16x16x32_bf16, two per 16-key tile; a lane ends up holding one
//          query column and four keys of each tile, so the softmax state is per lane;
//   mask: eight 64-bit lane masks per step, read with scalar loads and applied with one
//          v_cndmask per score (SGPR-pair select);
//   online softmax in base 2, row maxima combined across the four 16-lane rows with
//          v_permlane32_swap / v_permlane16_swap;
//   O^T (64 x queries) += V^T (A operand, via ds_read_b64_tr_b16) . P^T (B operand, the
//          lane's own eight probabilities rounded to bf16).
// Steps that do not touch a patch's windows are absent from its list, so fully masked
// tiles cost nothing.
//
// Synchronisation is producer/consumer through LDS words, not barriers: the loader
// publishes the number of chunks that have landed, every compute wave publishes the
// phase it has reached; a compute wave waits only when its next keys are not there yet,
// the loader only when the ring slot it wants to refill is still being read.  Waves of
// one workgroup may therefore be several chunks apart (the ring has S spare chunks).
#include <type_traits>

#include "attn_bf16_common.h"

namespace lv {

constexpr int kTokBatchChunks = 8;   // chunks covered by one token batch
constexpr int kAhead = 4;            // step descriptors fetched ahead by a compute wave

// (a nine-wave workgroup gets two per CU only up to 80 VGPRs: three of its waves share SIMD 0)
template <int NW, int C, int A, int D, int S>
__global__ __launch_bounds__((NW + 1) * 64) __attribute__((amdgpu_waves_per_eu((NW == 8 && C == 32) ? 6 : 2, 8))) void k_attn_bf16(AttnArgs a, float c) {
  constexpr int NR = A + 1 + D + S;             // ring depth in chunks: look-back, current, in flight, spare
  constexpr int R = NR * C;                     // ring slots
  constexpr int IPC = C * 2 * kRingRowBytes / 1024;   // DMA instructions per chunk (1 KiB each)
  constexpr int TB = kTokBatchChunks * C;       // tokens per batch
  static_assert(C % 8 == 0 && TB % 64 == 0, "chunk shape");
  static_assert((D - 1) * IPC < 64, "prefetch depth exceeds the vmcnt range");
  static_assert(D <= kTokBatchChunks, "token batches must land before their chunks are issued");
  // statically sized, so that ring addresses fold into the DS instructions' offset fields
  __shared__ __align__(1024) unsigned char smem[2 * R * kRingRowBytes + 2 * TB * sizeof(int32_t) + 64];
  unsigned char* const Kring = smem;
  unsigned char* const Vring = smem + R * kRingRowBytes;
  int32_t* const tokring = (int32_t*)(smem + 2 * R * kRingRowBytes);   // 2 batches of TB tokens
  int32_t* const progress = tokring + 2 * TB;   // [NW] phase each compute wave has reached
  int32_t* const landed = progress + 8;         // number of chunks that are in the ring

  // workgroup i runs on XCD i % 8: keep all groups of one (batch, head) on one XCD so
  // that its K/V are fetched into a single L2
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int bh = (seq / a.n_groups) * 8 + xcd, grp = seq % a.n_groups;
  if (bh >= a.B * a.H) return;
  const int b = bh / a.H, h = bh % a.H;
  if (!plan_usable(a.hdr)) return;
  const int grp_g = grp + (a.head_map ? a.head_map[h] * a.n_groups : 0);   // the head group's copy of the work-list
  const GroupDesc gd = a.groups[grp_g];
  const bool shared = a.cfg_share && a.cfg_share[h * a.n_scales + gd.k];
  if (shared && b >= a.B / 2) return;      // the conditional workgroup writes this row

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int P = gd.n_phases;
  if (tid < 16) progress[tid] = 0;             // progress[0..7], landed (and padding)
  __syncthreads();

  if (wave == NW) {
    // ---------------- loader wave ----------------
    const unsigned char* Kp = (const unsigned char*)((const __bf16*)a.k + b * a.ks[0] + h * a.ks[1]);
    const unsigned char* Vp = (const unsigned char*)((const __bf16*)a.v + b * a.ks[0] + h * a.ks[1]);
    const unsigned row_bytes = (unsigned)a.ks[2] * 2u;   // the API checks that a (batch, head) slab
                                                         // spans less than 2 GiB
    const int32_t* utok = a.union_tok + gd.union_base;
    const int n_tok = P * C;
    const int row8 = lane >> 3, pos = lane & 7;

    auto issue_tokens = [&](int batch) {       // TB tokens -> half (batch & 1) of the token ring
#pragma unroll
      for (int i = 0; i < TB / 64; ++i) {
        int t = batch * TB + i * 64 + lane;
        t = t < n_tok ? t : n_tok - 1;
        __builtin_amdgcn_global_load_lds((global_void*)(utok + t),
                                         (lds_void*)(tokring + (batch & 1) * TB + i * 64), 4, 0, 0);
      }
    };
    auto issue_chunk = [&](int chunk) {        // C keys -> ring slots (chunk % NR) * C ...
      const int ring0 = (chunk % NR) * C;
      int tok[C / 8];
      lds_read_tokens<C / 8>(tokring + (chunk % (2 * kTokBatchChunks)) * C + row8, tok);
#pragma unroll
      for (int i = 0; i < C / 8; ++i) {
        const int slot = ring0 + 8 * i + row8;
        const unsigned src = (unsigned)checked_index(a.hdr, tok[i], a.kv_len) * row_bytes + ((pos ^ ring_swizzle(slot)) << 4);
        __builtin_amdgcn_global_load_lds((global_void*)(Kp + src),
                                         (lds_void*)(Kring + (ring0 + 8 * i) * kRingRowBytes), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((global_void*)(Vp + src),
                                         (lds_void*)(Vring + (ring0 + 8 * i) * kRingRowBytes), 16, 0, 0);
      }
    };

    issue_tokens(0);
    if (P > kTokBatchChunks) issue_tokens(1);
    wait_vmcnt<0>();                           // the first token batches are needed right away
#pragma unroll
    for (int d = 0; d < D; ++d)
      if (d < P) issue_chunk(d);
    for (int ph = 0; ph < P; ++ph) {
      // chunk ph has landed once at most the D-1 younger chunks are outstanding
      if (ph + D <= P) wait_vmcnt<(D - 1) * IPC>(); else wait_vmcnt<0>();
      if (lane == 0) lds_store_i32_nowait(landed, ph + 1);
      const int nc = ph + D;
      if (nc < P) {
        // chunk nc reuses the slot of chunk nc - NR, which steps of phases up to
        // nc - NR + A may still read: wait until every compute wave is past them.  The wait
        // is bounded: when it runs out (a plan that does not fit this kernel) the loader
        // stops loading, marks the plan's header, lets every compute wave run to its end on
        // whatever the ring holds, and exits like any other wave.
        const int need = nc - NR + A + 1;
        if (need > 0) {
          int polls = 0;
          bool gave_up = false;
          while (lds_min_progress<NW>(progress) < need) {
            if (++polls > a.spin_limit) { gave_up = true; break; }
            __builtin_amdgcn_s_sleep(1);
          }
          if (gave_up) {
            wait_vmcnt<0>();
            if (lane == 0) {
              lds_store_i32_nowait(landed, 0x7fffffff);
              a.hdr->error = kErrWaitGaveUp;
            }
            return;
          }
        }
        // token batch nb serves chunks [T nb, T nb + T), T = kTokBatchChunks.  It is issued
        // together with chunk T (nb - 1): every chunk of batch nb - 2 (same half of the token
        // ring) has been issued by then, and the batch has landed before chunk T nb is issued
        // because D <= T.
        const int nb = nc / kTokBatchChunks + 1;
        if (nc % kTokBatchChunks == 0 && nb >= 2 && nb * kTokBatchChunks < P) issue_tokens(nb);
        issue_chunk(nc);
      }
    }
    return;
  }

  // ---------------- compute waves ----------------
  const int n = lane & 15, g4 = lane >> 4;
  const WaveDesc wd = a.waves[grp_g * NW + wave];
  const int n_steps = __builtin_amdgcn_readfirstlane(wd.n_steps);

  // Q^T as the B operand: lane (n, g4) holds Q[query n][16*g4 .. 16*g4+15]
  const int dy = n >> 2, dx = n & 3;
  const int qrow = ((wd.valid >> n) & 1u) ? checked_index(a.hdr, wd.q_base + dy * wd.sk + dx, a.q_len) : -1;
  bf16x8 qb0, qb1;
  {
    uint4 z = {0, 0, 0, 0}, q0 = z, q1 = z;
    if (qrow >= 0) {
      const __bf16* qp = (const __bf16*)a.q + b * a.qs[0] + h * a.qs[1] + qrow * a.qs[2] + 16 * g4;
      q0 = *(const uint4*)qp; q1 = *(const uint4*)(qp + 8);
    }
    qb0 = as_bf16x8(q0); qb1 = as_bf16x8(q1);
  }

  // Softmax state per lane (one query column): running reference m (not necessarily the
  // exact maximum, see below), O^T accumulators, and the row sum l, which is accumulated
  // by a fifth MFMA whose A operand is all ones (every row of Lacc holds the same sum of
  // the bf16-rounded probabilities of this query, over all four lane groups).
  float negm = 0.f, thr = kFloor;   // -m, and how far a score may rise above m before m moves (kFloor: m unset)
  f32x4 O[4], Lacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  // The reference m only moves when a score exceeds it by more than kSlack in the base-2
  // exponent (and once at the query's first kept key), so probabilities stay below 2^kSlack
  // and the accumulators are rescaled rarely.
  const float slack = kSlack / c;

  // scalar loads (constant address space) for the wave-uniform tables
  const const_i32_ptr pe = (const_i32_ptr)(a.phase_end + gd.phase_base + wave * P);
  const int64_t step0 = __builtin_amdgcn_readfirstlane(wd.step_begin);
  const uint2* addrs = a.step_addr + step0 * 64 + lane;
  const uint64_t* masks = a.step_mask + step0 * 8;

  // One step: 32 keys against the 16 queries.  `cur` is the lane's descriptor of step s
  // (ring byte offsets of its K rows and V reads); it is replaced by that of step
  // s + kAhead, so that descriptor loads run kAhead steps ahead of their use (one step is
  // shorter than an L2 hit).
  // The prefetch is unconditional (clamped to the wave's last step) so that the number of
  // loads in flight is the same on every path and the wait before `cur` is used can leave
  // the kAhead - 1 younger ones outstanding.
  const int last_step = n_steps - 1;
  auto run_step = [&](uint2& desc, int s, auto prefetch) {
    const uint2 cur = desc;
    if constexpr (decltype(prefetch)::value) desc = addrs[(int64_t)min(s + kAhead, last_step) * 64];
    const const_u64_ptr mk = (const_u64_ptr)(masks + (int64_t)s * 8);

    // S^T tiles: keys x queries
    constexpr int kRingBytes = R * kRingRowBytes;
    const unsigned ka0 = checked_index(a.hdr, cur.x & 0xffffu, kRingBytes), ka1 = checked_index(a.hdr, cur.x >> 16, kRingBytes);
    const bf16x8 k00 = as_bf16x8(*(const uint4*)(Kring + ka0));
    const bf16x8 k01 = as_bf16x8(*(const uint4*)(Kring + (ka0 ^ 16u)));
    const bf16x8 k10 = as_bf16x8(*(const uint4*)(Kring + ka1));
    const bf16x8 k11 = as_bf16x8(*(const uint4*)(Kring + (ka1 ^ 16u)));
    // accumulators start at -m where the pair is kept and at -inf where it is not
    f32x4 S0, S1;
#pragma unroll
    for (int e = 0; e < 4; ++e) { S0[e] = mask_select(negm, mk[e]); S1[e] = mask_select(negm, mk[4 + e]); }
    S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k00, qb0, S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k10, qb0, S1, 0, 0, 0);
    S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k01, qb1, S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k11, qb1, S1, 0, 0, 0);

    // V^T operand: transposing LDS reads, 4 keys x 16 dims per 16-lane block
    const unsigned v0 = checked_index(a.hdr, cur.y & 0xffffu, kRingBytes), v1 = checked_index(a.hdr, cur.y >> 16, kRingBytes);
    s16x4 va[4][2];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      va[dt][0] = lds_read_tr16(Vring + (v0 ^ (unsigned)(dt << 5)));
      va[dt][1] = lds_read_tr16(Vring + (v1 ^ (unsigned)(dt << 5)));
    }

    float sv[8] = {S0[0], S0[1], S0[2], S0[3], S1[0], S1[1], S1[2], S1[3]};
    const float m012 = fmaxf(fmaxf(sv[0], sv[1]), sv[2]), m345 = fmaxf(fmaxf(sv[3], sv[4]), sv[5]);   // (v_max3)
    const float mx = fmaxf(fmaxf(fmaxf(sv[6], sv[7]), m012), m345);
    // the maximum over the query's four lanes is formed only when some lane crossed its threshold
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(mx > thr) != 0, 0)) {      // rare after the first steps
      const float mxr = max_across_rows(mx);
      const bool grow = mxr > thr;
      const float shift = grow ? mxr : 0.f;               // m moves by this much (down only when m was unset)
      const float alpha = __builtin_amdgcn_exp2f(-fmaxf(shift, 0.f) * c);
      negm -= shift;
      thr = grow ? slack : thr;
#pragma unroll
      for (int e = 0; e < 8; ++e) sv[e] -= shift;
      Lacc *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) O[dt] *= alpha;
    }
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(sv[e] * c);

    bf16x8 pb;
#pragma unroll
    for (int e = 0; e < 8; ++e) pb[e] = (__bf16)p[e];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      s16x8 v8 = {va[dt][0][0], va[dt][0][1], va[dt][0][2], va[dt][0][3],
                  va[dt][1][0], va[dt][1][1], va[dt][1][2], va[dt][1][3]};
      O[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v8), pb, O[dt], 0, 0, 0);
    }
    Lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb, Lacc, 0, 0, 0);
  };

  uint2 ad[kAhead];
#pragma unroll
  for (int i = 0; i < kAhead; ++i) ad[i] = addrs[(int64_t)max(min(i, last_step), 0) * 64];

  // steps are listed in phase order; pe[ph] = number of steps runnable once chunk ph is in
  // (flag accesses in inline assembly: a volatile access would also wait for the wave's
  // outstanding descriptor prefetches)
  int32_t* const my_progress = progress + wave;
  bool gave_up = false;                        // a wait of this wave ran out: it waits no more
  auto enter_phase = [&](int ph) {             // all steps of earlier phases are done
    if (lane == 0) lds_store_i32_nowait(my_progress, ph);
    int polls = 0;
    while (!gave_up && lds_load_i32_nowait(landed) <= ph) {
      if (++polls > a.spin_limit) {            // (bounded: the loader may have stopped)
        gave_up = true;
        if (lane == 0) a.hdr->error = kErrWaitGaveUp;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  };
  int ph = 0;
  if (n_steps > 0) {
    enter_phase(0);
    int end = pe[0];
    auto advance_to = [&](int s) {             // wait until step s may run
      if (s >= end) {
        do { ++ph; end = pe[ph]; } while (s >= end && ph + 1 < P);   // (the table's last entry covers every step)
        enter_phase(ph);
      }
    };
    int s0 = 0;
    for (; s0 + kAhead <= n_steps; s0 += kAhead) {
#pragma unroll
      for (int i = 0; i < kAhead; ++i) {
        advance_to(s0 + i);
        run_step(ad[i], s0 + i, std::true_type{});
      }
    }
#pragma unroll
    for (int i = 0; i < kAhead - 1; ++i) {
      if (s0 + i < n_steps) {
        advance_to(s0 + i);
        run_step(ad[i], s0 + i, std::false_type{});
      }
    }
  }
  // every LDS read of this wave has returned (its results fed the MFMAs above)
  if (lane == 0) lds_store_i32_nowait(my_progress, P);

  if (qrow < 0) return;
  const float inv = 1.f / Lacc[0];
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

template <int NW, int C, int A, int D, int S>
static litevar_status launch(const AttnArgs& a, hipStream_t st) {
  const int64_t bh8 = ((int64_t)a.B * a.H + 7) / 8 * 8;
  const int64_t blocks = bh8 * a.n_groups;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  const float c = a.sm_scale * 1.4426950408889634f;
  hipLaunchKernelGGL((k_attn_bf16<NW, C, A, D, S>), dim3((unsigned)blocks), dim3((NW + 1) * 64), 0, st, a, c);
  return hip_check(hipGetLastError(), "bf16 attention launch");
}

litevar_status launch_attn_bf16(const litevar_plan* pl, const AttnArgs& a, hipStream_t st) {
  const int nw = pl->waves_per_group, C = pl->chunk_keys, NR = pl->ring_chunks;
  if (nw == 16) return launch_attn_bf16_pair(pl, a, st);
  const int D = pl->prefetch_chunks, S = NR - 2 - D;
  const int key = nw * 10000 + C * 100 + D * 10 + S;
  switch (key) {
#define LV_CASE(nw_, c_, d_, s_) case nw_ * 10000 + c_ * 100 + d_ * 10 + s_: return launch<nw_, c_, 1, d_, s_>(a, st);
    LV_CASE(8, 32, 2, 2) LV_CASE(8, 64, 2, 1)
    LV_CASE(4, 32, 2, 2) LV_CASE(4, 64, 2, 1)
#undef LV_CASE
    default: break;
  }
  return fail(LITEVAR_E_PLAN_CORRUPT, "no kernel for waves=%d chunk=%d ring=%d", nw, C, NR);
}

}  // namespace lv
