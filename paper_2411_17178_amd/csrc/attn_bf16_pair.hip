// bf16 windowed attention forward for gfx950 (CDNA4), Section 2 of the paper, for plans
// with 16 patches per group: O = softmax(sm_scale * Q K^T over the kept keys) V, with the
// Section 3 cond -> uncond output reuse folded into the store.
//
// One workgroup = eight waves = one group of up to 16 query patches (16 x 16 queries of
// one scale) of one (batch, head).  Every wave owns two patches (a top and a bottom one,
// so that it has keys in most parts of the stream) and one eighth of the loading.
//
// The group's key list is streamed once through an LDS ring of five chunks of 64 keys
// (one 128-byte K row and one 128-byte V row per key, 16-byte pieces XOR-swizzled by
// slot; 80 KiB, so that two workgroups share a CU); chunk t lives in slot t mod 5.  The
// plan counts NC chunks; the kernel runs P = NC / 2 + 1 phases: phase 0 is chunk 0 alone
// (the first steps start on as little data as possible), phase p >= 1 is chunks 2p-1 and
// 2p, i.e. the steps whose last key lies in one of them.  A step spans at most two
// consecutive chunks, so a step that ends in chunk t reads chunks t-1 .. t: phase p reads
// chunks 2p-2 .. 2p, which are three of the five slots; the other two slots held chunks
// 2p-4 and 2p-3, which nobody reads after the barrier that ended phase p-1, and receive
// chunks 2p+1 and 2p+2 (phase p+1) while phase p computes.
//   Prologue: all scalar plan words, then Q, the first step descriptors and the other small
//     loads, then chunks 0, 1 and 2.  (Where the list does not start with whole key scales,
//     the tokens of the chunks that need them travel with the small loads; the chunks that
//     need none go out meanwhile, one wait, then the rest.)  With at most the three chunks
//     outstanding (a wave issues PW transfers per chunk: vmcnt 3 PW) Q is in; with at most
//     chunks 1 and 2 outstanding (vmcnt 2 PW) comes the first barrier: chunk 0 is in.
//   Phase p: a wave
//     issues the descriptor loads of its steps of this phase beyond the first of each patch,
//     runs the first step of each patch,
//     waits for all its vector memory operations (p >= 1: the descriptors just requested;
//       chunks 2p-1 and 2p were waited for at the end of phase p-1),
//     requests the first descriptors and the tokens of phase p+1 and then issues its share
//       of chunks 2p+1 and 2p+2 (p >= 1; in phase 0 chunks 1 and 2 are already in flight) --
//       not right behind the barrier, where the loads of all eight waves would queue up in
//       front of the first K reads, and behind the small loads, because a load issued behind
//       a chunk is held up until the chunk's data is in,
//     runs its other steps, waits for all its vector memory operations (vmcnt 0: the chunks
//       of phase p+1 have landed) and joins the barrier.
// Two chunks (32 KiB) per workgroup are in flight during a phase, and a key row is moved
// from HBM/L2 to LDS exactly once per (batch, head, group).
//
// A wave that issues LDS-DMA loads must read LDS through inline assembly: the compiler
// cannot tell which of them a plain LDS read depends on and would wait for all
// (vmcnt(0)) before every read.
//
// Step arithmetic is that of the 8-patch kernel: S^T = K_tile . Q^T by
// v_mfma_f32_16x16x32_bf16 (a lane owns one query column and four keys per tile) on
// accumulators that start at minus the softmax reference where the scalar lane mask keeps the
// pair and at -inf elsewhere (one v_cndmask per score), so the tiles leave the matrix pipe as
// masked scores relative to the reference; base-2 online softmax with a lazily updated
// reference, O^T += V^T . P^T with ds_read_b64_tr_b16 operands, row sums by a fifth MFMA.
// (Folding the softmax scale into Q, which would save the multiplication per score, costs a
// second bf16 rounding of Q: with peaked attention -- scores of some tens -- the output
// error grows tenfold.  The scale is applied in fp32.)
#include <type_traits>

#include "attn_bf16_common.h"

namespace lv {

namespace {

constexpr int kGroupPatches = 16;     // query patches per workgroup
constexpr int kDmaKeys = 64;          // keys per chunk (the unit of loading and of ring slot reuse)
constexpr int kRingChunks = 5;        // ring depth: look-back, two current, two landing
constexpr int kBufferFlags = 0x00020000;   // word 3 of a raw buffer resource on gfx9: 32-bit data format
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int kBoostPhases = 3;       // phases that a later-arrived workgroup runs at raised priority
constexpr int kLater = 2;             // descriptors per patch, beyond the first step of a phase, that are
                                      // fetched at the start of the phase

__device__ inline unsigned lds_addr(const void* p) {
  return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// four 16-byte K pieces (two keys x two halves of the head dimension): issued only,
// lds_wait_k() must precede the first use
__device__ inline void lds_read_k_issue(unsigned a0, unsigned a1, u32x4& k00, u32x4& k01, u32x4& k10, u32x4& k11) {
  asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\t"
               "ds_read_b128 %2, %6\n\tds_read_b128 %3, %7"
               : "=&v"(k00), "=&v"(k01), "=&v"(k10), "=&v"(k11)
               : "v"(a0), "v"(a0 ^ 16u), "v"(a1), "v"(a1 ^ 16u) : "memory");
}

__device__ inline void lds_wait_k(u32x4& k00, u32x4& k01, u32x4& k10, u32x4& k11) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(k00), "+v"(k01), "+v"(k10), "+v"(k11) : : "memory");
}

// transposing reads of the V^T operands of one step (4 head-dim tiles x 2 key halves);
// issued only: lds_wait() must precede the first use
template <int VOFF>
__device__ inline void lds_read_v(unsigned v0, unsigned v1, const unsigned (&x)[3][2], uint2 (&va)[4][2]) {
  asm volatile("ds_read_b64_tr_b16 %0, %8 offset:%16\n\tds_read_b64_tr_b16 %1, %9 offset:%16\n\t"
               "ds_read_b64_tr_b16 %2, %10 offset:%16\n\tds_read_b64_tr_b16 %3, %11 offset:%16\n\t"
               "ds_read_b64_tr_b16 %4, %12 offset:%16\n\tds_read_b64_tr_b16 %5, %13 offset:%16\n\t"
               "ds_read_b64_tr_b16 %6, %14 offset:%16\n\tds_read_b64_tr_b16 %7, %15 offset:%16"
               : "=&v"(va[0][0]), "=&v"(va[0][1]), "=&v"(va[1][0]), "=&v"(va[1][1]),
                 "=&v"(va[2][0]), "=&v"(va[2][1]), "=&v"(va[3][0]), "=&v"(va[3][1])
               : "v"(v0), "v"(v1), "v"(x[0][0]), "v"(x[0][1]), "v"(x[1][0]), "v"(x[1][1]),
                 "v"(x[2][0]), "v"(x[2][1]), "i"(VOFF) : "memory");
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
  float thr, negm;        // minus the softmax reference m; thr = how far a score may rise above m
                          // before m moves: kFloor while m is unset
};

}  // namespace

// PW = query patches per wave: 2 (8 waves per workgroup, two workgroups per CU: the form for
// launches that fill the GPU) or 1 (16 waves per workgroup, one workgroup per CU: a launch with
// no more workgroups than CUs then still has four waves on every SIMD).  Same plan, same
// phases; with 16 waves the loading duty of a chunk is one K or one V transfer per wave.
//
// Q8 (Section 4, 8-bit Q, K, V): the operands are int8 codes with one (scale, zero point) per
// token row.  A wave's share of a chunk then comes through registers instead of LDS-DMA: one
// 16-byte load of codes and one of the row's parameters per lane (lanes 0-31 K rows, lanes
// 32-63 V rows with eight waves; K waves and V waves with sixteen), requested where the bf16
// form issues its transfers, converted to bf16(s code + z) and written to the ring -- same
// slots, same swizzle -- at the end of the phase, before the barrier.  Steps, masks and
// epilogue are the same code; the ring holds exactly what a dequantised bf16 copy would put
// there, so the results equal those of the bf16 kernel on such a copy bit for bit.
template <int PW, bool Q8>
__global__ __launch_bounds__((kGroupPatches / PW) * 64) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_attn_bf16_pair(AttnArgs a, float c) {
  [[maybe_unused]] constexpr int NWV = kGroupPatches / PW;   // waves per workgroup
  constexpr int C = kDmaKeys;
  constexpr int R = kRingChunks * C;               // ring slots
  constexpr int VOFF = R * kRingRowBytes;          // V ring follows the K ring
  __shared__ __align__(1024) unsigned char smem[2 * R * kRingRowBytes];
  unsigned char* const Kring = smem;
  unsigned char* const Vring = smem + VOFF;

  // workgroup i runs on XCD i % 8: all groups of one (batch, head) share one L2
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  int me, grp, b, h;                      // me: which of the (batch, head) pairs of this XCD
  divmod_by((uint32_t)seq, (uint32_t)a.n_groups, a.n_groups_magic, me, grp);
  const int bh = me * 8 + xcd;
  if (bh >= a.B * a.H) return;
  divmod_by((uint32_t)bh, (uint32_t)a.H, a.H_magic, b, h);
  // Scalar round trip 1: the header words that say whether the plan may be used at all (a
  // zeroed, stale or half-built blob makes the launch a no-op) and, for plans with a radius
  // table per head, the head's group, whose copy of the work-list this workgroup walks.
  // (Requested together and tied to one point, so that they cost one round trip, not four.)
  const const_i32_ptr hw = (const_i32_ptr)a.hdr;
  int magic_lo = hw[0], magic_hi = hw[1], herr = hw[offsetof(Header, error) / 4], hg = 0;
  if (a.head_map) hg = ((const_i32_ptr)a.head_map)[h];
  asm volatile("" : "+s"(magic_lo), "+s"(magic_hi), "+s"(herr), "+s"(hg));
  if (magic_lo != (int32_t)(kMagic & 0xffffffffu) || magic_hi != (int32_t)(kMagic >> 32) || herr == kErrBuilder) return;
  const int grp_g = grp + hg * a.n_groups;
  // Scalar round trip 2 (together with the patch descriptors below): the group descriptor.
  const const_i32_ptr gw = (const_i32_ptr)(a.groups + grp_g);
  GroupDesc gd;
  gd.union_base = gw[0]; gd.n_union = gw[1]; gd.n_phases = gw[2]; gd.k = gw[3];
  gd.gy = gw[4]; gd.gx = gw[5]; gd.phase_base = gw[6]; gd.ident = gw[7];

  // Two workgroups share a CU, and the instruction arbiter prefers the older waves: left
  // alone, the workgroup that arrived first runs as if it had the CU to itself and the other
  // one finishes a quarter later, alone on a CU that it cannot fill.  The later arrival (it
  // gets the higher wave slots of each SIMD) therefore runs at raised priority through its
  // first phases, which evens out the two finishing times.
  const bool later_arrival = PW == 2 && (__builtin_amdgcn_s_getreg(4 | (3 << 11)) & 0xf) >= 2;   // HW_ID.WAVE_ID
  if (later_arrival) __builtin_amdgcn_s_setprio(1);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n = lane & 15, g4 = lane >> 4;
  // The plan counts 64-key chunks.  Phase 0 is chunk 0 alone, so that the first steps start
  // on the smallest possible amount of data; phase p >= 1 is chunks 2 p - 1 and 2 p.
  const int NC = __builtin_amdgcn_readfirstlane(gd.n_phases);   // chunks of the (padded) key list
  const int P = NC / 2 + 1;                                     // phases

  // ---- loading duty: rows [8 w, 8 w + 8) of every chunk, w = wave mod 8: K and V rows with
  // eight waves, K rows (waves 0-7) or V rows (waves 8-15) with sixteen ----
  constexpr int kElem = Q8 ? 1 : 2;                    // bytes per operand element
  const unsigned char* Kp = (const unsigned char*)a.k + (b * a.ks[0] + h * a.ks[1]) * kElem;
  const unsigned char* Vp = (const unsigned char*)a.v + (b * a.ks[0] + h * a.ks[1]) * kElem;
  const unsigned row_bytes = (unsigned)a.ks[2] * kElem;   // a (batch, head) slab spans < 2 GiB (checked by the API)
  const int32_t* utok = a.union_tok + gd.union_base;
  const int ident = __builtin_amdgcn_readfirstlane(gd.ident);   // union entries [0, ident) are token i at position i
  // bf16: eight lanes per 128-byte row; Q8: four lanes per 64-byte row of codes
  const int row = Q8 ? 8 * (wave & 7) + ((lane >> 2) & 7) : 8 * (wave & 7) + (lane >> 3);
  // A lane's row of chunk t goes to slot (t % 5) * 64 + row.  Chunks start at multiples of 64
  // slots, so the slot's swizzle -- and with it the 16-byte piece of the source row that
  // this lane fetches -- does not depend on t.
  const unsigned piece_off = (((unsigned)lane & 7u) ^ ring_swizzle((unsigned)row)) << 4;
  static_assert((kDmaKeys & 63) == 0, "the swizzle folds slot bits 0..5 only");
  auto issue_chunk = [&](int t, int tok) {             // chunk t -> ring slots (t % 5) * 64 ...
    tok = checked_index(a.hdr, tok, a.kv_len);
    const int slot0 = (t % kRingChunks) * C + 8 * (wave & 7);
    const unsigned src = __umul24((unsigned)tok, row_bytes) + piece_off;   // (both below 2^24, checked by the API)
    if (PW == 2 || wave < 8)
      __builtin_amdgcn_global_load_lds((global_void*)(Kp + src), (lds_void*)(Kring + slot0 * kRingRowBytes), 16, 0, 0);
    if (PW == 2 || wave >= 8)
      __builtin_amdgcn_global_load_lds((global_void*)(Vp + src), (lds_void*)(Vring + slot0 * kRingRowBytes), 16, 0, 0);
  };
  constexpr int kDmaPerChunk = PW;                       // transfers that a wave issues per chunk
  // Q8: this lane's share of a chunk on its way through registers
  struct ChunkRegs { u32x4 codes; float2 sz; };
  const bool q8_v = PW == 2 ? lane >= 32 : wave >= 8;     // the lane works on V rows (else K rows)
  const bool q8_active = PW == 2 || lane < 32;
  [[maybe_unused]] auto load_chunk = [&](int tok) -> ChunkRegs {
    ChunkRegs r;
    r.codes = u32x4{0u, 0u, 0u, 0u}; r.sz = make_float2(0.f, 0.f);
    if (q8_active) {
      tok = checked_index(a.hdr, tok, a.kv_len);
      const unsigned char* base = q8_v ? Vp : Kp;
      const float2* sz = (q8_v ? a.v_sz : a.k_sz) + (int64_t)(b * a.H + h) * (a.ks[1] / a.ks[2]);
      r.codes = *(const u32x4*)(base + __umul24((unsigned)tok, row_bytes) + 16u * ((unsigned)lane & 3u));
      r.sz = sz[tok];
    }
    return r;
  };
  [[maybe_unused]] auto commit_chunk = [&](int t, const ChunkRegs& r) {   // chunk t -> ring slots (t % 5) * 64 ...
    if (!q8_active) return;
    const unsigned slot = (unsigned)((t % kRingChunks) * C + row);
    const unsigned sw = ring_swizzle((unsigned)row), p2 = 2u * ((unsigned)lane & 3u);
    unsigned char* dst = (q8_v ? Vring : Kring) + slot * kRingRowBytes;
    bf16x8 lo, hi;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int8_t c0 = (int8_t)((r.codes[e >> 2] >> (8 * (e & 3))) & 0xffu);
      const int8_t c1 = (int8_t)((r.codes[2 + (e >> 2)] >> (8 * (e & 3))) & 0xffu);
      lo[e] = (__bf16)fmaf(r.sz.x, (float)c0, r.sz.y);
      hi[e] = (__bf16)fmaf(r.sz.x, (float)c1, r.sz.y);
    }
    *(bf16x8*)(dst + ((p2 ^ sw) << 4)) = lo;
    *(bf16x8*)(dst + (((p2 + 1u) ^ sw) << 4)) = hi;
  };  // (tokens and descriptors through buffer loads: a scalar resource and a scalar offset plus a
  // lane offset register, where a flat address costs 64-bit vector arithmetic per load)
  const __amdgpu_buffer_rsrc_t tok_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)utok, 0, NC * C * 4, kBufferFlags);
  // this lane's row of chunk t (clamped to the last chunk): load_tok() fetches the list entry
  // unless the whole chunk lies in the identity prefix, tok_of() applied to its result at the
  // time of use (when the load has been waited for) gives the token
  auto load_tok = [&](int t) -> int {
    const int tc = min(t, NC - 1);
    if ((tc + 1) * C <= ident) return 0;               // (uniform)
    return (int)__builtin_amdgcn_raw_buffer_load_b32(tok_rsrc, row * 4, tc * C * 4, 0);
  };
  auto tok_of = [&](int t, int loaded) -> int {
    const int i = min(t, NC - 1) * C + row;
    return i < ident ? i : loaded;
  };

  // ---- prologue, scalar part.  Everything that comes through scalar loads (patch
  // descriptors, phase tables, the extent of the group's steps) is fetched before the first
  // vector memory operation: behind the burst of first chunks of all workgroups a scalar
  // miss would take microseconds, and the vector loads below depend on these values.
  // Patch descriptor words: {step_begin, n_steps, q_base, sk | ny << 16, nx | kq << 16, pairs, valid, first_ends}
  // (two patches per wave: p and its partner two patch rows below, columns swapped)
  const int pa = wave, pb_ = PW == 2 ? ((wave >> 2) + 2) * 4 + ((wave & 3) ^ 1) : wave;
  const const_i32_ptr wA = (const_i32_ptr)(a.waves + grp_g * 16 + pa), wB = (const_i32_ptr)(a.waves + grp_g * 16 + pb_);
  const const_i32_ptr wF = (const_i32_ptr)(a.waves + grp_g * 16), wL = (const_i32_ptr)(a.waves + grp_g * 16 + 15);
  const const_i32_ptr peA = (const_i32_ptr)(a.phase_end + gd.phase_base + pa * NC);
  const const_i32_ptr peB = (const_i32_ptr)(a.phase_end + gd.phase_base + pb_ * NC);
  auto last_chunk = [&](int ph) -> int { return min(2 * ph, NC - 1); };   // of phase ph (clamped)
  struct PatchWords { int step_begin, q_base, sk_ny, valid; };
  const PatchWords pwA = {wA[0], wA[2], wA[3], wA[6]}, pwB = {wB[0], wB[2], wB[3], wB[6]};
  const int first_step = wF[0], n_group_steps = wL[0] + wL[1] - first_step;
  const int lastA = max(wA[1] - 1, 0), lastB = max(wB[1] - 1, 0);     // last step of each patch
  // cumulative step counts of phases 0 and 1 (an idle patch has zeros); the entry of
  // phase p + 2 is fetched during phase p
  // (one patch per wave: the second patch's counts are the constant 0 and its code goes away)
  // (those of phases 0 and 1 sit in the patch descriptor, so that nothing the first vector
  // loads depend on waits for a second round of scalar loads behind the group descriptor)
  const unsigned feA = (unsigned)wA[7], feB = PW == 2 ? (unsigned)wB[7] : 0u;
  int endA = (int)(feA & 0xffffu), endB = (int)(feB & 0xffffu);
  int end1A = (int)(feA >> 16), end1B = (int)(feB >> 16);
  asm volatile("" : : "s"(pwA.step_begin), "s"(pwA.q_base), "s"(pwA.sk_ny), "s"(pwA.valid),
               "s"(pwB.step_begin), "s"(pwB.q_base), "s"(pwB.sk_ny), "s"(pwB.valid),
               "s"(n_group_steps), "s"(endA), "s"(endB), "s"(end1A), "s"(end1B), "s"(lastA), "s"(lastB),
               "s"(gd.union_base), "s"(gd.n_phases), "s"(gd.k), "s"(gd.phase_base), "s"(gd.ident));   // all in
  // Scalar round trip 3, only with an output sharing table: the flag of (head, query scale),
  // as the aligned word that holds the byte (a naturally aligned word lies in its byte's page).
  bool shared = false;
  if (a.cfg_share) {
    const uintptr_t sa = (uintptr_t)(a.cfg_share + h * a.n_scales + gd.k);
    const uint32_t share_word = (uint32_t)*(const_i32_ptr)(sa & ~(uintptr_t)3);
    shared = ((share_word >> (8u * (uint32_t)(sa & 3))) & 0xffu) != 0;
  }
  if (shared && b >= a.B / 2) return;      // the conditional workgroup writes this row

  // ---- prologue, vector part.  The key list usually starts with whole key scales (token =
  // position), which needs no token load; the tokens of the other chunks among the first
  // three are requested here and waited for together with the small loads below.
  // leading chunks (of the first three) that lie in the identity prefix: their transfers need no token
  auto in_prefix = [&](int t) -> bool { return (min(t, NC - 1) + 1) * C <= ident; };
  const int n_id = (int)in_prefix(0) + (int)in_prefix(1) + (int)in_prefix(2);   // (uniform; non-increasing in t)

  const int64_t sbA = pwA.step_begin, sbB = pwB.step_begin;
  const __amdgpu_buffer_rsrc_t descA = __builtin_amdgcn_make_buffer_rsrc((void*)(a.step_addr + sbA * 64), 0, (lastA + 1) * 512, kBufferFlags);
  const __amdgpu_buffer_rsrc_t descB = __builtin_amdgcn_make_buffer_rsrc((void*)(a.step_addr + sbB * 64), 0, (lastB + 1) * 512, kBufferFlags);
  const int lane8 = lane * 8;
  auto load_desc = [&](const __amdgpu_buffer_rsrc_t& rsrc, int s) -> uint2 {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane8, s * 512, 0);
    return make_uint2(v.x, v.y);
  };
  const uint64_t* maskA = a.step_mask + sbA * 8;
  const uint64_t* maskB = a.step_mask + sbB * 8;

  // local query row of this lane's query column (-1 = none)
  auto query_row = [&](const PatchWords& w, int n, bool clamped) -> int {
    const int sk = w.sk_ny & 0xffff;
    const int dy = n >> 2, dx = n & 3;
    const int r = w.q_base + dy * sk + dx;
    if (clamped) return max(min(r, a.q_len - 1), 0);
    return ((w.valid >> n) & 1) ? r : -1;
  };
  // Q rows are loaded unconditionally, from a clamped row where the lane has no query: such
  // a column of S^T holds scores of some other query, all of its mask bits are clear and it
  // is never stored, and MFMA columns do not mix
  auto init_patch = [&](PatchState& ps, const PatchWords& w) {
    const int ld_row = query_row(w, n, true);
    if constexpr (Q8) {
      const int8_t* qp = (const int8_t*)a.q + b * a.qs[0] + h * a.qs[1] + ld_row * a.qs[2] + 16 * g4;
      const u32x4 qc = *(const u32x4*)qp;
      const float2 qz = a.q_sz[(int64_t)(b * a.H + h) * a.q_len + ld_row];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        ps.qb0[e] = (__bf16)fmaf(qz.x, (float)(int8_t)((qc[e >> 2] >> (8 * (e & 3))) & 0xffu), qz.y);
        ps.qb1[e] = (__bf16)fmaf(qz.x, (float)(int8_t)((qc[2 + (e >> 2)] >> (8 * (e & 3))) & 0xffu), qz.y);
      }
    } else {
      const __bf16* qp = (const __bf16*)a.q + b * a.qs[0] + h * a.qs[1] + ld_row * a.qs[2] + 16 * g4;
      // (inline assembly: the compiler then does not know of a load into these registers and
      // places no wait of its own, which would cover the chunk transfers too, before their use)
      u32x4 r0, r1;
      asm volatile("global_load_dwordx4 %0, %2, off\n\tglobal_load_dwordx4 %1, %2, off offset:16"
                   : "=&v"(r0), "=&v"(r1) : "v"(qp) : "memory");
      ps.qb0 = __builtin_bit_cast(bf16x8, r0); ps.qb1 = __builtin_bit_cast(bf16x8, r1);
    }
    ps.thr = kFloor; ps.negm = 0.f;
    ps.Lacc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) ps.O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  PatchState A, B;
  init_patch(A, pwA);
  if constexpr (PW == 2) init_patch(B, pwB);

  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  asm volatile("" : "+v"(ones));     // kept in four registers (the compiler would rebuild it in every step)
  const float slack = kSlack / c;
  // Step descriptors of a patch for one phase: the first step's is fetched during the phase
  // before (d0), those of the next kLater steps at the start of the phase (dl).
  uint2 dA0 = make_uint2(0u, 0u), dB0 = dA0, dAl[kLater], dBl[kLater];
#pragma unroll
  for (int i = 0; i < kLater; ++i) { dAl[i] = dA0; dBl[i] = dA0; }
  // (Every register that a vector load fills is used only behind an explicit wait for all
  // of the wave's loads: with chunks in flight the compiler would otherwise place such a wait,
  // the chunks included, before the use.  That also allows loads under uniform conditions,
  // whose number the compiler cannot know: only the descriptors that the phase needs.)
  auto load_later = [&](uint2 (&d)[kLater], const __amdgpu_buffer_rsrc_t& rsrc, int first, int end) {
#pragma unroll
    for (int i = 0; i < kLater; ++i)
      if (first + 1 + i < end) d[i] = load_desc(rsrc, first + 1 + i);
  };
  dA0 = load_desc(descA, 0);
  if constexpr (PW == 2) dB0 = load_desc(descB, 0);
  int tokn0 = load_tok(3), tokn1 = load_tok(4);         // tokens of the chunks issued in phase 1
  // the later descriptors of phase 0, which has no wait of its own before their use
  load_later(dAl, descA, 0, endA);
  load_later(dBl, descB, 0, endB);
  // All workgroups walk the same plan in lock-step, so each phase's first access to its part
  // of the plan would be an HBM miss on every workgroup's critical path.  The workgroups of
  // one XCD (they share an L2) therefore touch the group's step descriptors and lane masks
  // once, each its own slice of the 128-byte lines, while the first chunks are on their way.
  int warm = 0;
  {
    const char* da = (const char*)(a.step_addr + (int64_t)first_step * 64);
    const char* ma = (const char*)(a.step_mask + (int64_t)first_step * 8);
    // one load per thread: workgroup `me` of this group on this XCD touches the lines
    // [me T, me T + T), T = threads per workgroup (the workgroups beyond the plan's end all
    // touch its last line; with more lines than workgroups x T the rest is touched in part
    // only, which costs nothing but speed)
    const int lines_d = n_group_steps * 4, lines = lines_d + (n_group_steps + 1) / 2;
    const int l = min(me * (int)blockDim.x + tid, lines - 1);
    const char* src = l < lines_d ? da + (int64_t)l * 128 : ma + (int64_t)(l - lines_d) * 128;
    warm = *(const int*)src;
  }
  // The chunks go out behind the small loads (a load issued behind a chunk is held up until
  // the chunk's data is in), chunks 1 and 2 (phase 1) last: phase 0 waits for everything but them.
  if constexpr (Q8) {
    // through registers: the three chunks are requested together, converted and written, and
    // the first barrier finds all of them in the ring
    int tok0 = 0, tok1 = 0, tok2 = 0;
    if (n_id < 3) { tok0 = load_tok(0); tok1 = load_tok(1); tok2 = load_tok(2); }
    const ChunkRegs c0 = load_chunk(tok_of(0, tok0)), c1 = load_chunk(tok_of(1, tok1)), c2 = load_chunk(tok_of(2, tok2));
    commit_chunk(0, c0); commit_chunk(1, c1); commit_chunk(2, c2);
  } else if (n_id == 3) {
    issue_chunk(0, tok_of(0, 0)); issue_chunk(1, tok_of(1, 0)); issue_chunk(2, tok_of(2, 0));
  } else {
    // Some of the three chunks need their tokens: these are requested behind the small loads
    // and travel with them; the chunks of the prefix go out meanwhile; then one wait for
    // everything issued so far.  (All in this branch, so that on the other one the compiler
    // knows of no token load in flight.)
    int tok0 = load_tok(0), tok1 = load_tok(1), tok2 = load_tok(2);
    if (n_id >= 1) issue_chunk(0, tok_of(0, 0));
    if (n_id >= 2) issue_chunk(1, tok_of(1, 0));
    wait_vmcnt<0>();
    asm volatile("" : "+v"(tok0), "+v"(tok1), "+v"(tok2));
    if (n_id < 1) issue_chunk(0, tok_of(0, tok0));
    if (n_id < 2) issue_chunk(1, tok_of(1, tok1));
    issue_chunk(2, tok_of(2, tok2));
  }
  // (Q was loaded through inline assembly: everything older than the three chunks is in once
  // at most their transfers are outstanding, and the registers are tied to that point)
  if constexpr (Q8) {
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // (the ring writes above are visible)
  } else {
    wait_vmcnt<3 * kDmaPerChunk>();
    asm volatile("" : "+v"(A.qb0), "+v"(A.qb1));
    if constexpr (PW == 2) asm volatile("" : "+v"(B.qb0), "+v"(B.qb1));
    wait_vmcnt<2 * kDmaPerChunk>();
    asm volatile("s_barrier" ::: "memory");
  }

  // One step: 32 keys against the 16 queries of patch ps.
  auto run_step = [&](PatchState& ps, const uint2 cur, const uint64_t* masks, int s) {
    // lane masks of the step (a scalar load): requested ahead of the K pieces so that the
    // two latencies overlap
    const const_u64_ptr mkp = (const_u64_ptr)((const char*)masks + (unsigned)s * 64u);
    uint64_t mk[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) mk[e] = mkp[e];
    u32x4 k00, k01, k10, k11;
    constexpr int kRingBytes = R * kRingRowBytes;       // (descriptor offsets are relative to either ring)
    lds_read_k_issue(lds_addr(Kring + checked_index(a.hdr, cur.x & 0xffffu, kRingBytes)),
                     lds_addr(Kring + checked_index(a.hdr, cur.x >> 16, kRingBytes)), k00, k01, k10, k11);
    // addresses of the V^T pieces: computed while the K pieces are on their way
    unsigned v0 = lds_addr(Kring + checked_index(a.hdr, cur.y & 0xffffu, kRingBytes)),
             v1 = lds_addr(Kring + checked_index(a.hdr, cur.y >> 16, kRingBytes));
    unsigned va_addr[3][2];
#pragma unroll
    for (int dt = 1; dt < 4; ++dt) { va_addr[dt - 1][0] = v0 ^ (32u * dt); va_addr[dt - 1][1] = v1 ^ (32u * dt); }
    asm volatile("" : "+v"(v0), "+v"(v1), "+v"(va_addr[0][0]), "+v"(va_addr[0][1]), "+v"(va_addr[1][0]),
                 "+v"(va_addr[1][1]), "+v"(va_addr[2][0]), "+v"(va_addr[2][1]));
    lds_wait_k(k00, k01, k10, k11);
    // (the masks were requested before the K pieces and share their counter: they are in,
    // and the compiler should know before the V^T reads go out, or it waits for those too)
    asm volatile("" : : "s"(mk[0]), "s"(mk[1]), "s"(mk[2]), "s"(mk[3]), "s"(mk[4]), "s"(mk[5]), "s"(mk[6]), "s"(mk[7]));
    // The accumulators of the score tiles start at -m where the pair is kept and at -inf
    // where it is not (one v_cndmask per score, by the lane masks, off the path that waits
    // for the matrix pipe): the tiles come out as masked scores relative to the reference.
    f32x4 S0, S1;
#pragma unroll
    for (int e = 0; e < 4; ++e) { S0[e] = mask_select(ps.negm, mk[e]); S1[e] = mask_select(ps.negm, mk[4 + e]); }
    S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k00), ps.qb0, S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k10), ps.qb0, S1, 0, 0, 0);
    S0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k01), ps.qb1, S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k11), ps.qb1, S1, 0, 0, 0);

    // V^T operands: issued behind the score MFMAs, consumed after the exponentials
    uint2 va[4][2];
    lds_read_v<VOFF>(v0, v1, va_addr, va);
    float sv[8] = {S0[0], S0[1], S0[2], S0[3], S1[0], S1[1], S1[2], S1[3]};
    // The reference m of a query only moves when one of its scores exceeds it by more than
    // the slack (probabilities stay below 2^kSlack), and once at the query's first kept key.
    // The common case needs the lane's own maximum only; the maximum over the query's four
    // lanes is formed when some lane of the wave has crossed its threshold.
    const float m012 = fmaxf(fmaxf(sv[0], sv[1]), sv[2]), m345 = fmaxf(fmaxf(sv[3], sv[4]), sv[5]);   // (v_max3)
    const float mx = fmaxf(fmaxf(fmaxf(sv[6], sv[7]), m012), m345);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(mx > ps.thr) != 0, 0)) {   // rare after the first steps
      const float mxr = max_across_rows(mx);
      const bool grow = mxr > ps.thr;
      const float shift = grow ? mxr : 0.f;               // m moves by this much (down only when m was unset)
      const float alpha = __builtin_amdgcn_exp2f(-fmaxf(shift, 0.f) * c);
      ps.negm -= shift;
      ps.thr = grow ? slack : ps.thr;
#pragma unroll
      for (int e = 0; e < 8; ++e) sv[e] -= shift;
      ps.Lacc *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) ps.O[dt] *= alpha;
    }
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(sv[e] * c);
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
  int doneA = 0, doneB = 0;                             // steps finished so far
  auto run_phase = [&](int ph, auto is_first, auto has_next) {
    constexpr bool FIRST = decltype(is_first)::value, NEXT = decltype(has_next)::value;
    if (!FIRST && ph == kBoostPhases) __builtin_amdgcn_s_setprio(0);
    [[maybe_unused]] ChunkRegs cr0, cr1;                 // Q8: the chunks of phase ph + 1 on their way
    // (scalar loads, two phases ahead of their use)
    const int end2A = peA[last_chunk(ph + 2)], end2B = PW == 2 ? peB[last_chunk(ph + 2)] : 0;
    if constexpr (!FIRST) {            // (phase 0: fetched in the prologue)
      load_later(dAl, descA, doneA, endA);
      load_later(dBl, descB, doneB, endB);
    }
    if (doneA < endA) run_step(A, dA0, maskA, doneA);
    if (doneB < endB) run_step(B, dB0, maskB, doneB);
    if constexpr (NEXT) {
      if constexpr (!FIRST) {
        // The later descriptors have had two steps to arrive; with nothing else outstanding
        // when the chunks go out, no later use of a loaded register has to wait for them
        // (the compiler would otherwise wait for everything, the chunks included).
        wait_vmcnt<0>();
      }
      // first descriptors and tokens of the next phase: in place, their users are done
      // (ahead of the chunks: a load issued behind a chunk is held up until its data is in)
      dA0 = load_desc(descA, min(endA, lastA));
      if constexpr (PW == 2) dB0 = load_desc(descB, min(endB, lastB));
      if constexpr (!FIRST) {
        const int t0 = tok_of(2 * ph + 1, tokn0), t1 = tok_of(2 * ph + 2, tokn1);
        tokn0 = load_tok(2 * ph + 3); tokn1 = load_tok(2 * ph + 4);
        // the chunks of phase ph + 1, into the slots of chunks 2 ph - 4 and 2 ph - 3
        if constexpr (Q8) { cr0 = load_chunk(t0); cr1 = load_chunk(t1); }
        else { issue_chunk(2 * ph + 1, t0); issue_chunk(2 * ph + 2, t1); }
      }
    }
#pragma unroll
    for (int i = 0; i < kLater; ++i)
      if (doneA + 1 + i < endA) run_step(A, dAl[i], maskA, doneA + 1 + i);
    // (a patch rarely has more steps in a phase; their descriptors are loaded on the spot)
    for (int s = doneA + 1 + kLater; s < endA; ++s) run_step(A, load_desc(descA, s), maskA, s);
#pragma unroll
    for (int i = 0; i < kLater; ++i)
      if (doneB + 1 + i < endB) run_step(B, dBl[i], maskB, doneB + 1 + i);
    for (int s = doneB + 1 + kLater; s < endB; ++s) run_step(B, load_desc(descB, s), maskB, s);
    doneA = endA; doneB = endB;
    endA = end1A; endB = end1B; end1A = end2A; end1B = end2B;
    // The chunks of phase ph + 1, the next descriptors and tokens are in once nothing of
    // this wave is outstanding.  All LDS reads of the phase have returned (each step waits
    // for its own), so after the barrier the slots of chunks 2 ph - 3 and 2 ph - 2 are free.
    wait_vmcnt<0>();
    if constexpr (Q8 && NEXT && !FIRST) {
      // (their slots held chunks 2 ph - 4 and 2 ph - 3, which nobody has read since the
      // barrier that ended phase ph - 1; the writes are complete before this phase's barrier)
      commit_chunk(2 * ph + 1, cr0); commit_chunk(2 * ph + 2, cr1);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    if constexpr (NEXT) asm volatile("s_barrier" ::: "memory");
  };
  {
    run_phase(0, std::true_type{}, std::true_type{});
    int ph = 1;
    for (; ph + 1 < P; ++ph) run_phase(ph, std::false_type{}, std::true_type{});
    run_phase(ph, std::false_type{}, std::false_type{});    // (no steps left when the list is one chunk)
  }


  asm volatile("" : : "v"(warm));      // the only use of the plan-touching load: keeps it

  // ---- epilogue ----
  auto store_patch = [&](const PatchState& ps, const PatchWords& w) {
    int n_again = n;                           // recomputed from scratch: the row is not worth a
    asm volatile("" : "+v"(n_again));          // register (or a spill slot) through the loop
    int qrow = query_row(w, n_again, false);
    if (qrow < 0) return;
    qrow = checked_index(a.hdr, qrow, a.q_len);
    const float inv = 1.f / ps.Lacc[0];
    __bf16* op = (__bf16*)a.o + b * a.os[0] + h * a.os[1] + qrow * a.os[2] + 4 * g4;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      bf16x4 r;
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = (__bf16)(ps.O[dt][i] * inv);
      *(bf16x4*)(op + 16 * dt) = r;
      if (shared) *(bf16x4*)(op + (a.B / 2) * a.os[0] + 16 * dt) = r;
    }
  };
  store_patch(A, pwA);
  if constexpr (PW == 2) store_patch(B, pwB);
}

litevar_status launch_attn_bf16_pair(const litevar_plan* pl, const AttnArgs& a, hipStream_t st) {
  if (pl->waves_per_group != 16 || pl->chunk_keys != kDmaKeys || pl->ring_chunks != kRingChunks)
    return fail(LITEVAR_E_PLAN_CORRUPT, "no 16-patch kernel for chunk=%d ring=%d", pl->chunk_keys, pl->ring_chunks);
  const int64_t bh8 = ((int64_t)a.B * a.H + 7) / 8 * 8;
  const int64_t blocks = bh8 * a.n_groups;
  if (blocks > 0x7fffffff) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  // One patch per wave when the launch has no more working workgroups than the GPU has CUs
  // (with output sharing about half of them exit at once): sixteen waves then fill the CU that
  // eight would leave half empty.
  int pw = pl->patches_per_wave;
  if (pw == 0) {
    static thread_local int n_cu[64] = {0};
    int dev = 0;
    if (litevar_status s = hip_check(hipGetDevice(&dev), "hipGetDevice")) return s;
    if (dev >= 0 && dev < 64 && n_cu[dev] == 0)
      if (litevar_status s = hip_check(hipDeviceGetAttribute(&n_cu[dev], hipDeviceAttributeMultiprocessorCount, dev),
                                       "hipDeviceGetAttribute")) return s;
    const int cus = dev >= 0 && dev < 64 ? n_cu[dev] : 256;
    const int64_t working = a.cfg_share ? ((int64_t)a.B * a.H * a.n_groups + 1) / 2 : (int64_t)a.B * a.H * a.n_groups;
    pw = working <= cus ? 1 : 2;
  }
  const float c = a.sm_scale * 1.4426950408889634f;
  const bool q8 = a.k_sz != nullptr;
  const dim3 grid((unsigned)blocks), wg1(kGroupPatches * 64), wg2(kGroupPatches / 2 * 64);
  if (pw == 1 && q8) hipLaunchKernelGGL((k_attn_bf16_pair<1, true>), grid, wg1, 0, st, a, c);
  else if (pw == 1) hipLaunchKernelGGL((k_attn_bf16_pair<1, false>), grid, wg1, 0, st, a, c);
  else if (q8) hipLaunchKernelGGL((k_attn_bf16_pair<2, true>), grid, wg2, 0, st, a, c);
  else hipLaunchKernelGGL((k_attn_bf16_pair<2, false>), grid, wg2, 0, st, a, c);
  return hip_check(hipGetLastError(), "bf16 attention launch");
}

}  // namespace lv
