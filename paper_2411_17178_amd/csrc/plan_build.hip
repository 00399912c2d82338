// Plan construction: host-side validation and sizing, device-side builder kernels
// (window table, work-list count -> scan -> fill) and the parity exports.
#include "internal.h"

#include <cmath>
#include <cstring>
#include <vector>

namespace lv {

// ---- host: descriptor -> geometry ------------------------------------------

static void choose_tiling(Geom& g, int waves, int chunk, int depth, int spare) {
  g.NW = waves;
  g.C = chunk; g.D = depth; g.A = 1;
  // group shape of every scale: 4 x 4 patches (16 x 16 queries) where the scale's patch grid
  // is a multiple of it, otherwise whatever needs the fewest workgroups (a 5 x 5 grid is
  // tiled by two groups of 3 x 5 and 2 x 5 patches rather than by four of 16, 4, 4 and 1)
  for (int k = 0; k < g.K; ++k) {
    int rh, rw;
    choose_group_shape((g.s[k] + kPatch - 1) / kPatch, waves, rh, rw);
    g.grh[k] = (short)rh; g.grw[k] = (short)rw;
  }
  g.NR = g.A + 1 + g.D + spare;
  g.logC = 0;
  while ((1 << g.logC) < g.C) ++g.logC;
  g.logS = g.logC; g.R = g.NR * g.C;
  if (waves == 16) {
    // The 16-patch kernel runs phases of two 64-key chunks (`chunk` = 128 keys) over a ring
    // of five: one chunk of look-back, the two of the phase and the two that are landing.
    // The plan counts in 64-key chunks (phase tables, list padding, ring depth).
    g.C = 64; g.logC = 6; g.logS = 6; g.NR = 5; g.R = 320;
  }
}

litevar_status make_spec(const litevar_mask_desc* d, const litevar_plan_opts* opts, PlanSpec& sp) {
  Geom& g = sp.g;
  if (!d) return fail(LITEVAR_E_INVALID_ARG, "desc is NULL");
  if (d->n_scales < 1 || d->n_scales > kMaxScales)
    return fail(LITEVAR_E_INVALID_ARG, "n_scales must be in 1..%d (got %d)", kMaxScales, d->n_scales);
  if (!d->scales) return fail(LITEVAR_E_INVALID_ARG, "scales is NULL");
  memset(&g, 0, sizeof g);
  g.K = d->n_scales;
  int64_t L = 0;
  for (int k = 0; k < g.K; ++k) {
    const int s = d->scales[k];
    if (s < 1 || s > kMaxSide)
      return fail(LITEVAR_E_INVALID_ARG, "scales[%d] = %d outside 1..%d", k, s, kMaxSide);
    g.s[k] = s; g.off[k] = (int)L; L += (int64_t)s * s;
    if (L > (int64_t)1 << 30) return fail(LITEVAR_E_UNSUPPORTED, "sequence longer than 2^30 tokens");
    if (s > g.smax) g.smax = s;
  }
  g.off[g.K] = (int)L; g.L = (int)L;
  if (d->mask_mode != LITEVAR_MASK_WINDOW_2D && d->mask_mode != LITEVAR_MASK_BAND_1D)
    return fail(LITEVAR_E_INVALID_ARG, "unknown mask_mode %d", d->mask_mode);
  g.mode = d->mask_mode == LITEVAR_MASK_BAND_1D ? kModeBand : kModeWindow;

  // radius tables: one per head when radius_per_head is given (heads with equal tables are
  // put into one head group and share its work-list), else one for all heads
  if (d->n_heads < 0 || d->n_heads > kMaxHeads)
    return fail(LITEVAR_E_INVALID_ARG, "n_heads must be in 0..%d (got %d)", kMaxHeads, d->n_heads);
  if ((d->n_heads > 0) != (d->radius_per_head != nullptr))
    return fail(LITEVAR_E_INVALID_ARG, "n_heads and radius_per_head must be given together");
  const int KK = g.K * g.K;
  sp.n_heads = d->n_heads;
  sp.rad_all.clear();
  const int n_tables = d->n_heads > 0 ? d->n_heads : 1;
  int n_hg = 0;
  std::vector<int16_t> tab(KK);
  for (int h = 0; h < n_tables; ++h) {
    for (int k = 0; k < g.K; ++k)
      for (int j = 0; j < g.K; ++j) {
        const int r = d->radius_per_head ? d->radius_per_head[(int64_t)h * KK + k * g.K + j]
                    : d->radius_per_scale_pair ? d->radius_per_scale_pair[k * g.K + j]
                    : d->radius_per_key_scale ? d->radius_per_key_scale[j] : d->radius;
        if (r < LITEVAR_RADIUS_DENSE)
          return fail(LITEVAR_E_INVALID_ARG, "radius %d of key scale %d (query scale %d) is below -1", r, j, k);
        // (entries above the diagonal are never used: normalised so that equal tables compare equal)
        tab[k * g.K + j] = j > k ? (int16_t)0 : (int16_t)(r > kMaxRadius ? kMaxRadius : r);
      }
    int found = -1;
    for (int q = 0; q < n_hg && found < 0; ++q)
      if (memcmp(&sp.rad_all[(size_t)q * KK], tab.data(), KK * sizeof(int16_t)) == 0) found = q;
    if (found < 0) { found = n_hg++; sp.rad_all.insert(sp.rad_all.end(), tab.begin(), tab.end()); }
    sp.head_group[h] = (uint8_t)found;
  }
  g.n_hg = n_hg;
  sp.load_head_group(0);

  if (d->n_sink_scales < 0 || d->n_sink_scales > g.K)
    return fail(LITEVAR_E_INVALID_ARG, "n_sink_scales %d outside 0..%d", d->n_sink_scales, g.K);
  g.n_sink = d->n_sink_scales;
  if (d->q_scale_begin < 0 || d->q_scale_end > g.K || d->q_scale_begin >= d->q_scale_end)
    return fail(LITEVAR_E_INVALID_ARG, "query scale range [%d, %d) is empty or outside [0, %d)",
                d->q_scale_begin, d->q_scale_end, g.K);
  g.qb = d->q_scale_begin; g.qe = d->q_scale_end;
  g.q0 = g.off[g.qb]; g.Lq = g.off[g.qe] - g.q0;

  int waves = opts ? opts->waves_per_group : 0;
  if (waves == 0) {
    int sq = 0;
    for (int k = g.qb; k < g.qe; ++k) if (g.s[k] > sq) sq = g.s[k];
    waves = sq > 8 ? 16 : 4;    // (queries of side <= 8 are one group of 2 x 2 patches: the smaller kernel is quicker)
    // A caller that says how many (batch, head) pairs its launches will have gets smaller
    // groups when 16-patch groups would leave most of the GPU's 256 CUs without a workgroup
    // (measured on the VAR-d30 KV step: 60 pairs 14.4 -> 10.4 us with 4 patches per group, 120
    // pairs 14.8 -> 13.4 us with 8, from 240 pairs on 16 patches per group are the quickest).
    const int hint = opts ? opts->batch_heads_hint : 0;
    if (hint < 0) return fail(LITEVAR_E_INVALID_ARG, "batch_heads_hint must not be negative (got %d)", hint);
    if (waves == 16 && hint > 0) {
      int64_t g16 = 0, g8 = 0;
      for (int k = g.qb; k < g.qe; ++k) {
        const int pps = (g.s[k] + kPatch - 1) / kPatch;
        g16 += (int64_t)((pps + 3) / 4) * ((pps + 3) / 4);
        g8 += (int64_t)((pps + 3) / 4) * ((pps + 1) / 2);
      }
      constexpr int64_t kEnoughWorkgroups = 230;
      if (hint * g16 < kEnoughWorkgroups) waves = hint * g8 >= kEnoughWorkgroups ? 8 : 4;
      // A full sequence of many query scales at a small batch: the launch is as long as its
      // largest workgroup, and a group of 2 x 2 patches streams about half the keys of a
      // group of 4 x 4 (VAR-d16, 32 pairs x 10 scales: 17.7 us with 16 patches per group,
      // 15.0 with 8, 12.4 with 4).
      else if (hint * g16 < 2 * 256 && g.qe - g.qb > 4) waves = 4;
    }
  }
  if (waves != 4 && waves != 8 && waves != 16)
    return fail(LITEVAR_E_INVALID_ARG, "waves_per_group must be 0, 4, 8 or 16 (got %d)", waves);
  int chunk = opts ? opts->chunk_keys : 0, depth = opts ? opts->prefetch_chunks : 0;
  int spare = opts ? opts->spare_chunks : -1;
  if (chunk == 0) chunk = waves == 16 ? 128 : 32;
  if (depth == 0) depth = 2;
  if (spare < 0) spare = waves == 16 ? 0 : chunk == 32 ? 2 : 1;
  if (waves == 16 && (chunk != 128 || depth != 2 || spare != 0))
    return fail(LITEVAR_E_INVALID_ARG, "16 patches per group need (chunk_keys, prefetch_chunks, spare_chunks) = (128, 2, 0)");
  static const int ok[][3] = {{32, 2, 2}, {64, 2, 1}};
  bool found = false;
  for (const auto& t : ok) found |= (t[0] == chunk && t[1] == depth && t[2] == spare);
  found |= waves == 16;
  if (!found)
    return fail(LITEVAR_E_INVALID_ARG, "unsupported (chunk_keys, prefetch_chunks, spare_chunks) = (%d, %d, %d)",
                chunk, depth, spare);
  choose_tiling(g, waves, chunk, depth, spare);

  int64_t ng = 0, np = 0;
  for (int i = 0; i < g.qe - g.qb; ++i) {
    const int k = g.qe - 1 - i;
    g.grp_off[i] = (int)ng;
    ng += (int64_t)groups_y(g, k) * groups_x(g, k);
    np += (int64_t)scale_patches(g, k);
  }
  g.grp_off[g.qe - g.qb] = (int)ng;
  if (ng * g.n_hg > (int64_t)1 << 26) return fail(LITEVAR_E_UNSUPPORTED, "too many groups");
  g.n_groups = (int)ng; g.n_patches = (int)np;
  return LITEVAR_OK;
}

static uint64_t align256(uint64_t x) { return (x + 255) & ~(uint64_t)255; }

// The sizing walk visits every (patch, key) pair on the host (tens of milliseconds for the
// largest plans).  Callers size and then build with the same descriptor, often repeatedly,
// so the last result is remembered per thread, keyed by the whole specification.
static thread_local struct { bool valid; PlanSpec sp; PlanSizes z; } g_last_sizing = {false, {}, {}};

static litevar_status size_plan_uncached(PlanSpec& sp, PlanSizes& z);

static bool same_spec(const PlanSpec& a, const PlanSpec& b) {
  // (the Geom holds the radii of the head group that was loaded last: compare it with
  // group 0 loaded on both sides, which is how make_spec leaves it)
  return memcmp(&a.g, &b.g, sizeof a.g) == 0 && a.n_heads == b.n_heads && a.rad_all == b.rad_all &&
         memcmp(a.head_group, b.head_group, sizeof a.head_group) == 0;
}

litevar_status size_plan(PlanSpec& sp, PlanSizes& z) {
  if (g_last_sizing.valid && same_spec(g_last_sizing.sp, sp)) { z = g_last_sizing.z; return LITEVAR_OK; }
  const litevar_status rc = size_plan_uncached(sp, z);
  sp.load_head_group(0);
  if (rc == LITEVAR_OK) { g_last_sizing.sp = sp; g_last_sizing.z = z; g_last_sizing.valid = true; }
  return rc;
}

static litevar_status size_plan_uncached(PlanSpec& sp, PlanSizes& z) {
  Geom& g = sp.g;
  memset(&z, 0, sizeof z);
  for (int hg = 0; hg < g.n_hg; ++hg) {
    sp.load_head_group(hg);
    const ArithWin win{g};
    const ArithRad rad{g};
    int64_t pairs_hg = 0;
    for (int grp = 0; grp < g.n_groups; ++grp) {
      int k, gy, gx;
      group_coords(g, grp, k, gy, gx);
      const GroupExtent e = group_extent(g, k, gy, gx);
      const int nu = group_union_keys(g, win, rad, e);
      const int nph = (nu + g.C - 1) / g.C;
      z.n_union += (int64_t)nph * g.C;
      z.n_phase_entries += (int64_t)nph * g.NW;
      for (int w = 0; w < g.NW; ++w) {
        CountSink sink;
        const int ns = walk_patch(g, e, patch_extent(g, k, gy, gx, w), sink);
        if (ns > 65535) return fail(LITEVAR_E_UNSUPPORTED, "a query patch needs more than 65535 steps");
        z.n_steps += ns;
        pairs_hg += sink.pairs;
      }
    }
    z.retained_pairs += pairs_hg;
    if (hg < kMaxHeads) z.pairs_of_group[hg] = pairs_hg;
  }
  if (z.n_steps > (int64_t)1 << 26 || z.n_union > (int64_t)1 << 30)
    return fail(LITEVAR_E_UNSUPPORTED, "work-list too large (%lld steps)", (long long)z.n_steps);
  const uint64_t ngt = (uint64_t)g.n_groups * g.n_hg;
  uint64_t o = 0;
  z.off[kSecHeader] = o; o += sizeof(Header);
  z.off[kSecWin] = o;
  o = align256(o + (g.mode == kModeWindow ? (uint64_t)g.n_hg * g.K * g.K * g.smax * 2 * sizeof(int16_t) : 0));
  z.off[kSecRad] = o; o = align256(o + (uint64_t)g.n_hg * g.K * g.K * sizeof(int16_t));
  z.off[kSecHeadMap] = o; o = align256(o + (uint64_t)kMaxHeads * sizeof(int32_t));
  z.off[kSecGroups] = o; o = align256(o + ngt * sizeof(GroupDesc));
  z.off[kSecWaves] = o; o = align256(o + ngt * g.NW * sizeof(WaveDesc));
  z.off[kSecPhaseEnd] = o; o = align256(o + (uint64_t)z.n_phase_entries * sizeof(int32_t));
  z.off[kSecUnion] = o; o = align256(o + (uint64_t)z.n_union * sizeof(int32_t));
  z.off[kSecStepAddr] = o; o = align256(o + (uint64_t)z.n_steps * 64 * sizeof(uint2));
  z.off[kSecStepMask] = o; o = align256(o + (uint64_t)z.n_steps * 8 * sizeof(uint64_t));
  z.off[kSecStepTok] = o; o = align256(o + (uint64_t)z.n_steps * kStepKeys * sizeof(int32_t));
  z.off[kSecEnd] = o;
  z.bytes = o;
  return LITEVAR_OK;
}

// ---- device: builder kernels -------------------------------------------------

struct BlobPtrs {
  Header* hdr; int16_t* win; int16_t* rad; int32_t* head_map; GroupDesc* groups; WaveDesc* waves;
  int32_t* phase_end; int32_t* union_tok; uint2* step_addr; uint64_t* step_mask; int32_t* step_tok;
};

static BlobPtrs blob_ptrs(void* blob, const uint64_t* off) {
  char* b = (char*)blob;
  BlobPtrs p;
  p.hdr = (Header*)(b + off[kSecHeader]); p.win = (int16_t*)(b + off[kSecWin]);
  p.rad = (int16_t*)(b + off[kSecRad]); p.head_map = (int32_t*)(b + off[kSecHeadMap]);
  p.groups = (GroupDesc*)(b + off[kSecGroups]); p.waves = (WaveDesc*)(b + off[kSecWaves]);
  p.phase_end = (int32_t*)(b + off[kSecPhaseEnd]); p.union_tok = (int32_t*)(b + off[kSecUnion]);
  p.step_addr = (uint2*)(b + off[kSecStepAddr]); p.step_mask = (uint64_t*)(b + off[kSecStepMask]);
  p.step_tok = (int32_t*)(b + off[kSecStepTok]);
  return p;
}

struct Caps { int64_t n_steps, n_union, n_phase_entries, retained_pairs; uint64_t bytes; };

// K1, once per head group (g.rad holds that group's radii): the radius table
// rad[hg][k][j] (-1: dense part) and, in window mode, the window table
// win[hg][k][j][c] = inclusive [lo, hi]; (-1,-1) where undefined.  Every other builder
// kernel reads these tables and never the radii of the descriptor.
__global__ void k_tables(Geom g, int hg, int16_t* win, int16_t* rad) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < g.K * g.K) {
    const int j = idx % g.K, k = idx / g.K;
    rad[(size_t)hg * g.K * g.K + idx] = j > k ? (int16_t)0 : (j < g.n_sink ? (int16_t)-1 : g.rad[k][j]);
  }
  if (g.mode != kModeWindow) return;
  const int total = g.K * g.K * g.smax;
  if (idx >= total) return;
  const int c = idx % g.smax, j = (idx / g.smax) % g.K, k = idx / (g.smax * g.K);
  Interval iv = {-1, -1};
  if (j <= k && c < g.s[k]) iv = win_interval(g, k, j, c);
  int16_t* out = win + ((size_t)hg * total + idx) * 2;
  out[0] = (int16_t)iv.lo; out[1] = (int16_t)iv.hi;
}

struct HeadMapArg { uint8_t group[kMaxHeads]; };

__global__ void k_head_map(HeadMapArg m, int n_heads, int32_t* out) {
  const int i = threadIdx.x;
  if (i < kMaxHeads) out[i] = i < n_heads ? m.group[i] : 0;
}

// value of `v` in lane `lane`, for a lane index that is the same in every lane of the wave:
// v_readlane_b32, where __shfl would go through the LDS crossbar
__device__ inline int lane_value(int v, int lane) {
  return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(lane));
}

// Placement of the kept keys of one pass (64 candidate keys, one per lane, in key order) in
// the patch's steps: they get consecutive places; a pass is cut where a step fills up (32
// keys) or where the next key's 2^logS-key block lies more than A blocks after the block of
// the step's first key, exactly as in the serial walk, so both produce the same steps.
// Sink receives
//   keys(step, idx, upos, token, qmask, take)   per pass segment: lanes with take set hold
//                                               the key that becomes entry idx of the step
//   close(step, n_keys, last_upos)              when a step is complete (wave-uniform)
template <class Sink>
struct WavePacker {
  const Geom& g; Sink& sink; int lane;
  int step = 0, cnt = 0, first_block = 0, last_upos = 0;
  __device__ void pass(bool kept, int upos, int tok, unsigned qmask) {
    const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    const int blk = upos >> g.logS;
    uint64_t km = __ballot(kept);                     // kept keys of this pass not yet placed
    while (km) {
      const int fl = __builtin_ctzll(km);
      const int fblk = lane_value(blk, fl);
      if (cnt > 0 && fblk - first_block > g.A) { sink.close(step, cnt, last_upos); ++step; cnt = 0; }
      if (cnt == 0) first_block = fblk;
      const bool mine = (km >> lane) & 1;
      // lanes whose key still fits the step's span (blocks grow with the lane), ranked
      const uint64_t fit = __ballot(mine && blk - first_block <= g.A);
      const int rank = __builtin_popcountll(fit & lt_mask);
      const bool take = ((fit >> lane) & 1) && rank < kStepKeys - cnt;
      const uint64_t tm = __ballot(take);
      sink.keys(step, cnt + rank, upos, tok, qmask, take);
      last_upos = lane_value(upos, 63 - __builtin_clzll(tm));
      cnt += __builtin_popcountll(tm);
      km &= ~tm;
      if (cnt == kStepKeys) { sink.close(step, cnt, last_upos); ++step; cnt = 0; }
    }
  }
  __device__ int finish() {
    if (cnt > 0) { sink.close(step, cnt, last_upos); ++step; cnt = 0; }
    return step;
  }
};

// Wave-cooperative form of walk_patch(): the 64 lanes of a wave take 64 consecutive candidate
// keys at a time (window mode: several rows of a narrow box, or 64 columns of one row of the
// patch's box in a key scale; band mode: 64 columns of the patch's range in a part).
template <class Sink>
__device__ int wave_walk_patch(const Geom& g, const TableWin& win, const TableRad& rad, const GroupExtent& e,
                               const PatchExtent& p, Sink& sink, int lane) {
  if (p.ny == 0) return 0;
  WavePacker<Sink> pack{g, sink, lane};
  int ubase = 0;
  if (g.mode == kModeBand) {
    const int nk = g.s[e.k] * g.s[e.k];
    for (int pt = 0; pt < band_parts(e.k); ++pt) {
      const BandPart b = band_part(g, rad, e.k, pt);
      const int glo = band_interval(b, nk, e.qy0).lo, ghi = band_interval(b, nk, e.qy1).hi;
      // the sixteen queries' intervals: one lane each (a 64-bit division), handed round
      Interval mine = {1, 0};
      if (lane < p.nx) mine = band_interval(b, nk, p.y0 + lane);
      Interval iv[kPatchQueries];
#pragma unroll
      for (int n = 0; n < kPatchQueries; ++n) { iv[n].lo = lane_value(mine.lo, n); iv[n].hi = lane_value(mine.hi, n); }
      const int clo = iv[0].lo, chi = lane_value(mine.hi, p.nx - 1);
      for (int c0 = clo; c0 <= chi; c0 += 64) {
        const int c = c0 + lane;
        unsigned qmask = 0;
        if (c <= chi) {
#pragma unroll
          for (int n = 0; n < kPatchQueries; ++n) qmask |= (unsigned)(c >= iv[n].lo && c <= iv[n].hi) << n;
        }
        pack.pass(qmask != 0, ubase + c - glo, b.tok0 + c, qmask);
      }
      ubase += ghi - glo + 1;
    }
    return pack.finish();
  }
  // The twelve window intervals that a key scale needs (four patch rows, four patch columns,
  // the group's first and last row and column) are fetched from the table for ALL key scales
  // before the walk: sixteen lanes per key scale, four key scales per round, so the walk pays
  // the table's latency once and not once per key scale.  They are handed round with
  // v_readlane.
  constexpr int kRounds = kMaxScales / 4;
  Interval pre[kRounds];
  {
    const int sk = g.s[e.k];
    const int role = lane & 15;
    int cq = role < 4 ? p.y0 + role : role < 8 ? p.x0 + role - 4 : role == 8 ? e.qy0 : role == 9 ? e.qy1 : role == 10 ? e.qx0 : e.qx1;
    cq = cq < sk ? cq : sk - 1;
#pragma unroll
    for (int t = 0; t < kRounds; ++t) {
      pre[t].lo = 1; pre[t].hi = 0;
      const int j = 4 * t + (lane >> 4);
      if (4 * t <= e.k && j <= e.k && role < 12) pre[t] = win(e.k, j, cq);
    }
  }
  for (int j = 0; j <= e.k; ++j) {
    Interval mine_iv = pre[0];
#pragma unroll
    for (int t = 1; t < kRounds; ++t)
      if ((j >> 2) == t) mine_iv = pre[t];             // (uniform)
    const int l0 = (j & 3) * 16;                         // first lane of this key scale's sixteen
    const Interval none = {1, 0};
    Interval rw[kPatch], cw[kPatch];
#pragma unroll
    for (int d = 0; d < kPatch; ++d) {
      const Interval r = {lane_value(mine_iv.lo, l0 + d), lane_value(mine_iv.hi, l0 + d)};
      const Interval cc = {lane_value(mine_iv.lo, l0 + 4 + d), lane_value(mine_iv.hi, l0 + 4 + d)};
      rw[d] = d < p.ny ? r : none;
      cw[d] = d < p.nx ? cc : none;
    }
    Box gb, pb;
    gb.ylo = lane_value(mine_iv.lo, l0 + 8); gb.yhi = lane_value(mine_iv.hi, l0 + 9);
    gb.xlo = lane_value(mine_iv.lo, l0 + 10); gb.xhi = lane_value(mine_iv.hi, l0 + 11);
    pb.ylo = rw[0].lo; pb.yhi = lane_value(mine_iv.hi, l0 + p.ny - 1);
    pb.xlo = cw[0].lo; pb.xhi = lane_value(mine_iv.hi, l0 + 4 + p.nx - 1);
    const int gw = gb.xhi - gb.xlo + 1;
    const int sj = g.s[j], offj = g.off[j];
    // lanes of a pass in key order: RP rows of the patch's box (W columns each) when the box
    // is narrower than a wave, else 64 columns of one row
    const int W = pb.xhi - pb.xlo + 1;
    const int WL = W < 64 ? W : 64, RP = 64 / WL;
    const int ry = lane / WL, xx = lane - ry * WL;
    for (int y0 = pb.ylo; y0 <= pb.yhi; y0 += RP) {
      const int y = y0 + ry;
      unsigned rb = 0;
      if (ry < RP && y <= pb.yhi) {
#pragma unroll
        for (int d = 0; d < kPatch; ++d) rb |= (unsigned)(y >= rw[d].lo && y <= rw[d].hi) << d;
      }
      const unsigned rowmask = ((rb & 1) ? 0x000fu : 0u) | ((rb & 2) ? 0x00f0u : 0u) |
                               ((rb & 4) ? 0x0f00u : 0u) | ((rb & 8) ? 0xf000u : 0u);
      const int urow = ubase + (y - gb.ylo) * gw - gb.xlo, trow = offj + y * sj;
      for (int x0 = pb.xlo; x0 <= pb.xhi; x0 += WL) {
        const int x = x0 + xx;
        unsigned cb = 0;
        if (rb && x <= pb.xhi) {
#pragma unroll
          for (int d = 0; d < kPatch; ++d) cb |= (unsigned)(x >= cw[d].lo && x <= cw[d].hi) << d;
        }
        pack.pass(cb != 0, urow + x, trow + x, (cb * 0x1111u) & rowmask);
      }
    }
    ubase += (gb.yhi - gb.ylo + 1) * gw;
  }
  return pack.finish();
}

struct WaveCountSink {
  int pairs = 0;                                         // this lane's share
  __device__ void keys(int, int, int, int, unsigned qmask, bool take) { if (take) pairs += __builtin_popcount(qmask); }
  __device__ void close(int, int, int) {}
};

// the tables of the head group that global group G belongs to
struct GroupTables { TableWin win; TableRad rad; int grp; };
__device__ inline GroupTables group_tables(const Geom& g, const BlobPtrs& p, int G) {
  const int hg = G / g.n_groups;
  GroupTables t;
  t.win = TableWin{p.win + (size_t)hg * g.K * g.K * g.smax * 2, g.K, g.smax};
  t.rad = TableRad{p.rad + (size_t)hg * g.K * g.K, g.K};
  t.grp = G - hg * g.n_groups;
  return t;
}

// K2a: one wave per (group, patch): number of steps and kept pairs; patch 0 also
// sizes the group's union list
__global__ __launch_bounds__(64) void k_count(Geom g, BlobPtrs p) {
  const int idx = blockIdx.x, lane = threadIdx.x;
  const int G = idx / g.NW, w = idx % g.NW;
  const GroupTables t = group_tables(g, p, G);
  int k, gy, gx;
  group_coords(g, t.grp, k, gy, gx);
  const GroupExtent e = group_extent(g, k, gy, gx);
  const PatchExtent pe = patch_extent(g, k, gy, gx, w);
  WaveCountSink sink;
  const int ns = wave_walk_patch(g, t.win, t.rad, e, pe, sink, lane);
  int pairs = sink.pairs;
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) pairs += __shfl_xor(pairs, d);
  if (lane == 0) {
    WaveDesc wd;
    int q_base, sk; uint32_t valid;
    patch_queries(g, k, pe, q_base, sk, valid);
    wd.step_begin = 0; wd.n_steps = ns;
    wd.q_base = q_base;
    wd.sk = (int16_t)sk; wd.ny = (int16_t)pe.ny; wd.nx = (int16_t)pe.nx; wd.kq = (int16_t)k;
    wd.pairs = pairs; wd.valid = valid; wd.first_ends = 0;
    p.waves[idx] = wd;
  }
  if (w == 0) {
    // the group's descriptor; in window mode lane j holds the group's box in key scale j, so
    // that the table is read once, by all lanes at the same time
    GroupDesc gd;
    int ident = 0;                                      // leading union entries whose token equals their position
    if (g.mode == kModeBand) {
      gd.n_union = group_union_keys(g, t.win, t.rad, e);
      const int nk = g.s[k] * g.s[k];
      for (int pt = 0; pt < band_parts(k); ++pt) {
        const BandPart b = band_part(g, t.rad, k, pt);
        const int glo = band_interval(b, nk, e.qy0).lo, ghi = band_interval(b, nk, e.qy1).hi;
        if (b.tok0 + glo != ident) break;
        ident += ghi - glo + 1;
        if (ghi != b.cols - 1) break;
      }
    } else {
      Box mine = {0, -1, 0, -1};
      if (lane <= k) mine = window_box(t.win, k, lane, e.qy0, e.qy1, e.qx0, e.qx1);
      int n = (mine.yhi - mine.ylo + 1) * (mine.xhi - mine.xlo + 1);
#pragma unroll
      for (int d = 32; d > 0; d >>= 1) n += __shfl_xor(n, d);
      gd.n_union = n;
      // whole key scales from scale 0 on, then the first rows of the next box if it starts
      // at the scale's origin
      for (int j = 0; j <= k; ++j) {
        const Box b = {lane_value(mine.ylo, j), lane_value(mine.yhi, j), lane_value(mine.xlo, j), lane_value(mine.xhi, j)};
        const int gw = b.xhi - b.xlo + 1, rows = b.yhi - b.ylo + 1;
        if (b.ylo != 0 || b.xlo != 0 || g.off[j] != ident) break;
        if (gw != g.s[j]) { ident += gw; break; }
        ident += rows * gw;
        if (rows != g.s[j]) break;
      }
    }
    gd.union_base = 0;
    gd.n_phases = (gd.n_union + g.C - 1) / g.C;
    gd.k = k; gd.gy = gy; gd.gx = gx; gd.phase_base = 0;
    gd.ident = ident;
    if (lane == 0) p.groups[G] = gd;
  }
}

// K2b: exclusive scans over groups (union keys, phase entries) and patches (steps) by one
// 1024-thread block: per-thread partial sums over a contiguous slice of groups, a block-wide
// scan of the partials (Hillis-Steele in LDS), then the slice is revisited
__global__ __launch_bounds__(1024) void k_scan(Geom g, BlobPtrs p, Caps caps) {
  __shared__ int64_t part[2][4][1024];
  const int t = threadIdx.x;
  const int n_all = g.n_groups * g.n_hg;
  const int per = (n_all + 1023) / 1024;
  const int g0 = t * per < n_all ? t * per : n_all;
  const int g1 = g0 + per < n_all ? g0 + per : n_all;
  int64_t v[4] = {0, 0, 0, 0};                          // steps, union keys, phase entries, pairs
  for (int grp = g0; grp < g1; ++grp) {
    v[1] += (int64_t)p.groups[grp].n_phases * g.C; v[2] += (int64_t)p.groups[grp].n_phases * g.NW;
    for (int w = 0; w < g.NW; ++w) { v[0] += p.waves[grp * g.NW + w].n_steps; v[3] += p.waves[grp * g.NW + w].pairs; }
  }
  int cur = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) part[0][i][t] = v[i];
  __syncthreads();
  for (int d = 1; d < 1024; d <<= 1) {                  // inclusive scan
#pragma unroll
    for (int i = 0; i < 4; ++i) part[cur ^ 1][i][t] = part[cur][i][t] + (t >= d ? part[cur][i][t - d] : 0);
    cur ^= 1;
    __syncthreads();
  }
  int64_t steps = part[cur][0][t] - v[0], uni = part[cur][1][t] - v[1], phe = part[cur][2][t] - v[2];
  for (int grp = g0; grp < g1; ++grp) {
    GroupDesc& gd = p.groups[grp];
    gd.union_base = (int32_t)uni; gd.phase_base = (int32_t)phe;
    uni += (int64_t)gd.n_phases * g.C; phe += (int64_t)gd.n_phases * g.NW;
    for (int w = 0; w < g.NW; ++w) {
      WaveDesc& wd = p.waves[grp * g.NW + w];
      wd.step_begin = (int32_t)steps; steps += wd.n_steps;
    }
  }
  if (t == 1023) {
    Header h;
    memset(&h, 0, sizeof h);
    h.magic = kMagic; h.blob_bytes = caps.bytes;
    h.n_groups = n_all; h.n_waves = n_all * g.NW;
    h.n_steps = part[cur][0][t]; h.n_union = part[cur][1][t]; h.n_phase_entries = part[cur][2][t];
    h.retained_pairs = part[cur][3][t];
    h.error = (h.n_steps != caps.n_steps || h.n_union != caps.n_union ||
               h.n_phase_entries != caps.n_phase_entries || h.retained_pairs != caps.retained_pairs) ? kErrBuilder : kErrNone;
    *p.hdr = h;
  }
}

// K2c: the group's key list (token indices), padded to whole chunks with its last key
__global__ void k_fill_union(Geom g, BlobPtrs p, Caps caps) {
  const int G = blockIdx.x;
  if (p.hdr->error) return;
  const GroupTables t = group_tables(g, p, G);
  const GroupDesc gd = p.groups[G];
  const GroupExtent e = group_extent(g, gd.k, gd.gy, gd.gx);
  int32_t* out = p.union_tok + gd.union_base;
  if ((int64_t)gd.union_base + (int64_t)gd.n_phases * g.C > caps.n_union) return;
  int ubase = 0, last_tok = 0;
  if (g.mode == kModeBand) {
    const int nk = g.s[e.k] * g.s[e.k];
    for (int pt = 0; pt < band_parts(e.k); ++pt) {
      const BandPart b = band_part(g, t.rad, e.k, pt);
      const int glo = band_interval(b, nk, e.qy0).lo, ghi = band_interval(b, nk, e.qy1).hi;
      const int n = ghi - glo + 1;
      for (int i = threadIdx.x; i < n; i += blockDim.x) out[ubase + i] = b.tok0 + glo + i;
      ubase += n;
      last_tok = b.tok0 + ghi;
    }
  } else {
    __shared__ Box boxes[kMaxScales];                   // (the table is read once, by K threads at the same time)
    if ((int)threadIdx.x <= e.k) boxes[threadIdx.x] = window_box(t.win, e.k, (int)threadIdx.x, e.qy0, e.qy1, e.qx0, e.qx1);
    __syncthreads();
    for (int j = 0; j <= e.k; ++j) {
      const Box b = boxes[j];
      const int gw = b.xhi - b.xlo + 1, n = (b.yhi - b.ylo + 1) * gw;
      for (int i = threadIdx.x; i < n; i += blockDim.x)
        out[ubase + i] = g.off[j] + (b.ylo + i / gw) * g.s[j] + b.xlo + i % gw;
      ubase += n;
      last_tok = g.off[j] + b.yhi * g.s[j] + b.xhi;
    }
  }
  for (int i = gd.n_union + threadIdx.x; i < gd.n_phases * g.C; i += blockDim.x) out[i] = last_tok;
}

// Step under construction: the wave's lanes deposit the keys they place (ring slot, token,
// query mask) in a 32-entry LDS buffer; when the step closes every lane picks the entries
// of its role in the attention kernel and the step is written with coalesced stores.
// Lane (n, g4) = (lane % 16, lane / 16):
//   K operand  rows of keys n and 16 + n          -> byte offset of its first 16-byte piece
//   V operand  rows of keys 4*g4 + n/4 (+16)      -> byte offset of its d-tile-0 8-byte read
//   mask bits  element e = 4*t + i  <->  key 16*t + 4*g4 + i against query n
struct StepBuf { uint32_t slot[kStepKeys]; int32_t tok[kStepKeys]; uint32_t qmask[kStepKeys]; };

struct FillSink {
  uint2* addr; uint64_t* mask; int32_t* toks; int32_t* phase_cnt;
  StepBuf* buf;
  int R, logC, lane;
  __device__ static uint32_t k_off(uint32_t slot, int g4) {
    return slot * kRingRowBytes + (((2u * g4) ^ ring_swizzle(slot)) << 4);
  }
  __device__ static uint32_t v_off(uint32_t slot, int n) {
    const uint32_t sw = ring_swizzle(slot), b = (n >> 1) & 1, half = n & 1;
    return slot * kRingRowBytes + 8u * half + 16u * ((b ^ sw) & 1u) + ((sw >> 1) << 5);
  }
  __device__ void keys(int, int idx, int upos, int t, unsigned qmask, bool take) {
    if (take) { buf->slot[idx] = (uint32_t)(upos % R); buf->tok[idx] = t; buf->qmask[idx] = qmask; }
  }
  __device__ void close(int step, int n_keys, int last_upos) {
    __syncthreads();                                   // (one wave per block) deposits are visible
    const int n = lane & 15, g4 = lane >> 4;
    const uint32_t pad = (uint32_t)(last_upos % R);    // padding keys read the step's last row
    auto slot_of = [&](int idx) { return idx < n_keys ? buf->slot[idx] : pad; };
    const uint32_t k0 = k_off(slot_of(n), g4), k1 = k_off(slot_of(16 + n), g4);
    const uint32_t v0 = v_off(slot_of(4 * g4 + (n >> 2)), n), v1 = v_off(slot_of(16 + 4 * g4 + (n >> 2)), n);
    addr[(int64_t)step * 64 + lane] = make_uint2(k0 | (k1 << 16), v0 | (v1 << 16));
    uint64_t mine = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int idx = 16 * (e >> 2) + 4 * g4 + (e & 3);
      const bool bit = idx < n_keys && ((buf->qmask[idx] >> n) & 1u);
      const uint64_t bal = __ballot(bit);
      if (lane == e) mine = bal;
    }
    if (lane < 8) mask[(int64_t)step * 8 + lane] = mine;
    if (lane < kStepKeys) toks[(int64_t)step * kStepKeys + lane] = lane < n_keys ? buf->tok[lane] : -1;
    if (lane == 0) phase_cnt[last_upos >> logC] += 1;
    __syncthreads();                                   // the buffer may be refilled
  }
};

// K2d: one wave per (group, patch): steps (ring addresses, lane masks, tokens) and the
// cumulative number of steps that are runnable after each phase
__global__ __launch_bounds__(64) void k_fill_steps(Geom g, BlobPtrs p, Caps caps) {
  __shared__ StepBuf buf;
  const int idx = blockIdx.x, lane = threadIdx.x;
  if (p.hdr->error) return;
  const int G = idx / g.NW, w = idx % g.NW;
  const GroupTables t = group_tables(g, p, G);
  const GroupDesc gd = p.groups[G];
  const WaveDesc wd = p.waves[idx];
  if ((int64_t)wd.step_begin + wd.n_steps > caps.n_steps ||
      (int64_t)gd.phase_base + (int64_t)gd.n_phases * g.NW > caps.n_phase_entries) return;
  int32_t* pe = p.phase_end + gd.phase_base + (int64_t)w * gd.n_phases;
  for (int i = lane; i < gd.n_phases; i += 64) pe[i] = 0;
  __syncthreads();
  const GroupExtent e = group_extent(g, gd.k, gd.gy, gd.gx);
  FillSink sink;
  sink.addr = p.step_addr + (int64_t)wd.step_begin * 64;
  sink.mask = p.step_mask + (int64_t)wd.step_begin * 8;
  sink.toks = p.step_tok + (int64_t)wd.step_begin * kStepKeys;
  sink.phase_cnt = pe; sink.buf = &buf; sink.R = g.R; sink.logC = g.logC; sink.lane = lane;
  wave_walk_patch(g, t.win, t.rad, e, patch_extent(g, gd.k, gd.gy, gd.gx, w), sink, lane);
  __syncthreads();
  if (lane == 0) {
    int acc = 0;
    for (int i = 0; i < gd.n_phases; ++i) { acc += pe[i]; pe[i] = acc; }
    const int i1 = gd.n_phases - 1 < 2 ? gd.n_phases - 1 : 2;
    p.waves[idx].first_ends = (uint32_t)pe[0] | ((uint32_t)pe[i1] << 16);   // (a patch has at most 65535 steps)
  }
}

litevar_status build_plan(PlanSpec& sp, const PlanSizes& z, void* d_blob, hipStream_t st) {
  Geom& g = sp.g;
  const BlobPtrs p = blob_ptrs(d_blob, z.off);
  Caps caps{z.n_steps, z.n_union, z.n_phase_entries, z.retained_pairs, z.bytes};
  const int ntab = g.mode == kModeWindow ? g.K * g.K * g.smax : g.K * g.K;
  for (int hg = 0; hg < g.n_hg; ++hg) {
    sp.load_head_group(hg);
    hipLaunchKernelGGL(k_tables, dim3((ntab + 255) / 256), dim3(256), 0, st, g, hg, p.win, p.rad);
  }
  sp.load_head_group(0);
  HeadMapArg hm;
  memcpy(hm.group, sp.head_group, sizeof hm.group);
  hipLaunchKernelGGL(k_head_map, dim3(1), dim3(kMaxHeads), 0, st, hm, sp.n_heads, p.head_map);
  const int n_all = g.n_groups * g.n_hg;
  const int nw = n_all * g.NW;
  hipLaunchKernelGGL(k_count, dim3(nw), dim3(64), 0, st, g, p);
  hipLaunchKernelGGL(k_scan, dim3(1), dim3(1024), 0, st, g, p, caps);
  hipLaunchKernelGGL(k_fill_union, dim3(n_all), dim3(256), 0, st, g, p, caps);
  hipLaunchKernelGGL(k_fill_steps, dim3(nw), dim3(64), 0, st, g, p, caps);
  return hip_check(hipGetLastError(), "plan builder launch");
}

// ---- parity exports -------------------------------------------------------------

__global__ void k_export_win(int n, const int16_t* win, int16_t* out) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) out[idx] = win[idx];
}

__global__ void k_fill_u8(uint8_t* p, size_t n, uint8_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

__global__ void k_zero_u64(unsigned long long* p) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0; }

// local query row handled by column n of a patch, or -1
__device__ inline int patch_query_row(const WaveDesc& wd, int n) {
  return ((wd.valid >> n) & 1u) ? wd.q_base + (n / 4) * wd.sk + n % 4 : -1;
}

// one 64-lane block per (group, wave) of the head's group; lane (n, g4) owns the bits of
// query n for the keys {16t + 4*g4 + i} of every step
__global__ void k_export_dense(int L, const WaveDesc* waves, const int32_t* head_map, int head, int waves_per_hg,
                               const uint64_t* masks, const int32_t* toks, uint8_t* mask, unsigned long long* count) {
  const WaveDesc wd = waves[(size_t)head_map[head] * waves_per_hg + blockIdx.x];
  const int lane = threadIdx.x, n = lane % 16, g4 = lane / 16;
  const int qrow = patch_query_row(wd, n);
  unsigned long long local = 0;
  for (int s = 0; s < wd.n_steps; ++s) {
    const int64_t S = (int64_t)wd.step_begin + s;
    for (int e = 0; e < 8; ++e) {
      if (!(masks[S * 8 + e] >> lane & 1)) continue;
      const int tok = toks[S * kStepKeys + 16 * (e / 4) + 4 * g4 + e % 4];
      if (qrow >= 0 && tok >= 0) { mask[(size_t)qrow * L + tok] = 1; ++local; }
    }
  }
  if (count && local) atomicAdd(count, local);
}

__global__ void k_csr_count(const WaveDesc* waves, const int32_t* head_map, int head, int waves_per_hg,
                            const uint64_t* masks, int64_t* rowptr) {
  const WaveDesc wd = waves[(size_t)head_map[head] * waves_per_hg + blockIdx.x];
  const int lane = threadIdx.x, n = lane % 16;
  int cnt = 0;
  for (int s = 0; s < wd.n_steps; ++s)
    for (int e = 0; e < 8; ++e) cnt += (int)(masks[((int64_t)wd.step_begin + s) * 8 + e] >> lane & 1);
  cnt += __shfl_xor(cnt, 16); cnt += __shfl_xor(cnt, 32);
  const int qrow = patch_query_row(wd, n);
  if (lane < 16 && qrow >= 0) rowptr[qrow + 1] = cnt;
}

// in-place inclusive scan of rowptr[1..n] by one 1024-thread block
__global__ void k_csr_scan(int64_t* rowptr, int n) {
  __shared__ int64_t part[1024];
  const int t = threadIdx.x, per = (n + 1023) / 1024;
  const int b = t * per, e = b + per < n ? b + per : n;
  int64_t sum = 0;
  for (int i = b; i < e; ++i) sum += rowptr[i + 1];
  part[t] = sum;
  __syncthreads();
  if (t == 0) {
    int64_t acc = 0;
    for (int i = 0; i < 1024; ++i) { const int64_t v = part[i]; part[i] = acc; acc += v; }
    rowptr[0] = 0;
  }
  __syncthreads();
  int64_t acc = part[t];
  for (int i = b; i < e; ++i) { acc += rowptr[i + 1]; rowptr[i + 1] = acc; }
}

// 16 threads per patch, one per query: walk the steps in order and list the kept tokens
__global__ void k_csr_fill(const WaveDesc* waves, const int32_t* head_map, int head, int waves_per_hg,
                           const uint64_t* masks, const int32_t* toks, const int64_t* rowptr, int32_t* cols, int64_t cap) {
  const WaveDesc wd = waves[(size_t)head_map[head] * waves_per_hg + blockIdx.x];
  const int n = threadIdx.x;
  const int qrow = patch_query_row(wd, n);
  if (n >= 16 || qrow < 0) return;
  int64_t w = rowptr[qrow];
  const int64_t end = rowptr[qrow + 1];
  for (int s = 0; s < wd.n_steps; ++s) {
    const int64_t S = (int64_t)wd.step_begin + s;
    for (int idx = 0; idx < kStepKeys; ++idx) {
      const int r = idx % 16;
      if (masks[S * 8 + 4 * (idx / 16) + r % 4] >> ((r / 4) * 16 + n) & 1) {
        if (w < end && w < cap) cols[w] = toks[S * kStepKeys + idx];
        ++w;
      }
    }
  }
}

static int head_group_of(const litevar_plan* pl, int head) { return pl->n_heads > 0 ? pl->head_group[head] : 0; }

litevar_status export_window_table(const litevar_plan* pl, int head, int16_t* d_out, hipStream_t st) {
  const BlobPtrs p = blob_ptrs(pl->d_blob, pl->off);
  const int n = pl->n_scales * pl->n_scales * pl->side_max * 2;
  hipLaunchKernelGGL(k_export_win, dim3((n + 255) / 256), dim3(256), 0, st, n,
                     p.win + (size_t)head_group_of(pl, head) * n, d_out);
  return hip_check(hipGetLastError(), "window table export launch");
}

litevar_status export_dense(const litevar_plan* pl, int head, uint8_t* d_mask, uint64_t* d_count,
                            hipStream_t st) {
  const BlobPtrs p = blob_ptrs(pl->d_blob, pl->off);
  const size_t n = (size_t)pl->q_len * pl->kv_len;
  hipLaunchKernelGGL(k_fill_u8, dim3(2048), dim3(256), 0, st, d_mask, n, (uint8_t)0);
  if (d_count) hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(64), 0, st, (unsigned long long*)d_count);
  const int nw = pl->n_groups * pl->waves_per_group;
  hipLaunchKernelGGL(k_export_dense, dim3(nw), dim3(64), 0, st, pl->kv_len, p.waves, p.head_map, head, nw,
                     p.step_mask, p.step_tok, d_mask, (unsigned long long*)d_count);
  return hip_check(hipGetLastError(), "dense mask export launch");
}

litevar_status export_csr(const litevar_plan* pl, int head, int64_t* d_rowptr, int32_t* d_cols, size_t cap,
                          hipStream_t st) {
  const BlobPtrs p = blob_ptrs(pl->d_blob, pl->off);
  const int nw = pl->n_groups * pl->waves_per_group;
  hipLaunchKernelGGL(k_csr_count, dim3(nw), dim3(64), 0, st, p.waves, p.head_map, head, nw, p.step_mask, d_rowptr);
  hipLaunchKernelGGL(k_csr_scan, dim3(1), dim3(1024), 0, st, d_rowptr, pl->q_len);
  hipLaunchKernelGGL(k_csr_fill, dim3(nw), dim3(64), 0, st, p.waves, p.head_map, head, nw, p.step_mask, p.step_tok,
                     d_rowptr, d_cols, (int64_t)cap);
  return hip_check(hipGetLastError(), "csr export launch");
}

litevar_status read_header(const litevar_plan* pl, hipStream_t st, Header& h) {
  litevar_status rc = hip_check(hipStreamSynchronize(st), "hipStreamSynchronize");
  if (rc) return rc;
  return hip_check(hipMemcpy(&h, pl->d_blob, sizeof h, hipMemcpyDeviceToHost), "header copy");
}

}  // namespace lv
