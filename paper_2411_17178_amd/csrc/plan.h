// Internal layout of a LiteVAR windowed-attention plan and the integer geometry
// shared by the host sizing pass and the device builder kernels.
//
// Vocabulary (Section 2 of the paper for scales/parts/windows; the tiling is ours):
//   patch   4x4 block of queries of one scale = the 16 columns of one MFMA tile,
//           handled by one 64-lane wave;
//   group   up to NW patches of one query scale handled by one workgroup that
//           stages the keys they need through an LDS ring;
//   union   the group's key list: for every key scale j <= k the bounding box of
//           the windows of all its queries, row-major, scales in ascending order;
//   step    32 keys of one patch's own key list (two 16-key MFMA tiles for
//           K Q^T, one K=32 MFMA slice for V^T P^T) with one mask bit per
//           (query, key);
//   phase   the group processes the union list in chunks of C keys; a step is
//           run in the phase of its last key and may reach back A chunks.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define LV_HD __host__ __device__ inline

namespace lv {

constexpr int kMaxScales = 32;
constexpr int kMaxSide = 1024;
constexpr int kStepKeys = 32;
constexpr int kPatch = 4;
constexpr uint64_t kMagic = 0x4c56415257494e31ull;  // "LVARWIN1"


struct Geom {
  int K, qb, qe, n_sink;
  int L, Lq, q0, smax;
  int NW, RH, RW;       // patches per group; group shape in patches (RH x RW)
  int C, NR, A, D;      // chunk keys (a power of two), ring depth in chunks, look-back and
                        // prefetch depth in chunks; NR = A + 1 + D
  int logC;
  int logS;             // a step spans at most A + 1 consecutive blocks of 2^logS keys (logS <= logC)
  int R;                // ring slots
  int n_groups, n_patches;
  int s[kMaxScales];
  int off[kMaxScales + 1];
  short rad[kMaxScales][kMaxScales];   // [query scale][key scale] (Section 2, step (3): one
                                       // window size per scale and part); < 0: dense part
  int grp_off[kMaxScales + 1];  // groups are ordered by DESCENDING query scale:
                                // slot i holds scale qe-1-i; grp_off is its prefix sum
};

struct GroupDesc {   // 32 bytes
  int32_t union_base;  // first entry in union_tok
  int32_t n_union;     // real keys
  int32_t n_phases;    // ceil(n_union / C), >= 1
  int32_t k;           // query scale
  int32_t gy, gx;      // group position in units of groups
  int32_t phase_base;  // first entry in phase_end (NW * n_phases int32 entries, wave-major)
  int32_t ident;       // union entries [0, ident) hold token i at position i
};

struct WaveDesc {    // 32 bytes
  int32_t step_begin;
  int32_t n_steps;
  int32_t q_base;      // local query row of the patch's (0,0) corner
  int16_t sk;          // query scale side = row stride of the patch in query rows
  int16_t ny, nx;      // valid extent of the patch (0 = idle wave)
  int16_t kq;          // query scale index
  int32_t pairs;       // kept pairs of this patch (statistics)
  int32_t pad[2];
};
static_assert(sizeof(WaveDesc) == 32 && sizeof(GroupDesc) == 32, "descriptor size");

struct Header {      // first 256 bytes of the blob
  uint64_t magic;
  uint64_t blob_bytes;
  int32_t n_groups, n_waves;
  int64_t n_steps, n_union, n_phase_entries;
  int64_t retained_pairs;
  int32_t error;       // kErrBuilder: set by the builder when a capacity would be exceeded (the
                       // work-list sections are then not written and no kernel uses the plan);
                       // kErrWaitGaveUp: an attention kernel's bounded wait on an LDS flag ran out
  int32_t pad0;
  uint64_t pad[24];
};
static_assert(sizeof(Header) == 256, "header size");

enum HeaderError { kErrNone = 0, kErrBuilder = 1, kErrWaitGaveUp = 2 };
constexpr int kDefaultSpinLimit = 1 << 22;   // polls of about 64 cycles each

enum Section { kSecHeader = 0, kSecWin, kSecGroups, kSecWaves, kSecPhaseEnd, kSecUnion,
               kSecStepAddr, kSecStepMask, kSecStepTok, kSecEnd, kNumSections };

// LDS ring geometry of the bf16 kernel: one 128-byte row per key in each of the K and V
// rings; the 16-byte piece c of the row in slot s is stored at piece position
// c ^ swizzle(s), so that 16 lanes reading one piece column of 16 consecutive slots
// touch 16 different bank groups.
constexpr int kRingRowBytes = 128;
LV_HD unsigned ring_swizzle(unsigned slot) { return (slot ^ (slot >> 3)) & 7u; }

// ---- window definition -------------------------------------------------------
// Inclusive interval of key coordinates of scale j kept along one axis by query
// coordinate c of scale k: centre = floor((2c+1) s_j / (2 s_k)), radius r, clipped.
struct Interval { int lo, hi; };   // empty when hi < lo

LV_HD Interval win_interval(const Geom& g, int k, int j, int c) {
  const int sj = g.s[j];
  Interval iv;
  const int rad = g.rad[k][j];
  if (j < g.n_sink || rad < 0) { iv.lo = 0; iv.hi = sj - 1; return iv; }
  // (sides are at most kMaxSide = 1024, so the product fits 32 bits: a 64-bit division would
  // cost an order of magnitude more on the device)
  const int ctr = (int)((unsigned)((2 * c + 1) * sj) / (unsigned)(2 * g.s[k]));
  iv.lo = ctr - rad < 0 ? 0 : ctr - rad;
  iv.hi = ctr + rad > sj - 1 ? sj - 1 : ctr + rad;
  return iv;
}

LV_HD int patches_per_side(const Geom& g, int k) { return (g.s[k] + kPatch - 1) / kPatch; }
LV_HD int groups_y(const Geom& g, int k) { return (patches_per_side(g, k) + g.RH - 1) / g.RH; }
LV_HD int groups_x(const Geom& g, int k) { return (patches_per_side(g, k) + g.RW - 1) / g.RW; }

// group index -> (query scale, gy, gx)
LV_HD void group_coords(const Geom& g, int grp, int& k, int& gy, int& gx) {
  int i = 0;
  while (i + 1 < g.qe - g.qb && grp >= g.grp_off[i + 1]) ++i;
  k = g.qe - 1 - i;
  const int local = grp - g.grp_off[i];
  const int nx = groups_x(g, k);
  gy = local / nx; gx = local % nx;
}

struct Box { int ylo, yhi, xlo, xhi; };  // inclusive; empty when yhi < ylo

// bounding box in key scale j of the windows of query rows [qy0, qy1] x cols [qx0, qx1]
LV_HD Box window_box(const Geom& g, int k, int j, int qy0, int qy1, int qx0, int qx1) {
  Box b;
  b.ylo = win_interval(g, k, j, qy0).lo; b.yhi = win_interval(g, k, j, qy1).hi;
  b.xlo = win_interval(g, k, j, qx0).lo; b.xhi = win_interval(g, k, j, qx1).hi;
  return b;
}

struct GroupExtent { int k, qy0, qy1, qx0, qx1; };  // valid query rows/cols of a group

LV_HD GroupExtent group_extent(const Geom& g, int k, int gy, int gx) {
  GroupExtent e; e.k = k;
  e.qy0 = gy * g.RH * kPatch; e.qx0 = gx * g.RW * kPatch;
  e.qy1 = e.qy0 + g.RH * kPatch - 1; if (e.qy1 > g.s[k] - 1) e.qy1 = g.s[k] - 1;
  e.qx1 = e.qx0 + g.RW * kPatch - 1; if (e.qx1 > g.s[k] - 1) e.qx1 = g.s[k] - 1;
  return e;
}

LV_HD int group_union_keys(const Geom& g, const GroupExtent& e) {
  int n = 0;
  for (int j = 0; j <= e.k; ++j) {
    const Box b = window_box(g, e.k, j, e.qy0, e.qy1, e.qx0, e.qx1);
    n += (b.yhi - b.ylo + 1) * (b.xhi - b.xlo + 1);
  }
  return n;
}

struct PatchExtent { int y0, x0, ny, nx; };  // ny == 0: no such patch (idle wave)

LV_HD PatchExtent patch_extent(const Geom& g, int k, int gy, int gx, int wave) {
  PatchExtent p;
  const int py = gy * g.RH + wave / g.RW, px = gx * g.RW + wave % g.RW;
  p.y0 = py * kPatch; p.x0 = px * kPatch;
  const int sk = g.s[k];
  if (wave >= g.RH * g.RW || p.y0 >= sk || p.x0 >= sk) { p.ny = p.nx = 0; return p; }
  p.ny = sk - p.y0 < kPatch ? sk - p.y0 : kPatch;
  p.nx = sk - p.x0 < kPatch ? sk - p.x0 : kPatch;
  return p;
}

// Walks the key list of one patch in visiting order (key scale, row, column) and
// packs it into steps.  Sink receives
//   key(step, idx_in_step, upos, token, qmask16)   for every kept key, and
//   close(step, n_keys, last_upos)                 when a step is complete.
// qmask16 bit (4*dy + dx) is set iff query (y0+dy, x0+dx) keeps the key.
// A step is closed when it holds 32 keys or when the next key's 2^logS-key block lies more
// than A blocks after the block of the step's first key (LDS ring constraint).
// Returns the number of steps.
template <class Sink>
LV_HD int walk_patch(const Geom& g, const GroupExtent& e, const PatchExtent& p, Sink& sink) {
  if (p.ny == 0) return 0;
  const int logS = g.logS, A = g.A;
  int step = 0, cnt = 0, first_chunk = 0, last_upos = 0, ubase = 0;
  for (int j = 0; j <= e.k; ++j) {
    const Box gb = window_box(g, e.k, j, e.qy0, e.qy1, e.qx0, e.qx1);
    const int gw = gb.xhi - gb.xlo + 1;
    const Box pb = window_box(g, e.k, j, p.y0, p.y0 + p.ny - 1, p.x0, p.x0 + p.nx - 1);
    const int sj = g.s[j], offj = g.off[j];
    const Interval none = {1, 0};
    Interval rw[kPatch], cw[kPatch];
#pragma unroll
    for (int d = 0; d < kPatch; ++d) {
      rw[d] = d < p.ny ? win_interval(g, e.k, j, p.y0 + d) : none;
      cw[d] = d < p.nx ? win_interval(g, e.k, j, p.x0 + d) : none;
    }
    for (int y = pb.ylo; y <= pb.yhi; ++y) {
      unsigned rb = 0;
#pragma unroll
      for (int d = 0; d < kPatch; ++d) rb |= (unsigned)(y >= rw[d].lo && y <= rw[d].hi) << d;
      if (!rb) continue;
      const unsigned rowmask = ((rb & 1) ? 0x000fu : 0u) | ((rb & 2) ? 0x00f0u : 0u) |
                               ((rb & 4) ? 0x0f00u : 0u) | ((rb & 8) ? 0xf000u : 0u);
      const int urow = ubase + (y - gb.ylo) * gw - gb.xlo, trow = offj + y * sj;
      for (int x = pb.xlo; x <= pb.xhi; ++x) {
        unsigned cb = 0;
#pragma unroll
        for (int d = 0; d < kPatch; ++d) cb |= (unsigned)(x >= cw[d].lo && x <= cw[d].hi) << d;
        if (!cb) continue;
        const unsigned qmask = (cb * 0x1111u) & rowmask;
        const int upos = urow + x;
        const int chunk = upos >> logS;
        if (cnt == kStepKeys || (cnt > 0 && chunk - first_chunk > A)) {
          sink.close(step, cnt, last_upos);
          ++step; cnt = 0;
        }
        if (cnt == 0) first_chunk = chunk;
        sink.key(step, cnt, upos, trow + x, qmask);
        ++cnt; last_upos = upos;
      }
    }
    ubase += (gb.yhi - gb.ylo + 1) * gw;
  }
  if (cnt > 0) { sink.close(step, cnt, last_upos); ++step; }
  return step;
}

LV_HD int popcount32(unsigned v) { return __builtin_popcount(v); }

struct CountSink {
  int64_t pairs = 0;
  LV_HD void key(int, int, int, int, unsigned qmask) { pairs += popcount32(qmask); }
  LV_HD void close(int, int, int) {}
};

}  // namespace lv
