// Internal layout of a LiteVAR windowed-attention plan and the integer geometry
// shared by the host sizing pass and the device builder kernels.
//
// Vocabulary (Section 2 of the paper for scales/parts/windows; the tiling is ours):
//   patch   16 queries of one scale = the 16 columns of one MFMA tile, handled by one
//           64-lane wave: a 4x4 block of the scale's grid (window mode) or 16 consecutive
//           queries (band mode);
//   group   up to NW patches of one query scale handled by one workgroup that
//           stages the keys they need through an LDS ring;
//   union   the group's key list: for every part of the attention map the keys that any of
//           its queries keeps (window mode: the bounding box of the windows in every key
//           scale, row-major; band mode: one column range per part), parts in ascending order;
//   step    32 keys of one patch's own key list (two 16-key MFMA tiles for
//           K Q^T, one K=32 MFMA slice for V^T P^T) with one mask bit per
//           (query, key);
//   phase   the group processes the union list in chunks of C keys; a step is
//           run in the phase of its last key and may reach back A chunks;
//   head group   heads that share one radius table share one set of groups, lists and steps.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define LV_HD __host__ __device__ inline

namespace lv {

constexpr int kMaxScales = 32;
constexpr int kMaxSide = 1024;
constexpr int kMaxRadius = 32767;    // radii are stored as int16 (band mode counts columns of a part)
constexpr int kMaxHeads = 256;       // heads with their own radius table
constexpr int kStepKeys = 32;
constexpr int kPatch = 4;
constexpr int kPatchQueries = 16;
constexpr int kMergedScales = 3;     // band mode: the first part spans the first three scales
constexpr uint64_t kMagic = 0x4c56415257494e32ull;  // "LVARWIN2"

enum MaskMode { kModeWindow = 0, kModeBand = 1 };

struct Geom {
  int K, qb, qe, n_sink;
  int L, Lq, q0, smax;
  int NW;               // patches per group
  short grh[kMaxScales], grw[kMaxScales];   // window mode: group shape in patches (grh x grw <= NW) of every query scale
  int C, NR, A, D;      // chunk keys (a power of two), ring depth in chunks, look-back and
                        // prefetch depth in chunks; NR = A + 1 + D
  int logC;
  int logS;             // a step spans at most A + 1 consecutive blocks of 2^logS keys (logS <= logC)
  int R;                // ring slots
  int n_groups, n_patches;   // per head group
  int mode;             // MaskMode
  int n_hg;             // head groups (1 unless the plan has one radius table per head)
  int s[kMaxScales];
  int off[kMaxScales + 1];
  short rad[kMaxScales][kMaxScales];   // radii of ONE head group, [query scale][key scale]
                                       // (Section 2, step (3): one window size per scale and
                                       // part); < 0: dense part.  The host sizes one head
                                       // group at a time; on the device only the kernel that
                                       // writes the tables reads this field.
  int grp_off[kMaxScales + 1];  // groups are ordered by DESCENDING query scale:
                                // slot i holds scale qe-1-i; grp_off is its prefix sum
};

struct GroupDesc {   // 32 bytes
  int32_t union_base;  // first entry in union_tok
  int32_t n_union;     // real keys
  int32_t n_phases;    // ceil(n_union / C), >= 1
  int32_t k;           // query scale
  int32_t gy, gx;      // group position in units of groups (band mode: gy = index in the scale, gx = 0)
  int32_t phase_base;  // first entry in phase_end (NW * n_phases int32 entries, wave-major)
  int32_t ident;       // union entries [0, ident) hold token i at position i
};

struct WaveDesc {    // 32 bytes
  int32_t step_begin;
  int32_t n_steps;
  int32_t q_base;      // local query row of the patch's first query
  int16_t sk;          // query n of the patch is row q_base + (n / 4) * sk + n % 4
  int16_t ny, nx;      // valid extent of the patch (0 = idle wave); band mode: (1, number of queries)
  int16_t kq;          // query scale index
  int32_t pairs;       // kept pairs of this patch (statistics)
  uint32_t valid;      // bit n set: column n of the patch holds a query
  uint32_t first_ends; // phase_end[0] | phase_end[min(2, n_phases - 1)] << 16: the step counts that the
                       // 16-patch kernel needs before it can start, next to the patch's other words
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
                       // kErrWaitGaveUp: an attention kernel's bounded wait on an LDS flag ran out;
                       // kErrBounds: a kernel of the bounds-checking build found a token, a query
                       // row or an LDS offset out of range (it used index 0 instead)
  int32_t pad0;
  uint64_t pad[24];
};
static_assert(sizeof(Header) == 256, "header size");

enum HeaderError { kErrNone = 0, kErrBuilder = 1, kErrWaitGaveUp = 2, kErrBounds = 3 };
constexpr int kDefaultSpinLimit = 1 << 22;   // polls of about 64 cycles each

enum Section { kSecHeader = 0, kSecWin, kSecRad, kSecHeadMap, kSecGroups, kSecWaves, kSecPhaseEnd,
               kSecUnion, kSecStepAddr, kSecStepMask, kSecStepTok, kSecEnd, kNumSections };

// LDS ring geometry of the bf16 kernel: one 128-byte row per key in each of the K and V
// rings; the 16-byte piece c of the row in slot s is stored at piece position
// c ^ swizzle(s).
constexpr int kRingRowBytes = 128;
LV_HD unsigned ring_swizzle(unsigned slot) { return (slot ^ (slot >> 3)) & 7u; }

// ---- window definition (window mode) -------------------------------------------
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

// Where the builder takes its intervals from: the arithmetic above (host sizing, and the
// kernel that writes the device table) or the device table (every other builder kernel).
struct ArithWin {
  const Geom& g;
  LV_HD Interval operator()(int k, int j, int c) const { return win_interval(g, k, j, c); }
};
struct TableWin {        // win[((k * K + j) * smax + c) * 2 + {0, 1}] of one head group
  const int16_t* win; int K, smax;
  LV_HD Interval operator()(int k, int j, int c) const {
    const int16_t* p = win + ((size_t)(k * K + j) * smax + c) * 2;
    Interval iv; iv.lo = p[0]; iv.hi = p[1];
    return iv;
  }
};

// ---- band mode (Section 2, step (2), read literally) -----------------------------
// The attention map of query scale k, [s_k^2, sum_{i<=k} s_i^2], is cut into parts: the
// first spans the first three key scales (as many of them as the query sees), every later
// key scale is a part of its own.  In a part of n columns query i (flattened, row-major)
// keeps the columns within `radius` of the part's diagonal, floor((2 i + 1) n / (2 s_k^2)).
LV_HD int band_parts(int k) { return k < kMergedScales ? 1 : k - kMergedScales + 2; }
LV_HD int band_part_first(int p) { return p == 0 ? 0 : p + kMergedScales - 1; }
LV_HD int band_part_last(int k, int p) {
  return p == 0 ? (k < kMergedScales - 1 ? k : kMergedScales - 1) : p + kMergedScales - 1;
}

struct BandPart { int tok0, cols, rad; };   // first token, columns, radius (< 0: dense)

template <class Rad>   // Rad(k, j) -> radius of (query scale k, key scale j)
LV_HD BandPart band_part(const Geom& g, const Rad& rad, int k, int p) {
  const int first = band_part_first(p), last = band_part_last(k, p);
  BandPart b;
  b.tok0 = g.off[first]; b.cols = g.off[last + 1] - g.off[first];
  b.rad = last < g.n_sink ? -1 : rad(k, last);
  return b;
}

LV_HD Interval band_interval(const BandPart& b, int nk, int i) {
  Interval iv;
  if (b.rad < 0) { iv.lo = 0; iv.hi = b.cols - 1; return iv; }
  const int ctr = (int)(((uint64_t)(2 * (int64_t)i + 1) * (uint64_t)b.cols) / (uint64_t)(2 * (int64_t)nk));
  iv.lo = ctr - b.rad < 0 ? 0 : ctr - b.rad;
  iv.hi = ctr + b.rad > b.cols - 1 ? b.cols - 1 : ctr + b.rad;
  return iv;
}

struct ArithRad { const Geom& g; LV_HD int operator()(int k, int j) const { return g.rad[k][j]; } };
struct TableRad { const int16_t* rad; int K; LV_HD int operator()(int k, int j) const { return rad[k * K + j]; } };

// ---- groups and patches ------------------------------------------------------------
// Shape (rows x columns of patches, at most nw patches) of the groups that tile a grid of
// pps x pps patches: the fewest groups; among those the most compact shape (a group streams
// the bounding box of its queries' windows), then the taller one.
inline void choose_group_shape(int pps, int nw, int& rh, int& rw) {
  long best = -1;
  rh = 1; rw = 1;
  for (int h = 1; h <= nw && h <= pps; ++h) {
    int w = nw / h; if (w > pps) w = pps;
    const long groups = (long)((pps + h - 1) / h) * ((pps + w - 1) / w);
    const long key = groups * 4096 + (h + w) * 32 + (32 - h);
    if (best < 0 || key < best) { best = key; rh = h; rw = w; }
  }
}

LV_HD int patches_per_side(const Geom& g, int k) { return (g.s[k] + kPatch - 1) / kPatch; }
LV_HD int scale_patches(const Geom& g, int k) {
  if (g.mode == kModeBand) return (g.s[k] * g.s[k] + kPatchQueries - 1) / kPatchQueries;
  return patches_per_side(g, k) * patches_per_side(g, k);
}
LV_HD int groups_y(const Geom& g, int k) {
  if (g.mode == kModeBand) return (scale_patches(g, k) + g.NW - 1) / g.NW;
  return (patches_per_side(g, k) + g.grh[k] - 1) / g.grh[k];
}
LV_HD int groups_x(const Geom& g, int k) {
  if (g.mode == kModeBand) return 1;
  return (patches_per_side(g, k) + g.grw[k] - 1) / g.grw[k];
}

// group index (inside a head group) -> (query scale, gy, gx)
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
template <class Win>
LV_HD Box window_box(const Win& win, int k, int j, int qy0, int qy1, int qx0, int qx1) {
  Box b;
  b.ylo = win(k, j, qy0).lo; b.yhi = win(k, j, qy1).hi;
  b.xlo = win(k, j, qx0).lo; b.xhi = win(k, j, qx1).hi;
  return b;
}

// valid queries of a group: rows/cols of the scale's grid (window mode) or the flattened
// query range [qy0, qy1] (band mode; qx0 = qx1 = 0)
struct GroupExtent { int k, qy0, qy1, qx0, qx1; };

LV_HD GroupExtent group_extent(const Geom& g, int k, int gy, int gx) {
  GroupExtent e; e.k = k;
  if (g.mode == kModeBand) {
    const int nk = g.s[k] * g.s[k];
    e.qy0 = gy * g.NW * kPatchQueries;
    e.qy1 = e.qy0 + g.NW * kPatchQueries - 1; if (e.qy1 > nk - 1) e.qy1 = nk - 1;
    e.qx0 = e.qx1 = 0;
    return e;
  }
  e.qy0 = gy * g.grh[k] * kPatch; e.qx0 = gx * g.grw[k] * kPatch;
  e.qy1 = e.qy0 + g.grh[k] * kPatch - 1; if (e.qy1 > g.s[k] - 1) e.qy1 = g.s[k] - 1;
  e.qx1 = e.qx0 + g.grw[k] * kPatch - 1; if (e.qx1 > g.s[k] - 1) e.qx1 = g.s[k] - 1;
  return e;
}

// window mode: (y0, x0) corner and ny x nx valid queries; band mode: y0 = first flattened
// query, nx = number of queries, ny = 1.  ny == 0: no such patch (idle wave)
struct PatchExtent { int y0, x0, ny, nx; };

LV_HD PatchExtent patch_extent(const Geom& g, int k, int gy, int gx, int wave) {
  PatchExtent p;
  const int sk = g.s[k];
  if (g.mode == kModeBand) {
    p.y0 = (gy * g.NW + wave) * kPatchQueries; p.x0 = 0;
    const int left = sk * sk - p.y0;
    if (wave >= g.NW || left <= 0) { p.ny = p.nx = 0; return p; }
    p.ny = 1; p.nx = left < kPatchQueries ? left : kPatchQueries;
    return p;
  }
  const int rh = g.grh[k], rw = g.grw[k];
  const int py = gy * rh + wave / rw, px = gx * rw + wave % rw;
  p.y0 = py * kPatch; p.x0 = px * kPatch;
  if (wave >= rh * rw || p.y0 >= sk || p.x0 >= sk) { p.ny = p.nx = 0; return p; }
  p.ny = sk - p.y0 < kPatch ? sk - p.y0 : kPatch;
  p.nx = sk - p.x0 < kPatch ? sk - p.x0 : kPatch;
  return p;
}

// descriptor fields of a patch: first local query row, row stride of the 4x4 arrangement,
// and the columns that hold a query
LV_HD void patch_queries(const Geom& g, int k, const PatchExtent& p, int& q_base, int& sk, uint32_t& valid) {
  valid = 0;
  if (g.mode == kModeBand) {
    q_base = g.off[k] - g.q0 + p.y0; sk = kPatch;
    valid = p.ny ? (p.nx >= kPatchQueries ? 0xffffu : ((1u << p.nx) - 1u)) : 0u;
    return;
  }
  q_base = g.off[k] - g.q0 + p.y0 * g.s[k] + p.x0; sk = g.s[k];
  for (int n = 0; n < kPatchQueries; ++n)
    if (n / kPatch < p.ny && n % kPatch < p.nx) valid |= 1u << n;
}

LV_HD int popcount32(unsigned v) { return __builtin_popcount(v); }

// ---- the serial walk (host sizing; the device runs a wave-cooperative form of it) -------
// Visits the key list of one patch in order and packs it into steps.  Sink receives
//   key(step, idx_in_step, upos, token, qmask16)   for every kept key, and
//   close(step, n_keys, last_upos)                 when a step is complete.
// qmask16 bit n is set iff query n of the patch keeps the key.
// A step is closed when it holds 32 keys or when the next key's 2^logS-key block lies more
// than A blocks after the block of the step's first key (LDS ring constraint).
template <class Sink>
struct StepPacker {
  const Geom& g; Sink& sink;
  int step = 0, cnt = 0, first_chunk = 0, last_upos = 0;
  LV_HD void key(int upos, int tok, unsigned qmask) {
    const int chunk = upos >> g.logS;
    if (cnt == kStepKeys || (cnt > 0 && chunk - first_chunk > g.A)) { sink.close(step, cnt, last_upos); ++step; cnt = 0; }
    if (cnt == 0) first_chunk = chunk;
    sink.key(step, cnt, upos, tok, qmask);
    ++cnt; last_upos = upos;
  }
  LV_HD int finish() {
    if (cnt > 0) { sink.close(step, cnt, last_upos); ++step; cnt = 0; }
    return step;
  }
};

// number of keys of a group's union list
template <class Win, class Rad>
LV_HD int group_union_keys(const Geom& g, const Win& win, const Rad& rad, const GroupExtent& e) {
  int n = 0;
  if (g.mode == kModeBand) {
    const int nk = g.s[e.k] * g.s[e.k];
    for (int p = 0; p < band_parts(e.k); ++p) {
      const BandPart b = band_part(g, rad, e.k, p);
      n += band_interval(b, nk, e.qy1).hi - band_interval(b, nk, e.qy0).lo + 1;
    }
    return n;
  }
  for (int j = 0; j <= e.k; ++j) {
    const Box b = window_box(win, e.k, j, e.qy0, e.qy1, e.qx0, e.qx1);
    n += (b.yhi - b.ylo + 1) * (b.xhi - b.xlo + 1);
  }
  return n;
}

// Returns the number of steps.
template <class Sink>
inline int walk_patch(const Geom& g, const GroupExtent& e, const PatchExtent& p, Sink& sink) {
  if (p.ny == 0) return 0;
  StepPacker<Sink> pack{g, sink};
  const ArithWin win{g};
  const ArithRad rad{g};
  int ubase = 0;
  if (g.mode == kModeBand) {
    const int nk = g.s[e.k] * g.s[e.k];
    for (int pt = 0; pt < band_parts(e.k); ++pt) {
      const BandPart b = band_part(g, rad, e.k, pt);
      const int glo = band_interval(b, nk, e.qy0).lo, ghi = band_interval(b, nk, e.qy1).hi;
      Interval iv[kPatchQueries];
      for (int n = 0; n < kPatchQueries; ++n) {
        iv[n].lo = 1; iv[n].hi = 0;
        if (n < p.nx) iv[n] = band_interval(b, nk, p.y0 + n);
      }
      for (int c = iv[0].lo; c <= iv[p.nx - 1].hi; ++c) {
        unsigned qmask = 0;
        for (int n = 0; n < kPatchQueries; ++n) qmask |= (unsigned)(c >= iv[n].lo && c <= iv[n].hi) << n;
        if (qmask) pack.key(ubase + c - glo, b.tok0 + c, qmask);
      }
      ubase += ghi - glo + 1;
    }
    return pack.finish();
  }
  for (int j = 0; j <= e.k; ++j) {
    const Box gb = window_box(win, e.k, j, e.qy0, e.qy1, e.qx0, e.qx1);
    const int gw = gb.xhi - gb.xlo + 1;
    const Box pb = window_box(win, e.k, j, p.y0, p.y0 + p.ny - 1, p.x0, p.x0 + p.nx - 1);
    const int sj = g.s[j], offj = g.off[j];
    const Interval none = {1, 0};
    Interval rw[kPatch], cw[kPatch];
    for (int d = 0; d < kPatch; ++d) {
      rw[d] = d < p.ny ? win(e.k, j, p.y0 + d) : none;
      cw[d] = d < p.nx ? win(e.k, j, p.x0 + d) : none;
    }
    for (int y = pb.ylo; y <= pb.yhi; ++y) {
      unsigned rb = 0;
      for (int d = 0; d < kPatch; ++d) rb |= (unsigned)(y >= rw[d].lo && y <= rw[d].hi) << d;
      if (!rb) continue;
      const unsigned rowmask = ((rb & 1) ? 0x000fu : 0u) | ((rb & 2) ? 0x00f0u : 0u) |
                               ((rb & 4) ? 0x0f00u : 0u) | ((rb & 8) ? 0xf000u : 0u);
      const int urow = ubase + (y - gb.ylo) * gw - gb.xlo, trow = offj + y * sj;
      for (int x = pb.xlo; x <= pb.xhi; ++x) {
        unsigned cb = 0;
        for (int d = 0; d < kPatch; ++d) cb |= (unsigned)(x >= cw[d].lo && x <= cw[d].hi) << d;
        if (!cb) continue;
        pack.key(urow + x, trow + x, (cb * 0x1111u) & rowmask);
      }
    }
    ubase += (gb.yhi - gb.ylo + 1) * gw;
  }
  return pack.finish();
}

struct CountSink {
  int64_t pairs = 0;
  LV_HD void key(int, int, int, int, unsigned qmask) { pairs += popcount32(qmask); }
  LV_HD void close(int, int, int) {}
};

}  // namespace lv
