// Window calibration with Section 2, step (2) of the paper read literally (the band mask mode):
// the attention map of query scale k is cut into parts -- the first three key scales together,
// then one part per key scale -- and in every part the window is the band of radius r around
// the part's diagonal, floor((2 i + 1) n / (2 s_k^2)) at query i of a part of n columns; the
// band grows from radius zero until it holds the fraction R_0 of the part's values.
//
// Layout of the work.  A value's distance from the diagonal depends only on its offset
// o = column - diagonal(row), in [-(n - 1), n - 1].  One thread owns one offset of one part and
// walks a block of query rows (and all samples), adding the map's value at (row, diagonal + o)
// where that column exists: consecutive lanes own consecutive offsets, i.e. consecutive columns
// of one map row (a part's columns are consecutive tokens); every value of the map is added
// exactly once, by exactly one thread, in a fixed order in fp64 (no atomics: two launches give
// identical bits).  A second, small kernel adds the row blocks of a part in a fixed order,
// folds offsets +d and -d, forms the in-band sums by prefix and picks the radius.
#include "internal.h"

#include <cstring>

namespace lv {

namespace {

constexpr int kBandThreads = 256;
constexpr int kBandRowBlocks = 16;    // row blocks of a part at most (the rows of a query scale are dealt to them)
constexpr int kMaxPartCols = 4096;    // per-distance sums of a part live in LDS in the pick kernel

struct BandArgs {
  int K, N, H, n_parts, mcols;
  int s[kMaxScales], off[kMaxScales + 1];
  int64_t L, head_stride;             // doubles of partial sums per head
  const float* p;       // [N][H][L][L]
  double* partial;      // per head: for every part, [row blocks][2 n - 1] sums by offset
  int32_t* radius;      // [H][K][K]
  double* mass;         // [H][K][K][mcols] or nullptr
  double r0;
};

__host__ __device__ inline int parts_of(int k) { return k < kMergedScales ? 1 : k - kMergedScales + 2; }
__host__ __device__ inline int row_blocks_of(int nk) { return nk < kBandRowBlocks ? nk : kBandRowBlocks; }

// part `idx` of the launch (parts of query scale 0, then of query scale 1, ...)
struct BandPartInfo {
  int k, first, last;       // query scale, key scales of the part
  int n, nk, tok0;          // columns, query rows, first column's token
  int row_blocks, rows_per_block;
  int64_t base;             // first double of the part's partial sums inside a head's region
  int block0;               // first workgroup of the part in the mass kernel's launch
};
__host__ __device__ inline int blocks_of(int n, int row_blocks) {
  return ((2 * n - 1 + kBandThreads - 1) / kBandThreads) * row_blocks;
}
// (by_block: `idx` is a workgroup of the mass kernel and the part that owns it is wanted)
__host__ __device__ inline BandPartInfo band_part_info(const BandArgs& a, int idx, bool by_block = false) {
  BandPartInfo r = {};
  int64_t base = 0;
  int at = 0, block0 = 0;
  for (int k = 0; k < a.K; ++k) {
    const int nk = a.s[k] * a.s[k], rb = row_blocks_of(nk);
    for (int pt = 0; pt < parts_of(k); ++pt, ++at) {
      const int first = pt == 0 ? 0 : pt + kMergedScales - 1;
      const int last = pt == 0 ? (k < kMergedScales - 1 ? k : kMergedScales - 1) : first;
      const int n = a.off[last + 1] - a.off[first];
      const int nb = blocks_of(n, rb);
      if (by_block ? idx < block0 + nb : at == idx) {
        r.k = k; r.first = first; r.last = last; r.n = n; r.nk = nk; r.tok0 = a.off[first];
        r.row_blocks = rb; r.rows_per_block = (nk + rb - 1) / rb; r.base = base; r.block0 = block0;
        return r;
      }
      base += (int64_t)rb * (2 * n - 1);
      block0 += nb;
    }
  }
  r.k = -1;
  return r;
}

// grid (workgroups of all parts, heads): the launch holds exactly the workgroups that have
// work (starting an empty one costs about as much as a short one); a part's workgroups are
// (row block, tile of 256 offsets)
__global__ __launch_bounds__(kBandThreads) void k_band_mass(BandArgs a) {
  const BandPartInfo pi = band_part_info(a, blockIdx.x, true);
  const int h = blockIdx.y;
  const int n_off = 2 * pi.n - 1, tiles = (n_off + kBandThreads - 1) / kBandThreads;
  const int local = (int)blockIdx.x - pi.block0;
  const int tile = local % tiles, rb = local / tiles;
  const int u = tile * kBandThreads + threadIdx.x;               // offset index: o = u - (n - 1)
  if (u >= n_off) return;
  const int o = u - (pi.n - 1);
  const int i0 = rb * pi.rows_per_block, i1 = min(pi.nk, i0 + pi.rows_per_block);
  const int64_t q0 = a.off[pi.k];
  double acc = 0.0;
  for (int i = i0; i < i1; ++i) {
    // the diagonal at row i, plus o (sides are at most 64: (2 i + 1) n stays below 2^26)
    const int c = (int)(((2u * (unsigned)i + 1u) * (unsigned)pi.n) / (2u * (unsigned)pi.nk)) + o;
    if (c < 0 || c >= pi.n) continue;
    const float* row = a.p + ((int64_t)h * a.L + q0 + i) * a.L + pi.tok0 + c;
    for (int s = 0; s < a.N; ++s) acc += (double)row[(int64_t)s * a.H * a.L * a.L];
  }
  a.partial[(int64_t)h * a.head_stride + pi.base + (int64_t)rb * n_off + u] = acc;
}

// grid (parts, heads): per-distance sums of the part, prefix, radius
__global__ __launch_bounds__(kBandThreads) void k_band_pick(BandArgs a) {
  __shared__ double by_dist[kMaxPartCols];
  const BandPartInfo pi = band_part_info(a, blockIdx.x);
  const int h = blockIdx.y;
  const int n_off = 2 * pi.n - 1;
  const double* part = a.partial + (int64_t)h * a.head_stride + pi.base;
  for (int d = threadIdx.x; d < pi.n; d += kBandThreads) {
    double m = 0.0;
    for (int rb = 0; rb < pi.row_blocks; ++rb) {                 // (fixed order)
      m += part[(int64_t)rb * n_off + (pi.n - 1) + d];
      if (d > 0) m += part[(int64_t)rb * n_off + (pi.n - 1) - d];
    }
    by_dist[d] = m;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double total = 0.0;
    for (int d = 0; d < pi.n; ++d) total += by_dist[d];
    int found = -1;
    double in = 0.0;
    for (int d = 0; d < pi.n; ++d) {                             // the band grows from zero
      in += by_dist[d];
      by_dist[d] = in;                                           // (in-band sum at radius d, for the mass output)
      if (found < 0 && (total == 0.0 || in / total >= a.r0)) found = d;
    }
    if (found < 0) found = pi.n - 1;
    int32_t* rad = a.radius + ((int64_t)h * a.K + pi.k) * a.K;
    for (int j = pi.first; j <= pi.last; ++j) rad[j] = found;
    if (pi.first == 0)                                           // the first part also marks the key scales above k
      for (int j = pi.k + 1; j < a.K; ++j) rad[j] = -1;
  }
  __syncthreads();
  if (a.mass) {
    for (int j = 0; j < a.K; ++j) {
      double* m = a.mass + (((int64_t)h * a.K + pi.k) * a.K + j) * a.mcols;
      if (j >= pi.first && j <= pi.last) {
        for (int r = threadIdx.x; r < a.mcols; r += kBandThreads) m[r] = by_dist[r < pi.n ? r : pi.n - 1];
      } else if (pi.first == 0 && j > pi.k) {
        for (int r = threadIdx.x; r < a.mcols; r += kBandThreads) m[r] = 0.0;
      }
    }
  }
}

litevar_status band_geom(const int32_t* scales, int32_t n_scales, int32_t H, BandArgs& a, int& n_blocks) {
  if (!scales) return fail(LITEVAR_E_INVALID_ARG, "scales is NULL");
  if (n_scales < 1 || n_scales > kMaxScales)
    return fail(LITEVAR_E_INVALID_ARG, "n_scales must be in 1..%d (got %d)", kMaxScales, n_scales);
  if (H < 1 || H > 65535) return fail(LITEVAR_E_INVALID_ARG, "H must be in 1..65535 (got %d)", H);
  std::memset(&a, 0, sizeof a);
  a.K = n_scales; a.H = H;
  int64_t L = 0;
  for (int k = 0; k < n_scales; ++k) {
    if (scales[k] < 1 || scales[k] > 64)
      return fail(LITEVAR_E_UNSUPPORTED, "band calibration takes scale sides 1..64 (got %d)", scales[k]);
    a.s[k] = scales[k]; a.off[k] = (int)L;
    L += (int64_t)scales[k] * scales[k];
  }
  a.off[n_scales] = (int)L;
  a.L = L;
  a.n_parts = 0;
  for (int k = 0; k < n_scales; ++k) a.n_parts += parts_of(k);
  if (a.n_parts > 65535) return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  a.mcols = 0; n_blocks = 0;
  int64_t stride = 0;
  for (int idx = 0; idx < a.n_parts; ++idx) {
    const BandPartInfo pi = band_part_info(a, idx);
    if (pi.n > kMaxPartCols) return fail(LITEVAR_E_UNSUPPORTED, "a part of %d columns (at most %d)", pi.n, kMaxPartCols);
    a.mcols = pi.n > a.mcols ? pi.n : a.mcols;
    n_blocks = pi.block0 + blocks_of(pi.n, pi.row_blocks);     // (running total: all parts' workgroups)
    stride = pi.base + (int64_t)pi.row_blocks * (2 * pi.n - 1);
  }
  a.head_stride = stride;
  return LITEVAR_OK;
}

}  // namespace

}  // namespace lv

using namespace lv;

extern "C" {

litevar_status litevar_window_calibrate_band_workspace_bytes(const int32_t* scales, int32_t n_scales, int32_t H,
                                                             size_t* out_bytes) {
  if (!out_bytes) return fail(LITEVAR_E_INVALID_ARG, "out_bytes is NULL");
  BandArgs a;
  int n_blocks = 0;
  if (litevar_status s = band_geom(scales, n_scales, H, a, n_blocks)) return s;
  *out_bytes = (size_t)a.head_stride * (size_t)H * sizeof(double);
  return LITEVAR_OK;
}

litevar_status litevar_window_calibrate_band(const int32_t* scales, int32_t n_scales, const float* d_attn, int32_t N,
                                             int32_t H, float r0, void* d_workspace, size_t workspace_bytes,
                                             int32_t* d_radius, double* d_mass, void* stream) {
  BandArgs a;
  int n_blocks = 0;
  if (litevar_status s = band_geom(scales, n_scales, H, a, n_blocks)) return s;
  if (N < 1) return fail(LITEVAR_E_INVALID_ARG, "N must be positive");
  if (!(r0 > 0.f) || r0 > 1.f) return fail(LITEVAR_E_INVALID_ARG, "r0 must be in (0, 1] (got %g)", r0);
  if (!d_attn || !d_radius || !d_workspace) return fail(LITEVAR_E_INVALID_ARG, "d_attn, d_radius or d_workspace is NULL");
  if (((uintptr_t)d_workspace & 7) || (d_mass && ((uintptr_t)d_mass & 7)))
    return fail(LITEVAR_E_INVALID_ARG, "d_workspace and d_mass must be 8-byte aligned");
  const size_t need = (size_t)a.head_stride * (size_t)H * sizeof(double);
  if (workspace_bytes < need) return fail(LITEVAR_E_INVALID_ARG, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
  a.N = N; a.p = d_attn; a.partial = (double*)d_workspace; a.radius = d_radius; a.mass = d_mass; a.r0 = (double)r0;
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(k_band_mass, dim3(n_blocks, H), dim3(kBandThreads), 0, st, a);
  if (litevar_status s = hip_check(hipGetLastError(), "band calibration mass launch")) return s;
  hipLaunchKernelGGL(k_band_pick, dim3(a.n_parts, H), dim3(kBandThreads), 0, st, a);
  return hip_check(hipGetLastError(), "band calibration pick launch");
}

}  // extern "C"
