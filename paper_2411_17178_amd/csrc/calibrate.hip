// Window calibration (paper Section 2: the metric R_w and the threshold R_0): from a
// post-softmax attention map, the smallest window radius per (head, query scale, key scale)
// whose window holds the fraction R_0 of the part's values.
//
// Layout of the work.  In a part (query scale k, key scale j) a key's distance from the
// window centre depends only on its offset (oy, ox) from that centre, and so does every
// window it belongs to: radius r holds the offsets with max(|oy|, |ox|) <= r.  One thread
// owns one offset and walks all queries of the part, adding the map's value at
// (query, centre + offset) where that key exists: consecutive lanes own consecutive ox, so a
// wave reads runs of consecutive keys of one map row; every value of the map is added exactly
// once per launch, by exactly one thread, in a fixed order in fp64 (no atomics: two launches
// give identical bits).  (Measured alternatives, both slower: copying the reachable key rows
// to LDS with coalesced loads and picking from there -- two barriers per batch of queries,
// 2.4 times slower; one thread per key with a private LDS column of per-distance sums --
// fully coalesced loads, but a dependent LDS read-add-write per value, 2 times slower.)  The (sample, query row) pairs of a part are dealt to
// `splits` workgroups per 256 offsets, so that small maps still fill the GPU.  A workgroup
// folds its 256 offsets into per-distance sums (fixed order again) and writes them to the
// workspace; a second, small kernel adds the workgroups of a part, forms the in-window sums
// by prefix and picks the radius.
#include "internal.h"

#include <mutex>

namespace lv {

namespace {

constexpr int kCalibThreads = 256;

struct CalibArgs {
  int K, N, H, smax, max_tiles, splits;
  int s[kMaxScales], off[kMaxScales + 1];
  int64_t L;
  uint16_t slot_begin[kMaxScales * kMaxScales + 1];   // first workgroup of part k * K + j in a head's launch
                                                      // (splits * tiles of the part's key scale each; none for j > k)
  int n_slots;
  const float* p;       // [N][H][L][L]
  double* partial;      // [H][K][K][splits][max_tiles][smax]: per-distance sums of one workgroup
  int32_t* radius;      // [H][K][K]
  double* mass;         // [H][K][K][smax] or nullptr
  double r0;
};

__host__ __device__ inline int tiles_of(int sj) {
  const int w = 2 * sj - 1;
  return (w * w + kCalibThreads - 1) / kCalibThreads;
}

// Which part and which of its workgroups a block is: the launch has one block per
// (part with j <= k, split, tile of the part's key scale) and nothing else -- a launch over
// the full (tiles x splits, K x K) rectangle spends most of its time starting workgroups
// that have nothing to do.
struct Slot { int k, j, tile, split; };
__device__ inline Slot decode_slot(const CalibArgs& a, int b) {
  int lo = 0, hi = a.K * a.K;                 // last part whose first workgroup is <= b
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.slot_begin[mid] <= b) lo = mid; else hi = mid;
  }
  Slot s;
  s.k = lo / a.K; s.j = lo % a.K;
  const int local = b - a.slot_begin[lo], nt = tiles_of(a.s[s.j]);
  s.tile = local % nt; s.split = local / nt;
  return s;
}

// grid (n_slots, 1, H)
__global__ __launch_bounds__(kCalibThreads) void k_calib_mass(CalibArgs a) {
  const Slot sl = decode_slot(a, blockIdx.x);
  const int k = sl.k, j = sl.j, h = blockIdx.z, tile = sl.tile, split = sl.split;
  const int sk = a.s[k], sj = a.s[j];
  __shared__ short cen[kMaxSide];          // centre of query coordinate c in key scale j
  __shared__ double sum_of[kCalibThreads];
  __shared__ short dist_of[kCalibThreads];
  __shared__ double sub_of[16][17];        // fold, first level: 16 distances x 16 runs of 16 threads
  for (int c = threadIdx.x; c < sk; c += kCalibThreads)
    cen[c] = (short)(((2 * c + 1) * sj) / (2 * sk));
  __syncthreads();

  const int w = 2 * sj - 1, o = tile * kCalibThreads + threadIdx.x;
  const bool live = o < w * w;
  const int oy = live ? o / w - (sj - 1) : 0, ox = live ? o % w - (sj - 1) : 0;
  // Eight loads in flight per thread: every load is unconditional, from the key column
  // clamped into the row (a value outside the row's keys is read and then not added), and
  // feeds its own running sum; the order of the additions is fixed.
  constexpr int U = 8;
  double acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u) acc[u] = 0.0;
  if (live) {
    const float* part = a.p + (int64_t)h * a.L * a.L + (int64_t)a.off[k] * a.L + a.off[j];
    for (int r = split; r < a.N * sk; r += a.splits) {     // (sample, query row) pairs of this split
      const int n = r / sk, qy = r % sk;
      const int ky = cen[qy] + oy;
      if (ky < 0 || ky >= sj) continue;
      const float* row = part + (int64_t)n * a.H * a.L * a.L + (int64_t)qy * sk * a.L + ky * sj;
      for (int qx = 0; qx < sk; qx += U) {
        float v[U];
        bool in[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int q = min(qx + u, sk - 1);               // (past the last query: re-read it, not added)
          const int kx = cen[q] + ox;
          in[u] = qx + u < sk && kx >= 0 && kx < sj;
          v[u] = row[(int64_t)q * a.L + min(max(kx, 0), sj - 1)];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] += in[u] ? (double)v[u] : 0.0;
      }
    }
  }
  double total = 0.0;
#pragma unroll
  for (int u = 0; u < U; ++u) total += acc[u];
  sum_of[threadIdx.x] = total;
  dist_of[threadIdx.x] = live ? (short)max(abs(oy), abs(ox)) : (short)-1;
  __syncthreads();
  double* out = a.partial +
      (((((int64_t)h * a.K + k) * a.K + j) * a.splits + split) * a.max_tiles + tile) * a.smax;
  // per-distance sums over the 256 threads, in a fixed order: 16 distances at a time, thread
  // (d, c) adds run c (16 consecutive threads), then thread (d, 0) adds the 16 runs
  const int dl = threadIdx.x >> 4, c = threadIdx.x & 15;
  for (int d0 = 0; d0 < sj; d0 += 16) {
    double s = 0.0;
    for (int i = 16 * c; i < 16 * c + 16; ++i)
      if (dist_of[i] == d0 + dl) s += sum_of[i];
    sub_of[dl][c] = s;
    __syncthreads();
    if (c == 0 && d0 + dl < sj) {
      double t = 0.0;
      for (int i = 0; i < 16; ++i) t += sub_of[dl][i];
      out[d0 + dl] = t;
    }
    __syncthreads();
  }
}

// The same sums for maps whose largest side is at most kRowsMaxSide, one map row at a time.
// Same grid and same partial-sum slots as k_calib_mass, but a workgroup owns a share of the
// part's (sample, query) rows instead of a tile of offsets: a wave reads the row's s_j^2 keys
// of the part with consecutive lanes on consecutive floats (whole cache lines, each value
// read exactly once), every lane works out its key's distance from the row's centre and
// adds the value to bin `distance` of a column of bins in LDS that belongs to this lane
// alone (no two lanes on one address, and a lane's additions happen in program order, so
// the sums repeat bit for bit).  At the end the 64 columns of a wave are folded by a fixed butterfly, the four waves
// of the workgroup in order.
constexpr int kRowsMaxSide = 64;           // bins of the four waves: 4 x side x 64 x 8 bytes of LDS
constexpr int kRowsThreads = 256;

// (A plain read-add-write on the lane's own column: LDS atomics -- ds_add_f64, and ds_add_u64
// alike -- were measured at about 240 cycles per wave instruction here, six times the cost of
// everything else in the loop; the read-add-write chains of the sixteen waves of a CU overlap.)
__device__ inline void lds_add_f64(double* col, int d, double v) { col[d * 64] += v; }

__global__ __launch_bounds__(kRowsThreads) void k_calib_mass_rows(CalibArgs a) {
  extern __shared__ __align__(16) unsigned char calib_smem[];
  const Slot sl = decode_slot(a, blockIdx.x);
  const int k = sl.k, j = sl.j, h = blockIdx.z, tile = sl.tile, split = sl.split;
  const int sk = a.s[k], sj = a.s[j];
  const int nt = tiles_of(sj);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // LDS: bins[wave][d][lane] (fp64), then the centres of the part's query coordinates
  double* const bins = (double*)calib_smem + (size_t)wave * sj * 64;
  double* const fold = (double*)calib_smem + (size_t)4 * a.smax * 64;          // [4][smax]
  short* const cen = (short*)(fold + 4 * a.smax);                              // [sk]
  for (int c = threadIdx.x; c < sk; c += kRowsThreads) cen[c] = (short)(((2 * c + 1) * sj) / (2 * sk));
  for (int i = lane; i < sj * 64; i += 64) bins[i] = 0.0;
  __syncthreads();

  double* const bins_lane = bins + lane;                                       // this lane's column of bins
  const int nkeys = sj * sj, nq = sk * sk;
  const int share = split * nt + tile, n_shares = a.splits * nt;               // this workgroup's rows
  const float* part = a.p + (int64_t)h * a.L * a.L + (int64_t)a.off[k] * a.L + a.off[j];
  const int64_t sample_stride = (int64_t)a.H * a.L * a.L;
  // this wave's queries: first, first + stride, ...; the N samples of a query share its centre,
  // so their values are added in registers first and binned once
  const int first = share * 4 + wave, stride = n_shares * 4;
  if (nkeys >= 64) {
    constexpr int U = 4, NB = 8;                          // an item: 256 keys of a query's row, 8 samples: 32 loads
    const int nchunk = (nkeys + 64 * U - 1) / (64 * U);
    const int my_q = first < nq ? (nq - first + stride - 1) / stride : 0;
    const int n_items = my_q * nchunk;
    auto load_item = [&](int t, int n0, float (&v)[NB][U]) {
      const int q = first + (t / nchunk) * stride, i0 = (t % nchunk) * 64 * U;
      const float* row = part + (int64_t)q * a.L;
#pragma unroll
      for (int m = 0; m < NB; ++m)
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int i = i0 + 64 * u + lane;
          v[m][u] = (n0 + m < a.N && i < nkeys) ? row[(n0 + m) * sample_stride + i] : 0.f;
        }
    };
    // the loads of the next item are in flight while this one is binned
    float cur[NB][U], nxt[NB][U];
    if (n_items > 0) load_item(0, 0, cur);
    for (int t = 0; t < n_items; ++t) {
      if (t + 1 < n_items) load_item(t + 1, 0, nxt);
      const int q = first + (t / nchunk) * stride, i0 = (t % nchunk) * 64 * U;
      const int cy = cen[q / sk], cx = cen[q % sk];
      double acc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) acc[u] = 0.0;
#pragma unroll
      for (int m = 0; m < NB; ++m)
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] += (double)cur[m][u];
      for (int n0 = NB; n0 < a.N; n0 += NB) {             // (more than eight samples: further batches, not overlapped)
        load_item(t, n0, cur);
#pragma unroll
        for (int m = 0; m < NB; ++m)
#pragma unroll
          for (int u = 0; u < U; ++u) acc[u] += (double)cur[m][u];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + 64 * u + lane;
        const int ky = i / sj, kx = i - ky * sj;
        if (i < nkeys) lds_add_f64(bins_lane, max(abs(ky - cy), abs(kx - cx)), acc[u]);
      }
#pragma unroll
      for (int m = 0; m < NB; ++m)
#pragma unroll
        for (int u = 0; u < U; ++u) cur[m][u] = nxt[m][u];
    }
  } else {
    // a part with fewer than 64 keys per row: a pass covers 64 / nkeys queries, lane = (query, key)
    const int qpp = 64 / nkeys;                           // queries per pass
    const int sub = lane / nkeys, key = lane - sub * nkeys;
    const int ky = key / sj, kx = key - ky * sj;
    for (int t0 = 0; first + (int64_t)t0 * stride < nq; t0 += qpp) {
      const int64_t q = first + (int64_t)(t0 + sub) * stride;
      const bool in = sub < qpp && q < nq;
      const int qq = in ? (int)q : first;
      const int d = max(abs(ky - cen[qq / sk]), abs(kx - cen[qq % sk]));
      const float* src = part + (int64_t)qq * a.L + key;
      double acc = 0.0;
      for (int n = 0; n < a.N; n += 8) {                  // eight loads in flight
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = n + u < a.N ? src[(n + u) * sample_stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (double)v[u];
      }
      if (in) lds_add_f64(bins_lane, d, acc);
    }
  }
  // fold the wave's 64 columns (fixed butterfly), then the four waves in order
  for (int d = 0; d < sj; ++d) {
    double x = bins[d * 64 + lane];
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) x += __shfl_xor(x, m);
    if (lane == 0) fold[wave * a.smax + d] = x;
  }
  __syncthreads();
  double* out = a.partial +
      (((((int64_t)h * a.K + k) * a.K + j) * a.splits + split) * a.max_tiles + tile) * a.smax;
  for (int d = threadIdx.x; d < sj; d += kRowsThreads)
    out[d] = ((fold[d] + fold[a.smax + d]) + fold[2 * a.smax + d]) + fold[3 * a.smax + d];
}

// grid (K * K, H), one wave
__global__ __launch_bounds__(64) void k_calib_pick(CalibArgs a) {
  const int k = blockIdx.x / a.K, j = blockIdx.x % a.K, h = blockIdx.y;
  const int64_t part = ((int64_t)h * a.K + k) * a.K + j;
  double* mass = a.mass ? a.mass + part * a.smax : nullptr;
  if (j > k) {
    if (threadIdx.x == 0) a.radius[part] = -1;
    if (mass) for (int r = threadIdx.x; r < a.smax; r += 64) mass[r] = 0.0;
    return;
  }
  const int sj = a.s[j], nt = tiles_of(sj);
  __shared__ double ring[kMaxSide];          // values at distance exactly d
  const double* in = a.partial + part * a.splits * a.max_tiles * a.smax;
  for (int d = threadIdx.x; d < sj; d += 64) {
    double s = 0.0;
    for (int sp = 0; sp < a.splits; ++sp)
      for (int t = 0; t < nt; ++t) s += in[((int64_t)sp * a.max_tiles + t) * a.smax + d];
    ring[d] = s;
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  double total = 0.0;
  for (int d = 0; d < sj; ++d) total += ring[d];
  // the window grows from zero until the ratio reaches the threshold
  double inside = 0.0;
  int found = -1;
  for (int r = 0; r < a.smax; ++r) {
    if (r < sj) inside += ring[r];
    if (mass) mass[r] = inside;
    if (found < 0 && r < sj && (total == 0.0 || inside / total >= a.r0)) found = r;
  }
  a.radius[part] = found < 0 ? sj - 1 : found;
}

litevar_status calib_geom(const int32_t* scales, int32_t K, CalibArgs& a) {
  if (!scales) return fail(LITEVAR_E_INVALID_ARG, "scales is NULL");
  if (K < 1 || K > kMaxScales)
    return fail(LITEVAR_E_INVALID_ARG, "n_scales must be in 1..%d (got %d)", kMaxScales, K);
  a.K = K; a.smax = 0; a.L = 0;
  for (int k = 0; k < K; ++k) {
    if (scales[k] < 1 || scales[k] > kMaxSide)
      return fail(LITEVAR_E_INVALID_ARG, "scales[%d] = %d outside 1..%d", k, scales[k], kMaxSide);
    a.s[k] = scales[k]; a.off[k] = (int)a.L; a.L += (int64_t)scales[k] * scales[k];
    if (a.L > ((int64_t)1 << 30)) return fail(LITEVAR_E_UNSUPPORTED, "sequence longer than 2^30 tokens");
    if (scales[k] > a.smax) a.smax = scales[k];
  }
  a.off[K] = (int)a.L;
  const int w = 2 * a.smax - 1;
  a.max_tiles = (w * w + kCalibThreads - 1) / kCalibThreads;
  a.splits = 64 / a.max_tiles < 1 ? 1 : (64 / a.max_tiles > 4 ? 4 : 64 / a.max_tiles);
  int n = 0;
  for (int kk = 0; kk < K; ++kk)
    for (int j = 0; j < K; ++j) {
      a.slot_begin[kk * K + j] = (uint16_t)n;
      if (j <= kk) n += a.splits * tiles_of(a.s[j]);
      if (n > 65535) return fail(LITEVAR_E_UNSUPPORTED, "too many parts and offset tiles for one launch");
    }
  a.slot_begin[K * K] = (uint16_t)n;
  a.n_slots = n;
  return LITEVAR_OK;
}

size_t calib_workspace(const CalibArgs& a, int H) {
  return (size_t)H * a.K * a.K * a.splits * a.max_tiles * a.smax * sizeof(double);
}

litevar_status calibrate_with(CalibArgs& a, const float* d_attn, int32_t N, int32_t H, float r0,
                              void* d_workspace, size_t workspace_bytes, int32_t* d_radius,
                              double* d_mass, void* stream);

litevar_status check_calib_args(const float* d_attn, int32_t N, int32_t H, float r0,
                                const int32_t* d_radius, const double* d_mass) {
  if (N < 1 || H < 1) return fail(LITEVAR_E_INVALID_ARG, "N and H must be positive");
  if (!(r0 > 0.f) || r0 > 1.f) return fail(LITEVAR_E_INVALID_ARG, "r0 must be in (0, 1] (got %g)", r0);
  if (!d_attn || !d_radius) return fail(LITEVAR_E_INVALID_ARG, "d_attn or d_radius is NULL");
  if (d_mass && ((uintptr_t)d_mass & 7)) return fail(LITEVAR_E_INVALID_ARG, "d_mass must be 8-byte aligned");
  return LITEVAR_OK;
}

// Scratch memory of litevar_window_calibrate_static, the entry point for callers that cannot
// allocate: the per-workgroup partial sums live in this array instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// kernels get the resolved device address as an argument like any other workspace.
constexpr size_t kStaticScratchBytes = LITEVAR_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};       // resolved once per device, with that device current

litevar_status static_scratch(void** out) {
  int dev = -1;
  if (litevar_status s = hip_check(hipGetDevice(&dev), "hipGetDevice")) return s;
  if (dev < 0 || dev >= kMaxDevices) return fail(LITEVAR_E_UNSUPPORTED, "device index %d above %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (litevar_status s = hip_check(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return s;
    if (!p) return fail(LITEVAR_E_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LITEVAR_OK;
}

}  // namespace

}  // namespace lv

using namespace lv;

extern "C" {

litevar_status litevar_window_calibrate_workspace_bytes(const int32_t* scales, int32_t n_scales,
                                                        int32_t H, size_t* out_bytes) {
  if (!out_bytes) return fail(LITEVAR_E_INVALID_ARG, "out_bytes is NULL");
  if (H < 1) return fail(LITEVAR_E_INVALID_ARG, "H must be positive");
  CalibArgs a;
  if (litevar_status s = calib_geom(scales, n_scales, a)) return s;
  *out_bytes = calib_workspace(a, H);
  return LITEVAR_OK;
}

litevar_status litevar_window_calibrate(const int32_t* scales, int32_t n_scales, const float* d_attn,
                                        int32_t N, int32_t H, float r0, void* d_workspace,
                                        size_t workspace_bytes, int32_t* d_radius, double* d_mass,
                                        void* stream) {
  CalibArgs a;
  if (litevar_status s = calib_geom(scales, n_scales, a)) return s;
  return calibrate_with(a, d_attn, N, H, r0, d_workspace, workspace_bytes, d_radius, d_mass, stream);
}

litevar_status litevar_window_calibrate_static(const int32_t* scales, int32_t n_scales,
                                               const float* d_attn, int32_t N, int32_t H, float r0,
                                               int32_t* d_radius, double* d_mass, void* stream) {
  CalibArgs a;
  if (litevar_status s = calib_geom(scales, n_scales, a)) return s;
  if (litevar_status s = check_calib_args(d_attn, N, H, r0, d_radius, d_mass)) return s;
  const size_t need = calib_workspace(a, H);
  if (need > kStaticScratchBytes)
    return fail(LITEVAR_E_UNSUPPORTED, "the partial sums need %zu bytes, the library's static scratch "
                "array holds %zu (LITEVAR_STATIC_SCRATCH_BYTES): use litevar_window_calibrate with a "
                "caller-owned workspace", need, (size_t)kStaticScratchBytes);
  void* ptr = nullptr;
  if (litevar_status s = static_scratch(&ptr)) return s;
  return calibrate_with(a, d_attn, N, H, r0, ptr, kStaticScratchBytes, d_radius, d_mass, stream);
}

}  // extern "C"

namespace lv {
namespace {

litevar_status calibrate_with(CalibArgs& a, const float* d_attn, int32_t N, int32_t H, float r0,
                              void* d_workspace, size_t workspace_bytes, int32_t* d_radius,
                              double* d_mass, void* stream) {
  if (litevar_status s = check_calib_args(d_attn, N, H, r0, d_radius, d_mass)) return s;
  if (!d_workspace) return fail(LITEVAR_E_INVALID_ARG, "d_workspace is NULL");
  if ((uintptr_t)d_workspace & 7) return fail(LITEVAR_E_INVALID_ARG, "d_workspace must be 8-byte aligned");
  if (workspace_bytes < calib_workspace(a, H))
    return fail(LITEVAR_E_INVALID_ARG, "workspace of %zu bytes, %zu needed", workspace_bytes,
                calib_workspace(a, H));
  if ((int64_t)a.K * a.K > 65535 || H > 65535)
    return fail(LITEVAR_E_UNSUPPORTED, "grid too large");
  a.N = N; a.H = H; a.p = d_attn; a.partial = (double*)d_workspace;
  a.radius = d_radius; a.mass = d_mass; a.r0 = (double)r0;
  hipStream_t st = (hipStream_t)stream;
  if (a.smax <= kRowsMaxSide) {
    // (maps of small scales, the usual case: whole rows with coalesced loads)
    const size_t lds = (size_t)4 * a.smax * 64 * sizeof(double) + (size_t)4 * a.smax * sizeof(double) +
                       (size_t)a.smax * sizeof(short) + 16;
    if (lds > 64 * 1024)     // (beyond the default limit of dynamically sized LDS; no allocation involved)
      if (litevar_status s = hip_check(hipFuncSetAttribute((const void*)k_calib_mass_rows,
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                                       "hipFuncSetAttribute")) return s;
    hipLaunchKernelGGL(k_calib_mass_rows, dim3(a.n_slots, 1, H), dim3(kRowsThreads), lds, st, a);
  } else {
    hipLaunchKernelGGL(k_calib_mass, dim3(a.n_slots, 1, H), dim3(kCalibThreads), 0, st, a);
  }
  if (litevar_status s = hip_check(hipGetLastError(), "calibration mass launch")) return s;
  hipLaunchKernelGGL(k_calib_pick, dim3(a.K * a.K, H), dim3(64), 0, st, a);
  return hip_check(hipGetLastError(), "calibration pick launch");
}

}  // namespace
}  // namespace lv
