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
  const float* p;       // [N][H][L][L]
  double* partial;      // [H][K][K][splits][max_tiles][smax]: per-distance sums of one workgroup
  int32_t* radius;      // [H][K][K]
  double* mass;         // [H][K][K][smax] or nullptr
  double r0;
};

__device__ inline int tiles_of(int sj) {
  const int w = 2 * sj - 1;
  return (w * w + kCalibThreads - 1) / kCalibThreads;
}

// grid (max_tiles * splits, K * K, H)
__global__ __launch_bounds__(kCalibThreads) void k_calib_mass(CalibArgs a) {
  const int k = blockIdx.y / a.K, j = blockIdx.y % a.K, h = blockIdx.z;
  const int tile = blockIdx.x % a.max_tiles, split = blockIdx.x / a.max_tiles;
  if (j > k) return;
  const int sk = a.s[k], sj = a.s[j];
  if (tile >= tiles_of(sj)) return;
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
  hipLaunchKernelGGL(k_calib_mass, dim3(a.max_tiles * a.splits, a.K * a.K, H), dim3(kCalibThreads), 0, st, a);
  if (litevar_status s = hip_check(hipGetLastError(), "calibration mass launch")) return s;
  hipLaunchKernelGGL(k_calib_pick, dim3(a.K * a.K, H), dim3(64), 0, st, a);
  return hip_check(hipGetLastError(), "calibration pick launch");
}

}  // namespace
}  // namespace lv
