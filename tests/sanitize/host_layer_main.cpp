// Exercises the library's host-only layer (descriptor validation, geometry, the sizing walk of
// every patch and key, handle filling) under AddressSanitizer and UBSan; no GPU call is made.
#include <cstdio>
#include <vector>

#include "litevar.h"

static int stats(const std::vector<int32_t>& scales, int radius, int n_sink, int qb, int qe, int mode, int waves,
                 const std::vector<int32_t>* per_head, int n_heads, long long* pairs) {
  litevar_mask_desc d = {};
  d.n_scales = (int32_t)scales.size(); d.scales = scales.data(); d.radius = radius; d.n_sink_scales = n_sink;
  d.q_scale_begin = qb; d.q_scale_end = qe; d.mask_mode = mode;
  if (per_head) { d.n_heads = n_heads; d.radius_per_head = per_head->data(); }
  litevar_plan_opts o = {};
  o.waves_per_group = waves; o.spare_chunks = -1;
  litevar_plan st;
  const int rc = litevar_mask_plan_stats(&d, &o, &st);
  if (rc == 0 && pairs) *pairs = (long long)st.retained_pairs;
  size_t bytes = 0;
  if (rc == 0 && litevar_mask_plan_bytes(&d, &o, &bytes) != 0) return -100;
  return rc;
}

int main() {
  const std::vector<int32_t> tiny = {1, 2, 3, 4}, var = {1, 2, 3, 4, 5, 6, 8, 10, 13, 16}, odd = {7, 2, 9, 4, 17},
                             big = {1, 2, 3, 4, 6, 9, 13, 18, 24, 32, 48, 64};
  long long p = 0;
  for (int waves : {0, 4, 8, 16})
    for (int mode : {0, 1}) {
      if (stats(tiny, 1, 0, 0, 4, mode, waves, nullptr, 0, &p)) return 1;
      printf("tiny mode %d waves %d: %lld\n", mode, waves, p);
      if (stats(var, 2, 3, 0, 10, mode, waves, nullptr, 0, &p)) return 1;
      if (stats(var, 3, 0, 9, 10, mode, waves, nullptr, 0, &p)) return 1;
      if (stats(odd, 40, 1, 2, 5, mode, waves, nullptr, 0, &p)) return 1;
      if (stats(odd, -1, 0, 0, 5, mode, waves, nullptr, 0, &p)) return 1;
      if (stats(big, 4, 0, 10, 12, mode, waves, nullptr, 0, &p)) return 1;
    }
  std::vector<int32_t> heads(3 * 100);
  for (size_t i = 0; i < heads.size(); ++i) heads[i] = (int32_t)((i * 7) % 6) - 1;
  if (stats(var, 0, 0, 0, 10, 0, 16, &heads, 3, &p)) return 1;
  if (stats(var, 0, 0, 0, 10, 1, 8, &heads, 3, &p)) return 1;
  // rejected descriptors
  if (stats(var, -2, 0, 0, 10, 0, 0, nullptr, 0, nullptr) != LITEVAR_E_INVALID_ARG) return 2;
  if (stats(var, 1, 11, 0, 10, 0, 0, nullptr, 0, nullptr) != LITEVAR_E_INVALID_ARG) return 2;
  if (stats(var, 1, 0, 5, 5, 0, 0, nullptr, 0, nullptr) != LITEVAR_E_INVALID_ARG) return 2;
  if (stats(var, 1, 0, 0, 10, 2, 0, nullptr, 0, nullptr) != LITEVAR_E_INVALID_ARG) return 2;
  if (stats(var, 1, 0, 0, 10, 0, 5, nullptr, 0, nullptr) != LITEVAR_E_INVALID_ARG) return 2;
  if (stats({0}, 1, 0, 0, 1, 0, 0, nullptr, 0, nullptr) != LITEVAR_E_INVALID_ARG) return 2;
  int64_t off[11];
  if (litevar_scale_offsets(var.data(), 10, off) || off[10] != 680) return 3;
  size_t ws = 0;
  if (litevar_window_calibrate_workspace_bytes(var.data(), 10, 30, &ws) || ws == 0) return 3;
  printf("ok\n");
  return 0;
}
