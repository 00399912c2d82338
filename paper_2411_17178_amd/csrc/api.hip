// C ABI of the library: argument validation, error strings, dispatch.
#include "internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

namespace lv {

static thread_local char g_err[512] = "";

litevar_status fail(litevar_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

litevar_status hip_check(hipError_t e, const char* what) {
  if (e == hipSuccess) return LITEVAR_OK;
  return fail(LITEVAR_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

static litevar_status check_plan(const litevar_plan* pl) {
  if (!pl) return fail(LITEVAR_E_INVALID_ARG, "plan is NULL");
  if (pl->magic != kMagic) return fail(LITEVAR_E_PLAN_CORRUPT, "plan handle has a bad magic");
  if (!pl->d_blob || pl->off[kSecEnd] != pl->blob_bytes)
    return fail(LITEVAR_E_PLAN_CORRUPT, "plan handle is inconsistent");
  return LITEVAR_OK;
}

}  // namespace lv

using namespace lv;

extern "C" {

const char* litevar_status_string(litevar_status s) {
  switch (s) {
    case LITEVAR_OK: return "ok";
    case LITEVAR_E_INVALID_ARG: return "invalid argument";
    case LITEVAR_E_UNSUPPORTED: return "unsupported";
    case LITEVAR_E_PLAN_TOO_SMALL: return "plan buffer too small";
    case LITEVAR_E_HIP: return "HIP runtime error";
    case LITEVAR_E_PLAN_CORRUPT: return "plan corrupt";
    default: return "unknown status";
  }
}

const char* litevar_last_error(void) { return g_err; }

int32_t litevar_version(void) { return 100; }

litevar_status litevar_scale_offsets(const int32_t* scales, int32_t n_scales, int64_t* out_offsets) {
  if (!scales || !out_offsets) return fail(LITEVAR_E_INVALID_ARG, "scales or out_offsets is NULL");
  if (n_scales < 1 || n_scales > kMaxScales)
    return fail(LITEVAR_E_INVALID_ARG, "n_scales must be in 1..%d (got %d)", kMaxScales, n_scales);
  int64_t L = 0;
  for (int k = 0; k < n_scales; ++k) {
    if (scales[k] < 1 || scales[k] > kMaxSide)
      return fail(LITEVAR_E_INVALID_ARG, "scales[%d] = %d outside 1..%d", k, scales[k], kMaxSide);
    out_offsets[k] = L; L += (int64_t)scales[k] * scales[k];
  }
  out_offsets[n_scales] = L;
  return LITEVAR_OK;
}

litevar_status litevar_mask_plan_bytes(const litevar_mask_desc* desc, const litevar_plan_opts* opts,
                                       size_t* out_bytes) {
  if (!out_bytes) return fail(LITEVAR_E_INVALID_ARG, "out_bytes is NULL");
  PlanSpec sp;
  litevar_status rc = make_spec(desc, opts, sp);
  if (rc) return rc;
  PlanSizes z;
  rc = size_plan(sp, z);
  if (rc) return rc;
  *out_bytes = (size_t)z.bytes;
  return LITEVAR_OK;
}

static litevar_status check_patches_per_wave(const litevar_plan_opts* opts) {
  const int pw = opts ? opts->patches_per_wave : 0;
  if (pw < 0 || pw > 2) return fail(LITEVAR_E_INVALID_ARG, "patches_per_wave must be 0, 1 or 2 (got %d)", pw);
  if (opts && opts->spin_limit < 0) return fail(LITEVAR_E_INVALID_ARG, "spin_limit must not be negative");
  return LITEVAR_OK;
}

static void fill_handle(const PlanSpec& sp, const PlanSizes& z, const litevar_plan_opts* opts, litevar_plan* plan) {
  const Geom& g = sp.g;
  memset(plan, 0, sizeof *plan);
  plan->mask_mode = g.mode == kModeBand ? LITEVAR_MASK_BAND_1D : LITEVAR_MASK_WINDOW_2D;
  plan->n_heads = sp.n_heads; plan->n_head_groups = g.n_hg;
  memcpy(plan->head_group, sp.head_group, sizeof plan->head_group);
  for (int i = 0; i < g.n_hg && i < kMaxHeads; ++i) plan->retained_pairs_of_group[i] = z.pairs_of_group[i];
  plan->patches_per_wave = (opts && g.NW == 16) ? opts->patches_per_wave : 0;
  plan->blob_bytes = z.bytes;
  plan->n_scales = g.K;
  plan->q_scale_begin = g.qb; plan->q_scale_end = g.qe;
  plan->kv_len = g.L; plan->q_len = g.Lq; plan->q_token_begin = g.q0;
  plan->side_max = g.smax;
  plan->waves_per_group = g.NW; plan->chunk_keys = g.C; plan->ring_chunks = g.NR;
  plan->prefetch_chunks = g.D;
  plan->n_groups = g.n_groups; plan->n_patches = g.n_patches;
  plan->n_steps = z.n_steps; plan->n_union_keys = z.n_union;
  plan->retained_pairs = z.retained_pairs;
  plan->computed_pairs = z.n_steps * 16 * kStepKeys;
  for (int i = 0; i < kNumSections; ++i) plan->off[i] = z.off[i];
  for (int k = 0; k < g.K; ++k) {
    plan->scales[k] = g.s[k];
    // widest window of key scale k over the plan's query scales and head groups (-1 if one
    // of them is dense)
    int r = 0;
    for (int hg = 0; hg < g.n_hg; ++hg)
      for (int q = (g.qb > k ? g.qb : k); q < g.qe; ++q) {
        const int rq = sp.rad_all[((size_t)hg * g.K + q) * g.K + k];
        r = (r < 0 || rq < 0) ? -1 : (rq > r ? rq : r);
      }
    plan->radii[k] = r;
  }
  plan->n_sink_scales = g.n_sink;
  plan->spin_limit = (opts && opts->spin_limit > 0) ? opts->spin_limit : kDefaultSpinLimit;
}

litevar_status litevar_mask_plan_stats(const litevar_mask_desc* desc, const litevar_plan_opts* opts,
                                       litevar_plan* stats) {
  if (!stats) return fail(LITEVAR_E_INVALID_ARG, "stats is NULL");
  PlanSpec sp;
  litevar_status rc = make_spec(desc, opts, sp);
  if (rc) return rc;
  PlanSizes z;
  rc = size_plan(sp, z);
  if (rc) return rc;
  if (litevar_status s = check_patches_per_wave(opts)) return s;
  fill_handle(sp, z, opts, stats);
  return LITEVAR_OK;
}

litevar_status litevar_mask_build(const litevar_mask_desc* desc, const litevar_plan_opts* opts,
                                  void* d_blob, size_t blob_bytes, void* stream,
                                  litevar_plan* plan) {
  if (!plan) return fail(LITEVAR_E_INVALID_ARG, "plan is NULL");
  PlanSpec sp;
  litevar_status rc = make_spec(desc, opts, sp);
  if (rc) return rc;
  PlanSizes z;
  rc = size_plan(sp, z);
  if (rc) return rc;
  if (!d_blob) return fail(LITEVAR_E_INVALID_ARG, "d_blob is NULL");
  if ((uintptr_t)d_blob & 255) return fail(LITEVAR_E_INVALID_ARG, "d_blob must be 256-byte aligned");
  if (blob_bytes < z.bytes)
    return fail(LITEVAR_E_PLAN_TOO_SMALL, "plan needs %llu bytes, buffer has %llu",
                (unsigned long long)z.bytes, (unsigned long long)blob_bytes);
  if (litevar_status s = check_patches_per_wave(opts)) return s;
  rc = build_plan(sp, z, d_blob, (hipStream_t)stream);
  if (rc) return rc;
  fill_handle(sp, z, opts, plan);
  plan->magic = kMagic;
  plan->d_blob = d_blob;
  return LITEVAR_OK;
}

litevar_status litevar_plan_check(const litevar_plan* plan, void* stream) {
  litevar_status rc = check_plan(plan);
  if (rc) return rc;
  Header h;
  rc = read_header(plan, (hipStream_t)stream, h);
  if (rc) return rc;
  if (h.magic != kMagic) return fail(LITEVAR_E_PLAN_CORRUPT, "device blob has a bad magic");
  if (h.error == kErrBuilder) return fail(LITEVAR_E_PLAN_CORRUPT, "device builder disagrees with the host sizing");
  if (h.error == kErrWaitGaveUp)
    return fail(LITEVAR_E_PLAN_CORRUPT, "an attention kernel's bounded wait gave up (its output is invalid)");
  if (h.error == kErrBounds)
    return fail(LITEVAR_E_PLAN_CORRUPT, "a kernel of the bounds-checking build found an index out of range");
  if (h.error) return fail(LITEVAR_E_PLAN_CORRUPT, "device blob carries the unknown error mark %d", h.error);
  if (h.blob_bytes != plan->blob_bytes || h.n_groups != plan->n_groups * plan->n_head_groups ||
      h.n_steps != plan->n_steps || h.n_union != plan->n_union_keys ||
      h.retained_pairs != plan->retained_pairs)
    return fail(LITEVAR_E_PLAN_CORRUPT, "device blob does not match the handle");
  return LITEVAR_OK;
}

static litevar_status check_head(const litevar_plan* plan, int32_t head) {
  const int n = plan->n_heads > 0 ? plan->n_heads : 1;
  if (head < 0 || head >= n) return fail(LITEVAR_E_INVALID_ARG, "head %d outside the plan's 0..%d", head, n - 1);
  return LITEVAR_OK;
}

litevar_status litevar_window_table_export(const litevar_plan* plan, int32_t head, int16_t* d_out,
                                           size_t out_bytes, void* stream) {
  litevar_status rc = check_plan(plan);
  if (rc) return rc;
  if (litevar_status s = check_head(plan, head)) return s;
  if (plan->mask_mode != LITEVAR_MASK_WINDOW_2D)
    return fail(LITEVAR_E_UNSUPPORTED, "the band mode has no window table");
  if (!d_out) return fail(LITEVAR_E_INVALID_ARG, "d_out is NULL");
  const size_t need = (size_t)plan->n_scales * plan->n_scales * plan->side_max * 2 * sizeof(int16_t);
  if (out_bytes < need)
    return fail(LITEVAR_E_INVALID_ARG, "window table needs %zu bytes, buffer has %zu", need, out_bytes);
  return export_window_table(plan, head, d_out, (hipStream_t)stream);
}

litevar_status litevar_mask_export_dense(const litevar_plan* plan, int32_t head, uint8_t* d_mask, size_t mask_bytes,
                                         uint64_t* d_pair_count, void* stream) {
  litevar_status rc = check_plan(plan);
  if (rc) return rc;
  if (litevar_status s = check_head(plan, head)) return s;
  if (!d_mask) return fail(LITEVAR_E_INVALID_ARG, "d_mask is NULL");
  const size_t need = (size_t)plan->q_len * plan->kv_len;
  if (mask_bytes < need)
    return fail(LITEVAR_E_INVALID_ARG, "dense mask needs %zu bytes, buffer has %zu", need, mask_bytes);
  return export_dense(plan, head, d_mask, d_pair_count, (hipStream_t)stream);
}

litevar_status litevar_mask_export_csr(const litevar_plan* plan, int32_t head, int64_t* d_rowptr, int32_t* d_cols,
                                       size_t cols_cap, void* stream) {
  litevar_status rc = check_plan(plan);
  if (rc) return rc;
  if (litevar_status s = check_head(plan, head)) return s;
  if (!d_rowptr || !d_cols) return fail(LITEVAR_E_INVALID_ARG, "d_rowptr or d_cols is NULL");
  const int64_t kept = plan->retained_pairs_of_group[plan->n_heads > 0 ? plan->head_group[head] : 0];
  if ((int64_t)cols_cap < kept)
    return fail(LITEVAR_E_INVALID_ARG, "cols_cap %zu below the %lld kept pairs", cols_cap, (long long)kept);
  return export_csr(plan, head, d_rowptr, d_cols, cols_cap, (hipStream_t)stream);
}

}  // extern "C"

namespace lv {

litevar_status make_attn_args(const litevar_plan* plan, int32_t B, int32_t H, int32_t D, float sm_scale,
                              const uint8_t* d_cfg_share, uint32_t flags, AttnArgs& a) {
  litevar_status rc = check_plan(plan);
  if (rc) return rc;
  if (B < 1 || H < 1) return fail(LITEVAR_E_INVALID_ARG, "B and H must be positive (got %d, %d)", B, H);
  if ((int64_t)B * H > (1 << 24)) return fail(LITEVAR_E_UNSUPPORTED, "B*H above 2^24");
  if (D != 64) return fail(LITEVAR_E_UNSUPPORTED, "head dimension %d is not supported (only 64)", D);
  if (!(sm_scale > 0.f) || !std::isfinite(sm_scale) || sm_scale > 1.0e4f)
    return fail(LITEVAR_E_INVALID_ARG, "sm_scale must be finite, positive and at most 1e4");
  if (flags & ~(uint32_t)LITEVAR_FLAG_CFG_SHARE) return fail(LITEVAR_E_INVALID_ARG, "unknown flag bits 0x%x", flags);
  if (flags & LITEVAR_FLAG_CFG_SHARE) {
    if (B & 1) return fail(LITEVAR_E_INVALID_ARG, "CFG sharing needs an even batch (got %d)", B);
    if (!d_cfg_share) return fail(LITEVAR_E_INVALID_ARG, "CFG sharing flag set but d_cfg_share is NULL");
  }
  if (plan->n_heads > 0 && H != plan->n_heads)
    return fail(LITEVAR_E_INVALID_ARG, "the plan holds radius tables for %d heads, the call has H = %d", plan->n_heads, H);
  memset(&a, 0, sizeof a);
  a.B = B; a.H = H; a.sm_scale = sm_scale;
  a.cfg_share = (flags & LITEVAR_FLAG_CFG_SHARE) ? d_cfg_share : nullptr;
  a.n_scales = plan->n_scales;
  const char* blob = (const char*)plan->d_blob;
  a.groups = (const GroupDesc*)(blob + plan->off[kSecGroups]);
  a.waves = (const WaveDesc*)(blob + plan->off[kSecWaves]);
  a.phase_end = (const int32_t*)(blob + plan->off[kSecPhaseEnd]);
  a.union_tok = (const int32_t*)(blob + plan->off[kSecUnion]);
  a.step_addr = (const uint2*)(blob + plan->off[kSecStepAddr]);
  a.step_mask = (const uint64_t*)(blob + plan->off[kSecStepMask]);
  a.step_tok = (const int32_t*)(blob + plan->off[kSecStepTok]);
  a.n_groups = plan->n_groups;
  a.head_map = plan->n_heads > 0 ? (const int32_t*)(blob + plan->off[kSecHeadMap]) : nullptr;
  a.q_len = plan->q_len;
  a.kv_len = plan->kv_len;
  a.hdr = (Header*)(plan->d_blob);
  a.spin_limit = plan->spin_limit > 0 ? plan->spin_limit : kDefaultSpinLimit;
  a.n_groups_magic = (uint32_t)(((uint64_t)1 << 32) / (uint64_t)(plan->n_groups > 1 ? plan->n_groups : 1) - (plan->n_groups <= 1));
  a.H_magic = (uint32_t)(((uint64_t)1 << 32) / (uint64_t)(H > 1 ? H : 1) - (H <= 1));
  return LITEVAR_OK;
}

}  // namespace lv

extern "C" {

static bool strides_ok(const int64_t* s, int B, int H, int64_t len, int D, int64_t out[3]) {
  if (!s) { out[2] = D; out[1] = len * D; out[0] = (int64_t)H * len * D; return true; }
  for (int i = 0; i < 3; ++i) out[i] = s[i];
  if (s[2] < D || s[2] % 8) return false;          // rows 16-byte aligned for bf16, 32 for fp32
  if (s[1] < 0 || s[0] < 0 || s[1] % 8 || s[0] % 8) return false;
  (void)B;
  return true;
}

litevar_status litevar_windowed_attn_fwd(const litevar_plan* plan, const void* d_q, const void* d_k,
                                         const void* d_v, void* d_o, int32_t B, int32_t H, int32_t D,
                                         litevar_dtype dt, const int64_t* q_strides,
                                         const int64_t* kv_strides, const int64_t* o_strides,
                                         float sm_scale, const uint8_t* d_cfg_share, uint32_t flags,
                                         void* stream) {
  AttnArgs a;
  if (litevar_status s = make_attn_args(plan, B, H, D, sm_scale, d_cfg_share, flags, a)) return s;
  if (!d_q || !d_k || !d_v || !d_o) return fail(LITEVAR_E_INVALID_ARG, "q, k, v or o is NULL");
  if (dt != LITEVAR_BF16 && dt != LITEVAR_F32) return fail(LITEVAR_E_UNSUPPORTED, "unknown dtype %d", (int)dt);
  if (d_o == d_q || d_o == d_k || d_o == d_v) return fail(LITEVAR_E_INVALID_ARG, "o aliases an input");
  const uintptr_t align = (uintptr_t)d_q | (uintptr_t)d_k | (uintptr_t)d_v | (uintptr_t)d_o;
  if (align & 15) return fail(LITEVAR_E_INVALID_ARG, "q, k, v, o must be 16-byte aligned");
  if (!strides_ok(q_strides, B, H, plan->q_len, D, a.qs) ||
      !strides_ok(kv_strides, B, H, plan->kv_len, D, a.ks) ||
      !strides_ok(o_strides, B, H, plan->q_len, D, a.os))
    return fail(LITEVAR_E_INVALID_ARG, "strides must be non-negative multiples of 8 with token stride >= D");
  const int64_t esize = dt == LITEVAR_BF16 ? 2 : 4;
  if ((int64_t)plan->kv_len * a.ks[2] * esize >= ((int64_t)1 << 31))
    return fail(LITEVAR_E_UNSUPPORTED, "one (batch, head) slab of k/v spans 2 GiB or more");
  // (the kernels form token x stride with 24-bit multiplies: tokens are below 2^24 by the
  // line above, since a token's row is at least 128 bytes from the next)
  if (a.ks[2] * esize >= ((int64_t)1 << 24))
    return fail(LITEVAR_E_UNSUPPORTED, "k/v token stride of 16 MiB or more");
  a.q = d_q; a.k = d_k; a.v = d_v; a.o = d_o;
  if (dt == LITEVAR_F32) return launch_attn_f32(plan, a, (hipStream_t)stream);
  return launch_attn_bf16(plan, a, (hipStream_t)stream);
}

}  // extern "C"
