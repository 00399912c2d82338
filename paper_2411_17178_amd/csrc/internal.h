// Declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>

#include <vector>

#include "../../include/litevar.h"
#include "plan.h"

namespace lv {

// records a printf-style message in the thread-local error string, returns `code`
litevar_status fail(litevar_status code, const char* fmt, ...);
litevar_status hip_check(hipError_t e, const char* what);

struct PlanSizes {
  int64_t n_steps, n_union, n_phase_entries, retained_pairs;   // summed over the head groups
  int64_t pairs_of_group[kMaxHeads];                           // kept pairs per (batch, head) of each head group
  uint64_t off[kNumSections];
  uint64_t bytes;
};

// What a mask descriptor asks for: the geometry, and one radius table per head group
// (heads with equal tables share a group).  g.rad holds the table of the group that was
// loaded last; make_spec and size_plan leave group 0 loaded.
struct PlanSpec {
  Geom g;
  int n_heads = 0;                      // 0: one table for all heads
  std::vector<int16_t> rad_all;         // [n_hg][K][K]
  uint8_t head_group[kMaxHeads] = {};   // head -> head group
  void load_head_group(int hg) {
    for (int k = 0; k < g.K; ++k)
      for (int j = 0; j < g.K; ++j) g.rad[k][j] = rad_all[((size_t)hg * g.K + k) * g.K + j];
  }
};

litevar_status make_spec(const litevar_mask_desc* d, const litevar_plan_opts* opts, PlanSpec& sp);
litevar_status size_plan(PlanSpec& sp, PlanSizes& z);
litevar_status build_plan(PlanSpec& sp, const PlanSizes& z, void* d_blob, hipStream_t st);
litevar_status read_header(const litevar_plan* pl, hipStream_t st, Header& h);

litevar_status export_window_table(const litevar_plan* pl, int head, int16_t* d_out, hipStream_t st);
litevar_status export_dense(const litevar_plan* pl, int head, uint8_t* d_mask, uint64_t* d_count, hipStream_t st);
litevar_status export_csr(const litevar_plan* pl, int head, int64_t* d_rowptr, int32_t* d_cols, size_t cap,
                          hipStream_t st);

struct AttnArgs {
  const void* q; const void* k; const void* v; void* o;
  int64_t qs[3], ks[3], os[3];   // element strides of (B, H, token)
  int B, H;
  float sm_scale;
  const uint8_t* cfg_share;      // [H][K] or nullptr
  int n_scales;
  // plan sections
  const GroupDesc* groups; const WaveDesc* waves; const int32_t* phase_end;
  const int32_t* union_tok; const uint2* step_addr; const uint64_t* step_mask;
  const int32_t* step_tok;
  int n_groups;                  // groups of one head group
  const int32_t* head_map;       // head -> head group, or nullptr when all heads share one
  int q_len;                     // query rows per (batch, head)
  int kv_len;                    // key rows per (batch, head)
  Header* hdr;                   // the blob's header: checked by every kernel before the plan is used
  int spin_limit;                // polls after which a kernel's wait on an LDS flag gives up
  // 8-bit operands (Section 4): q, k, v then hold int8 codes (strides in codes) and these the
  // (scale, zero point) of every token row, packed [B][H][len]; nullptr for bf16 / fp32 operands
  const float2* q_sz; const float2* k_sz; const float2* v_sz;
  // floor(2^32 / n) for n = n_groups and n = H: a workgroup's index is taken apart with two
  // multiplications instead of two divisions by run-time values (see divmod_by in the kernels' header)
  uint32_t n_groups_magic, H_magic;
};

// Checks what every attention entry point checks (plan, batch and head counts, softmax scale,
// flags) and fills the fields of `a` that come from the plan and from these arguments; the
// operand pointers and strides are the caller's.
litevar_status make_attn_args(const litevar_plan* plan, int32_t B, int32_t H, int32_t D, float sm_scale,
                              const uint8_t* d_cfg_share, uint32_t flags, AttnArgs& a);

litevar_status launch_attn_f32(const litevar_plan* pl, const AttnArgs& a, hipStream_t st);
litevar_status launch_attn_bf16(const litevar_plan* pl, const AttnArgs& a, hipStream_t st);
litevar_status launch_attn_bf16_pair(const litevar_plan* pl, const AttnArgs& a, hipStream_t st);

}  // namespace lv
