/*
 * litevar.h -- C ABI of the MI355X (gfx950) multi-diagonal windowed attention library.
 *
 * The operation is the attention of LiteVAR (arXiv 2411.17178) over VAR's
 * coarse-to-fine token sequence:
 *   - Section 2 ("Multi-Diagonal Window Attention"): K scales, scale k holds
 *     s_k^2 tokens, a query of scale k sees the tokens of scales 1..k, and inside
 *     each per-key-scale part of the attention map only a local window is kept;
 *   - Section 2, "MDWA implementation details": the leading parts may stay dense;
 *   - Section 3 ("Attention Sharing across CFG"): the unconditional rows may reuse
 *     the conditional rows' attention output.
 * Window geometry (the paper's figure is its only definition): query (k, y, x)
 * keeps key (j, y', x') of scale j <= k iff j < n_sink_scales, or
 * |y' - cy| <= r and |x' - cx| <= r with cy = floor((2y+1) s_j / (2 s_k)),
 * cx likewise, and r the radius of part j (one per key scale, or one per
 * (query scale, key scale): Section 2 determines it for each scale and part).  Tokens of a scale are stored row-major.  Masking precedes the
 * softmax, so the kept weights sum to 1.
 *
 * Conventions
 *   - Every pointer argument says HOST or DEVICE.  The library allocates no
 *     device memory.  Its only state: a thread-local error string, a thread-local memo of
 *     the last plan sizing, a per-thread cache of the devices' CU counts, and the static
 *     scratch array of litevar_window_calibrate_static with its resolved address.
 *   - All GPU work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and never synchronised, unless stated otherwise.
 *   - Arguments are validated on the host before any HIP call; a failed
 *     validation launches nothing.
 *   - Every function returns a litevar_status; details of the last failure on the
 *     calling thread are available from litevar_last_error().
 */
#ifndef LITEVAR_H_
#define LITEVAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t litevar_status;
enum {
  LITEVAR_OK = 0,
  LITEVAR_E_INVALID_ARG = -1,    /* null pointer, out-of-range value, inconsistent sizes */
  LITEVAR_E_UNSUPPORTED = -2,    /* valid but not implemented (e.g. head_dim != 64) */
  LITEVAR_E_PLAN_TOO_SMALL = -3, /* plan buffer smaller than litevar_mask_plan_bytes() */
  LITEVAR_E_HIP = -4,            /* a HIP runtime call failed; see litevar_last_error() */
  LITEVAR_E_PLAN_CORRUPT = -5    /* plan handle or device blob failed its self-check */
};

#define LITEVAR_MAX_SCALES 32
#define LITEVAR_MAX_SIDE 1024        /* largest s_k */
#define LITEVAR_RADIUS_DENSE (-1)    /* no window: dense block-causal part */

/* Static strings; never freed. */
const char* litevar_status_string(litevar_status s);
const char* litevar_last_error(void); /* thread-local */
int32_t litevar_version(void);

/*
 * Problem statement of one mask (Section 2).  All pointers are HOST pointers read
 * during the call only.
 */
typedef struct litevar_mask_desc {
  int32_t n_scales;                    /* K, 1..LITEVAR_MAX_SCALES */
  const int32_t* scales;               /* [K] side lengths s_k, 1..LITEVAR_MAX_SIDE, any order */
  int32_t radius;                      /* r >= 0 (window width 2r+1), or LITEVAR_RADIUS_DENSE */
  const int32_t* radius_per_key_scale; /* optional [K]; overrides `radius` when non-NULL */
  int32_t n_sink_scales;               /* leading key scales kept dense, 0..K (paper: 3) */
  int32_t q_scale_begin, q_scale_end;  /* query scales [begin, end): whole sequence = [0, K),
                                          last KV-cache step = [K-1, K) */
  const int32_t* radius_per_scale_pair; /* optional [K][K], [query scale][key scale] (Section 2:
                                          one window size per scale and part, e.g. from
                                          litevar_window_calibrate); overrides both radius
                                          fields when non-NULL; entries with key scale > query
                                          scale are ignored */
  int32_t n_heads;                     /* 0, or the number of heads H (<= LITEVAR_MAX_HEADS) of
                                          radius_per_head */
  const int32_t* radius_per_head;      /* optional [H][K][K], [head][query scale][key scale]
                                          (Section 2, step (3): the window size is determined for
                                          each scale, part and head; the layout of
                                          litevar_window_calibrate's d_radius); overrides the other
                                          radius fields; heads with equal tables share one
                                          work-list inside the plan.  Attention calls with such a
                                          plan must pass H = n_heads */
  int32_t mask_mode;                   /* LITEVAR_MASK_WINDOW_2D or LITEVAR_MASK_BAND_1D */
} litevar_mask_desc;

/*
 * The two readings of the window of Section 2 (the paper's figure is its only definition):
 *   LITEVAR_MASK_WINDOW_2D  a square window of radius r around the query's position mapped into
 *                           the key scale's grid, one part per key scale (the default; see the
 *                           top of this file);
 *   LITEVAR_MASK_BAND_1D    Section 2, step (2) read literally: the attention map of query
 *                           scale k, [s_k^2, sum of s_i^2], is cut into parts, the first
 *                           spanning the first three key scales (those of them the query sees),
 *                           every later key scale a part of its own; in a part of n columns the
 *                           query with flattened index i keeps the columns c with
 *                           |c - floor((2i+1) n / (2 s_k^2))| <= r, a band of width 2r+1 around
 *                           the part's diagonal.  The radius of a part is the entry of its last
 *                           key scale; a part whose last key scale is below n_sink_scales is
 *                           dense.  Radii up to 32767.  Query patches are 16 consecutive
 *                           queries.  No window table exists in this mode.
 */
enum { LITEVAR_MASK_WINDOW_2D = 0, LITEVAR_MASK_BAND_1D = 1 };
#define LITEVAR_MAX_HEADS 256

/*
 * Host-side handle of a built plan.  Plain data, owned by the caller, may be
 * copied.  The device blob it points to is owned by the caller too and must stay
 * alive and unmodified while the handle is used.  Fields are filled by
 * litevar_mask_build(); callers may read them, never write them.
 */
typedef struct litevar_plan {
  uint64_t magic;
  void* d_blob;             /* DEVICE */
  uint64_t blob_bytes;
  int32_t n_scales;
  int32_t q_scale_begin, q_scale_end;
  int32_t kv_len;           /* L  = sum of s_k^2 over all scales */
  int32_t q_len;            /* Lq = tokens of the query scales */
  int32_t q_token_begin;    /* index in the full sequence of query row 0 */
  int32_t side_max;         /* largest s_k */
  int32_t waves_per_group;  /* 4x4 query patches handled by one workgroup */
  int32_t chunk_keys;       /* keys per chunk of the key stream (the unit of loading and of LDS ring reuse;
                               64 for 16 patches per group, whose kernel runs phases of two chunks) */
  int32_t ring_chunks;      /* LDS ring depth in chunks = look-back (1) + 1 + prefetch + spare */
  int32_t prefetch_chunks;  /* chunks the loader keeps in flight */
  int32_t n_groups;         /* workgroup tiles per (batch, head) */
  int32_t n_patches;        /* 4x4 query patches per (batch, head) */
  int64_t n_steps;          /* 32-key MFMA steps per (batch, head) */
  int64_t n_union_keys;     /* keys staged through LDS per (batch, head), padded */
  int64_t retained_pairs;   /* allowed (query, key) pairs per (batch, head) */
  int64_t computed_pairs;   /* 16 * 32 * n_steps: pairs the MFMA tiles cover */
  uint64_t off[12];         /* byte offsets of the blob's sections (private) */
  int32_t scales[LITEVAR_MAX_SCALES];
  int32_t radii[LITEVAR_MAX_SCALES];   /* per key scale: the widest radius over the plan's query scales */
  int32_t n_sink_scales;
  int32_t patches_per_wave; /* 16 patches per group only: 0 = chosen per launch, else 1 or 2 */
  int32_t spin_limit;       /* bound of the kernels' LDS-flag waits, in polls */
  int32_t mask_mode;
  int32_t n_heads;          /* 0, or the number of heads the plan holds radius tables for */
  int32_t n_head_groups;    /* distinct radius tables; n_groups, n_patches count one head group,
                               n_steps, n_union_keys, retained_pairs and computed_pairs are summed
                               over the head groups (one group: the values of every head) */
  uint8_t head_group[LITEVAR_MAX_HEADS];           /* head -> head group */
  int64_t retained_pairs_of_group[LITEVAR_MAX_HEADS]; /* kept pairs per (batch, head) of a head group */
} litevar_plan;

/* Tuning knobs of the plan; zero-initialise for the defaults. */
typedef struct litevar_plan_opts {
  int32_t waves_per_group;  /* 4x4 query patches per workgroup: 0 = choose; else 4, 8 or 16 */
  int32_t chunk_keys;       /* keys per phase of the key stream: 0 = choose; else 32, 64 or 128 */
  int32_t prefetch_chunks;  /* chunks kept in flight: 0 = choose */
  int32_t spare_chunks;     /* extra ring chunks that let waves drift apart: -1 = choose.
                               Supported (chunk, prefetch, spare) for 4 and 8 patches per group:
                               (32,2,2) and (64,2,1).  16 patches per group take (128,2,0) only:
                               phases of 128 keys, ring and prefetch depth counted in 64-key chunks */
  int32_t patches_per_wave; /* 16 patches per group only: 0 = choose at each launch (one patch per
                               wave, sixteen waves per workgroup, when the launch has no more
                               working workgroups than the GPU has CUs; else two patches per wave,
                               eight waves), else 1 or 2 */
  int32_t batch_heads_hint; /* 0 = unknown, else the B * H of the launches this plan is for: when
                               waves_per_group is left to the library, few (batch, head) pairs get
                               smaller groups, so that the launch still fills the GPU */
  int32_t spin_limit;       /* 4 and 8 patches per group only: polls (of about 64 cycles) after which a
                               wave's wait on another wave's LDS flag gives up, marks the plan's header
                               (litevar_plan_check then fails) and runs to its end without waiting;
                               0 = default (2^22).  Tests of that path pass 1. */
  int32_t reserved[1];
} litevar_plan_opts;

/*
 * Scale table (Section 2: scale k holds s_k^2 tokens, stored one scale after the other):
 * out_offsets[k] = index of scale k's first token, out_offsets[K] = sequence length.
 * Host-only.  scales: HOST [n_scales]; out_offsets: HOST [n_scales + 1].
 */
litevar_status litevar_scale_offsets(const int32_t* scales, int32_t n_scales, int64_t* out_offsets);

/*
 * Size in bytes of the device blob a plan for `desc` needs.  Host-only, no HIP
 * call.  opts may be NULL.  out_bytes: HOST.
 */
litevar_status litevar_mask_plan_bytes(const litevar_mask_desc* desc,
                                       const litevar_plan_opts* opts, size_t* out_bytes);

/*
 * Host-only dry run of litevar_mask_build(): fills `stats` with the sizes and
 * counts the plan would have (kv_len, q_len, n_groups, n_steps, retained_pairs,
 * computed_pairs, blob_bytes ...) but with magic = 0 and d_blob = NULL, so the
 * result cannot be passed to the device entry points.  No HIP call.
 */
litevar_status litevar_mask_plan_stats(const litevar_mask_desc* desc,
                                       const litevar_plan_opts* opts, litevar_plan* stats);

/*
 * Build the plan on the device (Section 2: per-key-scale parts and their windows):
 * per-(query scale, key scale) window tables, then the work-list (query patches,
 * the key list each workgroup stages through LDS, and per-wave 32-key steps with
 * their mask bits).  d_blob: DEVICE, blob_bytes >= litevar_mask_plan_bytes(), 256-byte
 * aligned.  plan: HOST, filled on success.  The kernels are enqueued on `stream`;
 * the plan may be used by later calls on the same stream without synchronising.
 */
litevar_status litevar_mask_build(const litevar_mask_desc* desc, const litevar_plan_opts* opts,
                                  void* d_blob, size_t blob_bytes, void* stream,
                                  litevar_plan* plan);

/*
 * Synchronises `stream`, reads the blob's header back and checks it against the
 * handle: magic, sizes, the builder's overflow flag, and the mark that an attention
 * kernel leaves when one of its bounded waits gave up.  (Every attention kernel checks
 * magic and builder flag itself and does nothing when they are bad, so a zeroed or
 * half-built blob yields an untouched output, never a hang.)  For tests and debugging.
 */
litevar_status litevar_plan_check(const litevar_plan* plan, void* stream);

/*
 * Window table as built on the device (Section 2: the window of every scale and part), for
 * parity checks; `head` selects the radius table (0 when the plan has one for all heads);
 * window mode only.  d_out is DEVICE int16 [K][K][side_max][2]; entry (k, j, c) holds the inclusive [lo, hi] key
 * coordinates of scale j that query coordinate c of scale k keeps along one axis
 * (the 2-D window is the product of the row and column intervals); (-1, -1) where
 * j > k or c >= s_k.
 */
litevar_status litevar_window_table_export(const litevar_plan* plan, int32_t head, int16_t* d_out,
                                           size_t out_bytes, void* stream);

/*
 * What the work-list encodes (Section 2: the kept pairs of every part), as a dense byte mask
 * of head `head`: d_mask is DEVICE uint8 [q_len][kv_len], 1 = kept pair.  Written from the per-wave steps the attention
 * kernel consumes (not from the window table).  d_pair_count: optional DEVICE
 * uint64[1], receives the number of (query, key) entries in the work-list, which
 * equals the mask's popcount iff no pair is listed twice.
 */
litevar_status litevar_mask_export_dense(const litevar_plan* plan, int32_t head, uint8_t* d_mask,
                                         size_t mask_bytes, uint64_t* d_pair_count,
                                         void* stream);

/*
 * Same content in CSR form (the index sets of Section 2's windows): d_rowptr DEVICE int64
 * [q_len + 1]; d_cols DEVICE int32 [cols_cap], each row's kept keys in ascending token
 * order.  cols_cap >= the head's kept pairs (plan->retained_pairs_of_group[...]).
 */
litevar_status litevar_mask_export_csr(const litevar_plan* plan, int32_t head, int64_t* d_rowptr,
                                       int32_t* d_cols, size_t cols_cap, void* stream);

typedef enum { LITEVAR_BF16 = 0, LITEVAR_F32 = 1 } litevar_dtype;
enum {
  LITEVAR_FLAG_CFG_SHARE = 1u,       /* batch rows [0, B/2) conditional, b + B/2 its partner */
  LITEVAR_FLAG_QKV8_IN_KERNEL = 2u   /* litevar_windowed_attn_qkv8_fwd only: convert the 8-bit operands in
                                        the attention kernel whatever the plan's shape (the plan must have
                                        16 patches per group); no workspace is used */
};

/*
 * O = softmax(sm_scale * Q K^T restricted to the plan's kept pairs) V   (Section 2),
 * optionally followed by the cond -> uncond output reuse of Section 3.
 *
 *   d_q            DEVICE [B, H, q_len, D]; d_k, d_v DEVICE [B, H, kv_len, D];
 *   d_o            DEVICE [B, H, q_len, D], written; must not alias the inputs.
 *   D              head dimension, must be 64.
 *   dt             element type of q, k, v, o.  BF16: bf16 MFMA with fp32 accumulation,
 *                  probabilities rounded to bf16 before P V.  F32: fp32 throughout.
 *   q_strides, kv_strides, o_strides
 *                  HOST, element strides of the (B, H, token) axes; the D axis is
 *                  contiguous.  NULL = packed.  Rows must be 16-byte aligned.
 *   sm_scale       softmax scale (1/sqrt(D) in VAR), finite, > 0.
 *   d_cfg_share    DEVICE uint8 [H][K], indexed by (head, query scale); read only
 *                  when LITEVAR_FLAG_CFG_SHARE is set (then B must be even): where
 *                  non-zero the conditional workgroup stores its output to both rows
 *                  and the unconditional one does no work.
 * Inputs must be finite.  Asynchronous on `stream`.
 */
litevar_status litevar_windowed_attn_fwd(const litevar_plan* plan, const void* d_q,
                                         const void* d_k, const void* d_v, void* d_o,
                                         int32_t B, int32_t H, int32_t D, litevar_dtype dt,
                                         const int64_t* q_strides, const int64_t* kv_strides,
                                         const int64_t* o_strides, float sm_scale,
                                         const uint8_t* d_cfg_share, uint32_t flags,
                                         void* stream);

/*
 * Window calibration (paper Section 2: the metric R_w and the threshold R_0).  From
 * post-softmax attention maps of N reference samples, for every head, query scale k and
 * key scale j <= k: the smallest radius r >= 0 such that the values inside the radius-r
 * windows of the part (query scale k, key scale j), summed over the part's queries and the
 * samples, reach the fraction r0 of all of the part's values (r0 = 1 keeps every non-zero
 * value).  Windows and centres are those of litevar_mask_build's window mode; a part without
 * mass gets radius 0.  Parts are one per key scale here: the merged first part of Section 2,
 * step (2) is not modelled, which is immaterial when the first three key scales are kept
 * dense (n_sink_scales = 3).
 *
 *   scales, n_scales  HOST, as in litevar_mask_desc
 *   d_attn       DEVICE float32 [N][H][L][L], contiguous, L = sum of s_k^2: row q holds
 *                query q's weights over all keys (entries of later scales are not read)
 *   r0           in (0, 1]
 *   d_workspace  DEVICE, 8-byte aligned, at least
 *                litevar_window_calibrate_workspace_bytes() bytes; contents undefined
 *                before and after; calls that share a workspace must not overlap
 *   d_radius     DEVICE int32 [H][K][K], written: [h][k][j] as above, -1 where j > k
 *   d_mass       DEVICE float64 [H][K][K][smax] or NULL (smax = largest side): the sum
 *                inside the window of radius r, for the parity tests
 * Sums are formed in fp64 in a fixed order (repeatable bit for bit).  Host arrays are read
 * during the call only; the library allocates nothing; asynchronous on `stream`.
 */
litevar_status litevar_window_calibrate_workspace_bytes(const int32_t* scales, int32_t n_scales,
                                                        int32_t H, size_t* out_bytes);
litevar_status litevar_window_calibrate(const int32_t* scales, int32_t n_scales,
                                        const float* d_attn, int32_t N, int32_t H, float r0,
                                        void* d_workspace, size_t workspace_bytes,
                                        int32_t* d_radius, double* d_mass, void* stream);

/*
 * The same calibration for the band mask mode (Section 2, step (2) read literally:
 * LITEVAR_MASK_BAND_1D): the map of query scale k is cut into parts -- the first three key
 * scales together, then one part per key scale -- and in every part the band around the
 * part's diagonal grows from radius zero until it holds the fraction r0 of the part's values
 * (n - 1 at the latest, n = the part's columns).
 *   d_radius     DEVICE int32 [H][K][K]: the radius of the part that key scale j belongs to,
 *                the same value for the key scales of the merged part, -1 for j > k: the layout
 *                of litevar_mask_desc.radius_per_head for a band plan.
 *   d_mass       DEVICE double [H][K][K][C] or NULL, C = the largest number of columns of a part
 *                (max of s_1^2 + s_2^2 + s_3^2 and the later s_j^2): in-band sums by radius, the
 *                part's sum from radius n - 1 on.
 *   d_workspace  DEVICE, 8-byte aligned, litevar_window_calibrate_band_workspace_bytes() bytes.
 * Scale sides up to 64, parts of at most 4096 columns.  Other arguments and conventions as
 * litevar_window_calibrate.
 */
litevar_status litevar_window_calibrate_band_workspace_bytes(const int32_t* scales, int32_t n_scales,
                                                             int32_t H, size_t* out_bytes);
litevar_status litevar_window_calibrate_band(const int32_t* scales, int32_t n_scales,
                                             const float* d_attn, int32_t N, int32_t H, float r0,
                                             void* d_workspace, size_t workspace_bytes,
                                             int32_t* d_radius, double* d_mass, void* stream);

/*
 * QKV8 (Section 4, "Quantization Scheme": min-max quantisation of Q, K and V to 8-bit
 * integers with dynamic parameters computed online from the data's maximum and minimum).
 * One (scale s, zero point z) per token row of D = 64 values:
 *   z = (max + min)/2,  s = ((max - min)/2) / 127,  code = rne(clamp((x - z)/s, -128, 127)),
 *   dequantised value = s * code + z   (a constant row has s = 0 and codes 0).
 * The printed formula's scale lacks the integer range and its clamp's upper bound is not an
 * 8-bit code; this is the repaired min-max form with the paper's zero point.  Codes are
 * decided in binary32 in the order written above.
 *
 * litevar_qkv8_quantize    d_x DEVICE bf16 or fp32 [rows][row_stride >= 64] (16-byte aligned
 *                          rows), d_codes DEVICE int8 [rows][64], d_scale_zero DEVICE float
 *                          [rows][2] = (s, z) per row.
 * litevar_qkv8_dequantize  d_out_bf16 DEVICE bf16 [rows][64] = bf16(s * code + z).
 * litevar_windowed_attn_qkv8_fwd
 *                          litevar_windowed_attn_fwd on 8-bit operands: d_q int8
 *                          [B,H,q_len,64] with d_q_sz float [B,H,q_len,2], d_k / d_v int8
 *                          [B,H,kv_len,64] with their (s, z); all packed.  d_o DEVICE bf16
 *                          [B,H,q_len,64].  Plans with 16 patches per group whose groups
 *                          stream at most a quarter more key rows than the tensors hold (KV-cache steps) hand codes and
 *                          parameters to the attention kernel, which converts them on their way
 *                          into LDS; litevar_windowed_attn_qkv8_workspace_bytes() is then 0 and
 *                          d_workspace is ignored.  For other plans the operands are
 *                          dequantised once into d_workspace (DEVICE, 256-byte aligned, that
 *                          many bytes, contents undefined before and after) and the bf16 kernels
 *                          run on that copy.  Either way the results equal attention on the
 *                          dequantised tensors up to their rounding to bf16 and the bf16 path's
 *                          own rounding.  LITEVAR_FLAG_QKV8_IN_KERNEL in `flags` asks for the
 *                          first form whatever the plan's shape (LITEVAR_E_UNSUPPORTED unless
 *                          the plan has 16 patches per group).  Other arguments as
 *                          litevar_windowed_attn_fwd.  Asynchronous on `stream`.
 */
litevar_status litevar_qkv8_quantize(const void* d_x, litevar_dtype dt, int64_t rows, int64_t row_stride,
                                     int32_t D, int8_t* d_codes, float* d_scale_zero, void* stream);
litevar_status litevar_qkv8_dequantize(const int8_t* d_codes, const float* d_scale_zero, int64_t rows,
                                       int32_t D, void* d_out_bf16, void* stream);
litevar_status litevar_windowed_attn_qkv8_workspace_bytes(const litevar_plan* plan, int32_t B, int32_t H,
                                                          size_t* out_bytes);
litevar_status litevar_windowed_attn_qkv8_fwd(const litevar_plan* plan, const int8_t* d_q,
                                              const float* d_q_sz, const int8_t* d_k,
                                              const float* d_k_sz, const int8_t* d_v,
                                              const float* d_v_sz, void* d_o, int32_t B, int32_t H,
                                              int32_t D, float sm_scale, const uint8_t* d_cfg_share,
                                              uint32_t flags, void* d_workspace, size_t workspace_bytes,
                                              void* stream);

/*
 * Diagnostics for benchmark reports (measurement, Section 4's efficiency figures are quoted
 * against what the hardware delivers): litevar_peak_copy enqueues a streaming copy of `bytes`
 * bytes (DEVICE pointers, 16-byte aligned, size a multiple of 16; HBM traffic = 2 x bytes);
 * litevar_peak_read enqueues a read-only pass over `bytes` bytes (HBM traffic = bytes);
 * litevar_peak_mfma_bf16 enqueues a register-only loop of v_mfma_f32_16x16x32_bf16 (8 waves on
 * every SIMD, `iters` x 8 independent MFMAs per wave) and returns the floating-point
 * operations it performs in *flops (HOST, optional).  d_out: DEVICE, 4 bytes, never written
 * in practice.  The caller times them with events on `stream`.
 */
litevar_status litevar_peak_copy(const void* d_src, void* d_dst, size_t bytes, void* stream);
litevar_status litevar_peak_read(const void* d_src, size_t bytes, void* d_out, void* stream);
litevar_status litevar_peak_mfma_bf16(int32_t iters, void* d_out, double* flops, void* stream);

/*
 * litevar_window_calibrate for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as litevar_window_calibrate, but the
 * per-workgroup partial sums live in an array that is part of the library's device image
 * (LITEVAR_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of a caller's
 * workspace.  Calls no allocating routine.  Problems whose partial sums
 * (litevar_window_calibrate_workspace_bytes) exceed the array are rejected with
 * LITEVAR_E_UNSUPPORTED before anything is launched (the 256x256 VAR scale list fits for
 * up to 40 heads).  The first call on a device resolves the array's address
 * (hipGetSymbolAddress); make that call outside a capture.  All calls on one GPU share the
 * array: calls that overlap on one GPU (different streams) race; calls on one stream are
 * ordered and need no clearing, since every partial sum that is read is written first.
 */
#define LITEVAR_STATIC_SCRATCH_BYTES (8u << 20)
litevar_status litevar_window_calibrate_static(const int32_t* scales, int32_t n_scales,
                                               const float* d_attn, int32_t N, int32_t H, float r0,
                                               int32_t* d_radius, double* d_mass, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LITEVAR_H_ */
