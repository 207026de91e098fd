/*
 * slkv.h - C ABI of the SurfaceLogicKV prefill KV-compression pass for AMD MI355X (gfx950).
 *
 * The paper (arXiv 2508.15806) defines a two-stage method:
 *   Stage 1 (Section 3.2, Algorithm 1): per attention head, count how the attention mass of
 *     decode rows over a needle-in-a-haystack prompt splits into correct / distracted /
 *     subconscious weight and form SF_sc, LG_sc and INF_sc          -> slkv_score_heads
 *   Stage 2a (Section 3.3, Eq. 6, Algorithm 2): turn the INF_sc map into one integer KV
 *     capacity per (layer, head): a fixed part plus a share of a dynamic pool
 *                                                                    -> slkv_allocate_budgets
 *   Stage 2b (Section 3.4, Eq. 7-8, Algorithm 3): at prefill, per layer and head, score the
 *     history keys against the last window of queries, keep the top-ranked history entries
 *     within the capacity plus the whole window                      -> slkv_compress_layer
 *     The same selection on a cache that is already compacted and has grown during generation
 *     (heads of different lengths)                                   -> slkv_recompress_layer
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller owns every
 *     buffer; the library allocates no device memory.  What it keeps between calls: per device,
 *     that its one-time set-up has been done (slkv_init), the counters at the start of a
 *     workspace (see slkv_compress_layer), and the optional kernel-timing recorder at the end
 *     of this header.
 *   - slkv_score_heads, slkv_compress_layer and slkv_recompress_layer only enqueue work on `hip_stream` (a
 *     hipStream_t passed as void*, NULL = the default stream) and return without
 *     synchronising.  Host-side descriptors are consumed before the call returns.
 *   - Every argument is validated before the first GPU call; on any error nothing is
 *     enqueued and no output is written.  slkv_last_error() gives a detail string for the
 *     calling thread.
 *   - Device pointers must be 16-byte aligned.
 */
#ifndef SLKV_H
#define SLKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SLKV_OK = 0,
  SLKV_ERR_NULL = 1,        /* a required pointer is NULL */
  SLKV_ERR_BAD_ARG = 2,     /* a size / count / stride / alignment is invalid */
  SLKV_ERR_BAD_VALUE = 3,   /* host data out of range (INF_sc not in [0,1], NaN, ...) */
  SLKV_ERR_UNSUPPORTED = 4, /* valid but outside what the kernels cover (head_dim, rows) */
  SLKV_ERR_WORKSPACE = 5,   /* workspace smaller than slkv_workspace_bytes() */
  SLKV_ERR_CAPACITY = 6,    /* output buffers smaller than slkv_compacted_sizes() */
  SLKV_ERR_HIP = 7          /* a HIP call failed (kernel launch) */
} slkv_status;

/* Element type of Q, K and V.  SLKV_BF16_KV_FP8: queries bfloat16, keys and values 8-bit floating
 * point in the OCP E4M3 encoding (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals,
 * no infinities, S.1111.111 = NaN), one byte per element; strides of d_k / d_v count bytes then. */
typedef enum { SLKV_F32 = 0, SLKV_BF16 = 1, SLKV_F16 = 2, SLKV_BF16_KV_FP8 = 3 } slkv_dtype;
typedef enum { SLKV_POOL_NONE = 0, SLKV_POOL_MAX = 1, SLKV_POOL_AVG = 2 } slkv_pool;
typedef enum { SLKV_BUDGET_EXACT = 0, SLKV_BUDGET_PAPER_LITERAL = 1, SLKV_BUDGET_EXACT_PER_QUERY_HEAD = 2 } slkv_budget_mode;

/* Static description of a status code. */
const char* slkv_status_str(slkv_status s);
/* Detail of the last error on the calling thread; valid until its next slkv call. */
const char* slkv_last_error(void);
/* ABI version: major * 1000 + minor. */
int32_t slkv_version(void);
/* One-time set-up on the CURRENT device (host pointer arguments: none): raises the LDS limit of
 * the selection kernels and looks up the scratch of slkv_compress_layer_static.  Optional: a
 * call that finds its device not set up does this itself, which is why the first call on a
 * device must not be the one a stream capture records unless slkv_init() has run there before.
 * Thread-safe, idempotent, enqueues nothing on a stream.  SLKV_ERR_HIP if a HIP call fails. */
slkv_status slkv_init(void);

/* ------------------------------------------------------------------ Stage 1 -----------
 * Algorithm 1 (Section 3.2).  For every row W (length n) of every head: T_k = the `topk`
 * largest weights (equal weights rank by lower position),
 *   WO = sum of W over needle and T_k, WD = sum of W over T_k outside the needle,
 *   TNW = sum of W over the needle, WS = max(0, TNW - WO), Wide = sum(W) - WO - WD - WS.
 * The five accumulators of head (l,h) are increased by the sums over its T rows, so several
 * calls (other prompts, depths, lengths) accumulate into the same d_acc.  If d_scores is not
 * NULL it receives, from the updated accumulators,
 *   SF = WO/(WO+WD), LG = WO/(WO+WS), INF = 2 SF LG/(SF+LG)   (0/0 = 0).
 *
 * d_rows    [L][H][T][n] fp32, rows contiguous (device, read only)
 * needle    [needle_start, needle_start + needle_len) inside [0, n), the same for all rows
 * topk      1..n
 * d_acc     [L][H][5] double, in/out: sum WO, sum WD, sum WS, sum Wide, row count.  The
 *           caller zeroes it before the first call.
 * d_scores  [L][H][3] double out, may be NULL
 * d_workspace / workspace_bytes: at least slkv_score_heads_workspace_bytes(L,H,T,n) bytes
 * Errors: NULL, BAD_ARG (sizes, needle, topk, alignment), WORKSPACE, HIP.
 */
slkv_status slkv_score_heads(const float* d_rows, int32_t L, int32_t H, int32_t T, int64_t n,
                             int64_t needle_start, int32_t needle_len, int32_t topk,
                             double* d_acc, double* d_scores,
                             void* d_workspace, size_t workspace_bytes, void* hip_stream);
size_t slkv_score_heads_workspace_bytes(int32_t L, int32_t H, int32_t T, int64_t n);

/* Algorithm 1 with the ablation of Section 4.2 (Table 4) and the aggregation over a head's rows
 * as parameters.  The paper prints no formula for an ablated score; here a component that is
 * switched off enters steps 5-6 of Algorithm 1 as 0 (without WS: LG = WO/WO; without WD:
 * SF = WO/WO; without WO: both 0).
 *   aggregation SLKV_AGG_MICRO: the head's scores come from its cells summed over all rows
 *     (what slkv_score_heads does);
 *   aggregation SLKV_AGG_MACRO: SF and LG are taken per row, averaged over the head's rows
 *     (every row counts, a row with 0/0 as 0), and step 7 (INF) is applied to the two means.
 * d_acc [L][H][8] double, in/out, zeroed by the caller before the first call:
 *   sum WO, sum WD, sum WS, sum Wide, row count, sum of per-row SF, sum of per-row LG, 0
 *   (the per-row SF / LG use the same components).  Everything else as slkv_score_heads.
 */
typedef enum { SLKV_AGG_MICRO = 0, SLKV_AGG_MACRO = 1 } slkv_aggregation;
typedef struct {
  uint32_t struct_size;   /* sizeof(slkv_score_params) */
  int32_t aggregation;    /* slkv_aggregation */
  int32_t use_wo, use_wd, use_ws;   /* 0 / 1: the "-" / "+" of Table 4 */
  int32_t reserved;       /* 0 */
} slkv_score_params;
slkv_status slkv_score_heads_ex(const slkv_score_params* params, const float* d_rows,
                                int32_t L, int32_t H, int32_t T, int64_t n,
                                int64_t needle_start, int32_t needle_len, int32_t topk,
                                double* d_acc, double* d_scores,
                                void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Stage 1 without attention rows in memory (Section 3.1, Eq. 2-4, feeding Algorithm 1): the row of
 * query head hq at decode step t is softmax_j(q[l][hq][t] . k[l][hq / (Hq/Hkv)][j] / sqrt(d)) over the
 * n context keys; the kernels compute the logits, the top-K set and the weight cells of every row
 * on chip and add them into d_acc exactly as slkv_score_heads does.  Logits are fp32 sums of exact
 * bf16 products, weights fp32 exponentials of them, so the cells agree with float64 arithmetic on
 * the same inputs to about 1e-5 relative; two logits that differ by less than fp32 rounding may
 * swap places in the top-K set.
 *
 * d_q   [L][Hq][T][d] bf16 queries of the T decode steps (device, read only)
 * d_k   [L][Hkv][n][d] bf16 context keys (device, read only); Hq % Hkv == 0, d in {64, 128},
 *       n*d*2 < 2^31; topk <= 64 (larger K: materialise the rows and call slkv_score_heads)
 * d_acc [L][Hq][5], d_scores [L][Hq][3] (may be NULL): as in slkv_score_heads
 * Errors: NULL, BAD_ARG, UNSUPPORTED (d, topk, size), WORKSPACE, HIP.
 */
slkv_status slkv_score_heads_qk(const void* d_q, const void* d_k, int32_t L, int32_t Hq, int32_t Hkv,
                                int32_t T, int64_t n, int32_t d,
                                int64_t needle_start, int32_t needle_len, int32_t topk,
                                double* d_acc, double* d_scores,
                                void* d_workspace, size_t workspace_bytes, void* hip_stream);
size_t slkv_score_heads_qk_workspace_bytes(int32_t L, int32_t Hq, int32_t T, int64_t n);

/* ------------------------------------------------------------------ Stage 2a ----------
 * Eq. (6) / Algorithm 2.  Pure host code, no GPU call.
 *
 * h_inf      [L][Hq] INF_sc per query head, each finite and in [0, 1]
 * Hkv        KV heads per layer; Hq % Hkv == 0.  The INF_sc of the Hq/Hkv query heads that
 *            share a KV head are averaged first; capacities are per KV head.
 * avg_budget average capacity per KV head (b_c); fixed_budget the fixed part b_c(1 - 1/beta),
 *            0 <= fixed <= avg.
 * mode       SLKV_BUDGET_EXACT: a layer's share of the dynamic pool (avg-fixed)*L*Hkv is
 *              proportional to 0.01 + (layer INF sum / total INF sum), a head's share inside
 *              its layer is proportional to its INF_sc; both splits use the largest-remainder
 *              rule on exact integers (INF_sc quantised to 2^-30), so the capacities are
 *              integers >= fixed that sum to avg*L*Hkv exactly.
 *            SLKV_BUDGET_PAPER_LITERAL: Algorithm 2 as printed (global normalisation, the 0.01
 *              offset not renormalised, each head rounded half up on its own); does not sum
 *              to the total.
 *            SLKV_BUDGET_EXACT_PER_QUERY_HEAD: Algorithm 2 read with its heads = the Hq query
 *              heads (the paper does not mention grouped-query attention): the EXACT rule gives
 *              every query head a capacity (average avg_budget, fixed part fixed_budget), and
 *              a KV head, whose cache serves its Hq/Hkv query heads, keeps the sum of theirs;
 *              the capacities sum to avg*L*Hq.
 * h_budgets  [L][Hkv] out.
 * Errors: NULL, BAD_ARG (sizes, Hq % Hkv, fixed > avg, overflow), BAD_VALUE (INF_sc).
 */
slkv_status slkv_allocate_budgets(const double* h_inf, int32_t L, int32_t Hq, int32_t Hkv,
                                  int32_t avg_budget, int32_t fixed_budget, int32_t mode,
                                  int32_t* h_budgets);
/* floor(avg * (1 - 1/beta) + 0.5): the fixed part of Algorithm 2 for a ratio beta >= 1. */
int32_t slkv_fixed_from_beta(int32_t avg_budget, double beta);

/* ------------------------------------------------------------------ Stage 2b ----------
 * Algorithm 3 for one layer over a ragged batch of B sequences.
 * Sequence b has n_b = cu_seqlens[b+1] - cu_seqlens[b] tokens; its last w tokens are the
 * observation window, the first m_b = n_b - w its history.  For KV head h with capacity C_h:
 *   n_b <= C_h or n_b <= w : every token is kept;
 *   otherwise k = min(max(C_h - w, 0), m_b) history tokens are kept, those with the largest
 *   pooled importance (equal scores rank by lower position), followed by the window.
 * importance[j] = sum over the G = Hq/Hkv query heads of the group and the w window queries of
 *   softmax_j(q . k_j / sqrt(d)) with the softmax over the m_b history keys only;
 * pooled = stride-1 same-length pool of width pool_kernel over importance (max: window clipped
 *   at the ends; avg: zeros outside, divided by pool_kernel).
 * Kept rows of K and V are copied bit for bit, history positions ascending then the window.
 */
typedef struct {
  uint32_t struct_size;       /* sizeof(slkv_layer_desc) */
  int32_t dtype;              /* slkv_dtype of Q, K, V: fp32 (plain FMA kernels), bf16, fp16, or bf16 queries with
                                 E4M3 keys and values (MFMA kernels, products exact in the fp32 accumulators) */
  int32_t B, Hq, Hkv, d, w;   /* d in {64, 128}; w >= 1; Hq % Hkv == 0; (Hq/Hkv)*w <= 512 */
  int32_t pool_kernel;        /* odd, 1..63; 1 = no pooling */
  int32_t pool;               /* slkv_pool */
  int32_t reserved;           /* 0 */
  const int64_t* h_cu_seqlens; /* [B+1] host: token offsets into the packed K/V, non-decreasing,
                                  cu[0] >= 0, cu[B] < 2^31 */
  int64_t k_stride_tok, k_stride_head; /* elements between tokens / KV heads of d_k; rows of d
                                          elements are contiguous; both multiples of 8 */
  int64_t v_stride_tok, v_stride_head; /* same for d_v */
  const int32_t* h_budgets;   /* [Hkv] host: this layer's capacities C_h >= 0 */
} slkv_layer_desc;

/* Kept-row counts.  h_out_offsets[B*Hkv+1] (host, may be NULL) receives the exclusive scan of
 * the kept counts in segment order s = b*Hkv + h; *total_kept (may be NULL) their sum. */
slkv_status slkv_compacted_sizes(const slkv_layer_desc* desc, int64_t* h_out_offsets,
                                 int64_t* total_kept);
/* Device workspace slkv_compress_layer needs for this descriptor.
 * A workspace has to be ZERO-FILLED ONCE by the caller before the first call that uses it (its
 * first SLKV_WORKSPACE_HEADER_BYTES hold counters with which the workgroups of a kernel find
 * out which of them finishes a segment last); every call leaves them zero again, so the same
 * workspace serves any number of later calls, of any descriptor it is large enough for, also
 * from a replayed HIP graph.  Its other contents are scratch.  Two calls that may overlap in
 * time need a workspace each. */
#define SLKV_WORKSPACE_HEADER_BYTES 65536
slkv_status slkv_workspace_bytes(const slkv_layer_desc* desc, size_t* bytes);

/* d_qwin   [B][Hq][w][d] window queries (device, read only)
 * d_k, d_v packed keys / values: element (h, t, :) at h*stride_head + t*stride_tok
 * d_k_out, d_v_out [total_kept][d] out, segment s at row h_out_offsets[s]
 * d_kept_idx [total_kept] int32 out: kept positions inside the sequence, per segment
 * d_out_offsets [B*Hkv+1] int64 out, may be NULL: device copy of the offsets
 * d_importance, d_pooled: may be NULL.  fp32 [Hkv * cu[B]] each; segment (b,h) occupies
 *          m_b entries starting at Hkv*cu[b] + h*n_b and is written only when the segment is
 *          actually ranked (n_b > max(C_h, w) and 0 < k < m_b).
 * out_capacity_rows: rows available in d_k_out / d_v_out / d_kept_idx
 * d_k, d_v may be NULL when the batch holds no tokens; d_k_out, d_v_out, d_kept_idx when nothing is kept.
 * Errors: NULL, BAD_ARG, UNSUPPORTED, WORKSPACE, CAPACITY, HIP.
 */
slkv_status slkv_compress_layer(const slkv_layer_desc* desc, const void* d_qwin,
                                const void* d_k, const void* d_v,
                                void* d_k_out, void* d_v_out, int32_t* d_kept_idx,
                                int64_t* d_out_offsets, float* d_importance, float* d_pooled,
                                int64_t out_capacity_rows,
                                void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* slkv_compress_layer for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as slkv_compress_layer without the workspace: the scratch
 * (chunk statistics, log-sum-exp, importance, pooled scores, block histograms, segment table) lives in a buffer of
 * SLKV_STATIC_SCRATCH_BYTES that is part of the library's code object, one copy per GPU, held
 * until the process ends.  A call whose slkv_workspace_bytes() exceeds that size returns
 * SLKV_ERR_WORKSPACE and enqueues nothing.  The call allocates nothing (no hipMalloc / hipFree).
 * All calls on one GPU share the buffer: calls that may overlap on one GPU (different streams
 * without ordering between them, or several host threads) race and must be serialised by the
 * caller.  The buffer's address is looked up on the first call on each device; make that call
 * outside stream capture.
 */
#define SLKV_STATIC_SCRATCH_BYTES (8u << 20)
slkv_status slkv_compress_layer_static(const slkv_layer_desc* desc, const void* d_qwin,
                                       const void* d_k, const void* d_v,
                                       void* d_k_out, void* d_v_out, int32_t* d_kept_idx,
                                       int64_t* d_out_offsets, float* d_importance, float* d_pooled,
                                       int64_t out_capacity_rows, void* hip_stream);

/* ------------------------------------------------------------------ Stage 2b on a ragged cache
 * Section 3.4 runs the selection whenever a head's cache length exceeds its capacity, which
 * also happens during generation, when the cache is the compacted output of an earlier call
 * plus the tokens appended since.  Input here is such a cache: segment s = b*Hkv + h owns the
 * packed rows h_in_offsets[s] .. h_in_offsets[s+1] of d_k_in / d_v_in ([rows][d], rows
 * contiguous), its length n_s differs from head to head, and its last w rows are the window
 * (the latest w tokens, whose queries are d_qwin[b]).  Everything else is Algorithm 3 exactly
 * as in slkv_compress_layer, with n_s in place of n_b.
 */
typedef struct {
  uint32_t struct_size;        /* sizeof(slkv_ragged_desc) */
  int32_t dtype;               /* slkv_dtype of Q, K, V */
  int32_t B, Hq, Hkv, d, w;    /* as in slkv_layer_desc */
  int32_t pool_kernel, pool;   /* as in slkv_layer_desc */
  int32_t reserved;            /* 0 */
  const int64_t* h_in_offsets; /* [B*Hkv+1] host: first input row of every segment, non-decreasing,
                                  >= 0, last < 2^31 */
  const int32_t* h_budgets;    /* [Hkv] host: capacities C_h >= 0 */
} slkv_ragged_desc;

/* Kept-row counts of slkv_recompress_layer (same outputs as slkv_compacted_sizes). */
slkv_status slkv_recompress_sizes(const slkv_ragged_desc* desc, int64_t* h_out_offsets,
                                  int64_t* total_kept);
/* Device workspace slkv_recompress_layer needs for this descriptor (zero-filled once before its
 * first use, like the workspace of slkv_compress_layer). */
slkv_status slkv_recompress_workspace_bytes(const slkv_ragged_desc* desc, size_t* bytes);

/* d_qwin   [B][Hq][w][d] queries of the latest w tokens (device, read only)
 * d_k_in, d_v_in [rows][d] packed cache (device, read only)
 * d_pos_in  [rows] int32, may be NULL: original token position of every cached row
 * d_k_out, d_v_out [total_kept][d] out; d_kept_idx [total_kept] int32 out: kept row numbers
 *           inside the segment (ascending, the window last)
 * d_pos_out [total_kept] int32 out, NULL exactly when d_pos_in is NULL: d_pos_in at the kept rows,
 *           so that positions survive any number of compressions
 * d_out_offsets [B*Hkv+1] int64 out, may be NULL
 * d_importance, d_pooled: may be NULL.  fp32 [rows] each; segment s occupies n_s - w entries
 *           starting at h_in_offsets[s] - h_in_offsets[0], written only when the segment is ranked.
 * The outputs must not overlap the inputs.  Errors as slkv_compress_layer.
 */
slkv_status slkv_recompress_layer(const slkv_ragged_desc* desc, const void* d_qwin,
                                  const void* d_k_in, const void* d_v_in, const int32_t* d_pos_in,
                                  void* d_k_out, void* d_v_out, int32_t* d_kept_idx,
                                  int32_t* d_pos_out, int64_t* d_out_offsets,
                                  float* d_importance, float* d_pooled, int64_t out_capacity_rows,
                                  void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------ kernel timing -----
 * Optional instrumentation for benchmarks: between slkv_profile_begin and slkv_profile_end
 * every kernel the library launches is bracketed by a HIP event pair on the call's stream.
 * slkv_profile_begin creates the events it needs (the only state the library ever keeps);
 * slkv_profile_end waits for the recorded events, writes up to `capacity` records in launch
 * order and sets *count to the number recorded.  Process-wide; not meant for production.
 */
typedef enum {
  SLKV_K_SCORE_STATS = 0,   /* logits + per-row sum-exp of every key chunk */
  SLKV_K_COMBINE = 1,       /* not launched any more: the statistics pass folds the chunks itself */
  SLKV_K_SCORE_ACCUM = 2,   /* logits + exp(logit - lse) summed down the rows */
  SLKV_K_SELECT = 3,        /* pooling + top-k (one record per launch: one launch for histories up to 32768 positions, six for longer ones) */
  SLKV_K_GATHER = 4,        /* K/V row gather */
  SLKV_K_ROW_CELLS = 5,     /* Stage 1: per-row weight cells */
  SLKV_K_HEAD_REDUCE = 6,   /* Stage 1: per-head sums and scores */
  SLKV_K_QK_CELLS = 7,      /* Stage 1 from queries and keys: logits, top-K and cells of every row */
  SLKV_K_QK_FALLBACK = 8    /* the same for rows whose candidate list overflowed */
} slkv_kernel_id;
typedef struct {
  int32_t kernel; /* slkv_kernel_id */
  float ms;       /* elapsed time between the launch's two events */
} slkv_kernel_time;
slkv_status slkv_profile_begin(int32_t max_records);
slkv_status slkv_profile_end(slkv_kernel_time* h_records, int32_t capacity, int32_t* count);

#ifdef __cplusplus
}
#endif
#endif /* SLKV_H */
