/*
 * wkv.h — C ABI of the MI355X (gfx950) WindowKV prefill-time KV-cache window selection.
 *
 * The library computes, for one batch of sequences and one or more layer groups, what
 * Section 2.2 of the WindowKV paper (arXiv 2503.17922) defines:
 *
 *   Eq. 1   A = softmax(Q K^T / sqrt(d_k))           causal, over the whole prefix
 *   Eq. 2   t_j = sum_{i in last w_obs rows} A_ij      j in the review context [0, L - w_obs)
 *           (summed also over the G = Hq/Hkv query heads that share a KV head)
 *   Eq. 3   review windows W_k of `win` consecutive tokens (the last may be partial)
 *   Eq. 4   s_k = sum(Top-p(W_k)) / min(p, win)
 *   2.2.1   keep the k highest-scoring windows plus the last w_obs tokens
 *   2.2.2   the first layer of a group is scored; every layer of the group keeps the rows
 *           at those indices.
 *
 * Notation: L = prefix length (paper: n), w_obs = observation window (alpha), win = review
 * window size (omega), p = top_p, gamma = layers per group, NW = ceil((L - w_obs)/win).
 *
 * Conventions common to every call
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are read
 *     during the call only and may be freed on return.
 *   - Work is enqueued on the caller's hipStream_t (passed as void*; NULL = default stream).
 *     Calls return without synchronising; results are valid in stream order.
 *   - The library allocates nothing, frees nothing and keeps no device state between calls (its
 *     only state is the calling thread's last error message, see wkv_last_error).
 *     Every call except wkv_compress_groups_profiled is a fixed sequence of kernel launches on
 *     the stream (no memset or copy nodes, no host synchronisation), so it can be captured into
 *     a HIP graph; host arrays are read at capture time.
 *   - Every argument is validated on the host before the first launch; a failed validation
 *     launches nothing.  Errors come back as wkv_status; nothing is thrown.
 *   - All index outputs are int32.  Tensors are addressed with 64-bit offsets.
 */
#ifndef WKV_H
#define WKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WKV_MAX_BATCH      64     /* sequences per call                                   */
#define WKV_MAX_GROUPS     64     /* layer groups per wkv_compress_groups call            */
#define WKV_MAX_LAYERS     64     /* layers per wkv_gather_group / wkv_compress_groups    */
#define WKV_MAX_WIN        128    /* largest review-window size                           */
#define WKV_MAX_OBS_ROWS   256    /* largest G * w_obs                                    */
#define WKV_MAX_WINDOWS    32768  /* largest NW of any sequence                           */

/* wkv_problem.flags.  By default the gather zero-fills rows n_keep[b,h] .. nkeep_max-1 of every
 * compact cache, so that the whole output is defined.  In a batch of mixed lengths these rows
 * are a large share of the bytes written; a caller that never reads them (the decode step
 * does not) sets WKV_KEEP_PADDING and they are left as they were. */
#define WKV_KEEP_PADDING   1
/* How Eq. 1-2 read the keys of the scored layer.  The library uses its two-pass kernels (softmax
 * statistics, then scores: the keys are streamed twice).  WKV_SCORE_SINGLE_READ selects the
 * single-read kernel instead where it applies (16-bit inputs, at most 128 softmax rows per KV head,
 * no normalisers handed over; ignored elsewhere): every key slice stays on chip between the
 * statistics phase and the score phase and workgroups exchange the row statistics through the
 * workspace.  On MI355X that exchange costs more than the second read it saves, so this is an
 * option for measurements, not the default.  WKV_SCORE_TWO_PASS states the default explicitly.
 * Results of the two agree to fp32 rounding of the normalisers.
 * WKV_DEBUG_WAIT_GIVES_UP makes every cross-workgroup wait of the
 * single-read kernel give up at once, which exercises its fall-back: the kernel exits normally,
 * raises a word in the workspace, and the two-pass kernels enqueued behind it (which return at
 * once otherwise) recompute the scores.  The same happens by itself if a wait ever runs out, e.g.
 * when other work keeps part of the grid from being resident. */
#define WKV_SCORE_TWO_PASS        2
#define WKV_SCORE_SINGLE_READ     4
#define WKV_DEBUG_WAIT_GIVES_UP   8

typedef enum {
  WKV_OK = 0,
  WKV_ERR_INVALID_ARG = -1,   /* null pointer, inconsistent sizes, out-of-range parameter */
  WKV_ERR_UNSUPPORTED = -2,   /* valid problem outside the limits above / dtype / head_dim */
  WKV_ERR_WORKSPACE   = -3,   /* workspace missing, misaligned or too small                */
  WKV_ERR_HIP         = -4    /* a HIP call or kernel launch failed                        */
} wkv_status;

typedef enum { WKV_F32 = 0, WKV_BF16 = 1, WKV_F16 = 2 } wkv_dtype;   /* fp32, bfloat16, IEEE half */

/*
 * One batch of sequences.  The same description serves one layer group or several (the
 * per-sequence parameters are shared by all groups of a call).
 *
 * Tensor layouts (strides in ELEMENTS; the head_dim axis always has stride 1):
 *   q_obs   [batch, n_q_heads,  w_obs,       head_dim]   the last w_obs query vectors of the
 *                                                         scored layer, positions L-w_obs..L-1
 *   K, V    [batch, n_kv_heads, max_seq_len, head_dim]   full cache of one layer; sequence b
 *                                                         uses token rows 0 .. seq_len[b]-1
 *   K_out,
 *   V_out   [batch, n_kv_heads, nkeep_max,   head_dim]   compact cache of one layer
 * Query head hq belongs to KV head hq / (n_q_heads / n_kv_heads).
 */
typedef struct {
  int32_t batch;             /* 1 .. WKV_MAX_BATCH                                        */
  int32_t n_q_heads;         /* Hq, multiple of n_kv_heads                                */
  int32_t n_kv_heads;        /* Hkv                                                       */
  int32_t head_dim;          /* d: 64 or 128                                              */
  int32_t w_obs;             /* alpha, >= 1; (Hq/Hkv) * w_obs <= WKV_MAX_OBS_ROWS          */
  int32_t max_seq_len;       /* token capacity of the K/V tensors, >= every seq_len[b]    */
  int32_t dtype;             /* wkv_dtype of q_obs, K, V and the compact cache            */
  float   scale;             /* logit scale; 0 selects 1/sqrt(head_dim) (Eq. 1)           */
  const int32_t *seq_len;    /* host [batch]  L_b,   w_obs <= L_b <= max_seq_len          */
  const int32_t *win;        /* host [batch]  omega, 1 .. WKV_MAX_WIN                     */
  const int32_t *top_p;      /* host [batch]  p, >= 1 (p >= win means the window mean)    */
  const int32_t *k_windows;  /* host [batch]  windows to keep, 0 .. NW_b                  */
  int64_t q_stride_b, q_stride_h, q_stride_t;        /* q_obs                             */
  int64_t kv_stride_b, kv_stride_h, kv_stride_t;     /* full K and V (same for both)      */
  int64_t out_stride_b, out_stride_h, out_stride_t;  /* compact K_out and V_out           */
  int32_t flags;             /* 0, or an OR of the WKV_... flags above                    */
} wkv_problem;

/* Sizes derived from a problem; every output buffer below is sized by these. */
typedef struct {
  int32_t obs_rows;      /* (Hq/Hkv) * w_obs : softmax rows per KV head                   */
  int32_t t_stride;      /* max_seq_len - w_obs : row length of the token-score array     */
  int32_t nw_max;        /* max_b NW_b          : row length of the window-score array    */
  int32_t k_max;         /* max_b k_windows[b]  : row length of win_idx                   */
  int32_t nkeep_max;     /* max_b k_b*win_b + w_obs : row length of tok_idx, rows of K_out */
  int64_t total_tokens;  /* sum_b L_b                                                     */
} wkv_dims;

/* Validates the problem (host only, no GPU needed) and fills *dims. */
wkv_status wkv_get_dims(const wkv_problem *problem, wkv_dims *dims);

/* Bytes of device workspace the calls below need for `n_groups` groups (n_groups = 1 for
 * the per-stage calls).  Returns 0 for an invalid problem.  The workspace must be 256-byte
 * aligned; its contents on entry are irrelevant and on return unspecified. */
size_t wkv_workspace_bytes(const wkv_problem *problem, int32_t n_groups);

/*
 * Diagnostic (host only): where wkv_compress_groups leaves the intermediate results of Eq. 2
 * and Eq. 3-4 inside the caller's workspace, so that a test can compare them element by element.
 *   t_offset   byte offset of the token scores  float32 [n_groups, batch, n_kv_heads, t_stride]
 *   s_offset   byte offset of the window scores float32 [n_groups, batch, n_kv_heads, nw_max]
 *   t_written  1 if the batched call writes the token scores to memory for this problem; 0 when
 *              its score kernel pools them on chip (every window size divides 128, 16-bit
 *              inputs) and they never leave the compute unit
 *   s_written  1 if the batched call writes the window scores to memory (entries w < NW_b of
 *              each row; the rest of a row is unspecified); 0 when pooling happens inside its
 *              selection kernel
 * Exactly one of t_written / s_written is 1.  The stage calls do not use these regions.
 */
typedef struct {
  size_t t_offset, s_offset;
  int32_t t_written, s_written;
} wkv_workspace_layout;
wkv_status wkv_get_workspace_layout(const wkv_problem *problem, int32_t n_groups,
                                    wkv_workspace_layout *layout);

/*
 * Eq. 1-2: token scores of one layer group.
 *   q_obs   device, layout above
 *   k_first device, K of the group's first layer
 *   lse_obs device float32 [batch, n_q_heads, w_obs] (contiguous), or NULL.  The prefill
 *           attention that produced the cache already holds, for every query row i, the
 *           normaliser of Eq. 1 as lse_i = ln sum_{j <= pos(i)} exp(scale * q_i . k_j) (natural
 *           logarithm, causal, over the whole prefix, the same `scale` as here).  When it is
 *           passed for the w_obs observation rows, A_ij = exp(scale * q_i . k_j - lse_i) is
 *           evaluated directly and the keys are read once; with NULL the library computes the
 *           normalisers itself in a first pass over the keys.  A wrong lse_obs gives wrong
 *           scores; it is not checked.
 *   t_out   device float32 [batch, n_kv_heads, t_stride]; entries j < L_b - w_obs are written,
 *           the rest of each row is set to 0.
 * The softmax runs in fp32 on fp32-accumulated logits; no exponent is taken of an
 * unshifted logit, so any finite inputs are safe.
 */
wkv_status wkv_score(const wkv_problem *problem, const void *q_obs, const void *k_first,
                     const float *lse_obs, float *t_out, void *workspace, size_t workspace_bytes,
                     void *hip_stream);

/*
 * Eq. 3-4: window scores.
 *   t      device float32 [batch, n_kv_heads, t_stride]
 *   s_out  device float32 [batch, n_kv_heads, nw_max]; entries w < NW_b are written, the rest
 *          of each row is set to -inf.
 * A partial last window takes the min(p, size) largest of the tokens it has and keeps the
 * divisor min(p, win).
 */
wkv_status wkv_window_pool(const wkv_problem *problem, const float *t, float *s_out,
                           void *hip_stream);

/*
 * Section 2.2.1, selection: the k_windows[b] highest-scoring windows of every (b, KV head),
 * equal scores resolved towards the lower window index, reported in ascending order, and the
 * retained token positions: all tokens of the selected windows followed by L_b-w_obs .. L_b-1.
 *   s            device float32 [batch, n_kv_heads, nw_max]
 *   win_idx_out  device int32   [batch, n_kv_heads, k_max]      ascending, padded with -1
 *   tok_idx_out  device int32   [batch, n_kv_heads, nkeep_max]  ascending, padded with -1
 *   n_keep_out   device int32   [batch, n_kv_heads]             valid entries of tok_idx
 * (n_keep is k*win + w_obs, less the missing tokens of a selected partial last window.)
 */
wkv_status wkv_topk_windows(const wkv_problem *problem, const float *s, int32_t *win_idx_out,
                            int32_t *tok_idx_out, int32_t *n_keep_out, void *hip_stream);

/*
 * Section 2.2.2: every layer of a group keeps the rows at the group's shared indices.
 *   n_layers               1 .. WKV_MAX_LAYERS
 *   k_layers, v_layers     host arrays [n_layers] of device pointers to full K / V
 *   tok_idx, n_keep        device, as written by wkv_topk_windows
 *   k_out_layers,
 *   v_out_layers           host arrays [n_layers] of device pointers to compact K_out / V_out
 * Row r < n_keep[b,h] of an output is a bit-exact copy of input row tok_idx[b,h,r]; rows
 * n_keep[b,h] .. nkeep_max-1 are zero-filled (left as they were with WKV_KEEP_PADDING).
 * Inputs and outputs must not overlap.
 */
wkv_status wkv_gather_group(const wkv_problem *problem, int32_t n_layers,
                            const void *const *k_layers, const void *const *v_layers,
                            const int32_t *tok_idx, const int32_t *n_keep,
                            void *const *k_out_layers, void *const *v_out_layers,
                            void *hip_stream);

/*
 * Section 2.2 for ONE layer group of gamma layers: Eq. 1-4 and the selection (2.2.1) on the
 * group's first layer, then every layer of the group keeps the rows at the shared indices
 * (2.2.2).  The same results as wkv_score, wkv_window_pool, wkv_topk_windows and
 * wkv_gather_group called in turn; a thin wrapper over wkv_compress_groups with n_groups = 1.
 *   q_obs, lse_obs         device, as at wkv_score (lse_obs may be NULL)
 *   k_layers, v_layers,
 *   k_out_layers,
 *   v_out_layers           host arrays [gamma] of device pointers; k_layers[0] is scored
 *   win_idx_out            device int32 [batch, n_kv_heads, k_max]
 *   tok_idx_out            device int32 [batch, n_kv_heads, nkeep_max]
 *   n_keep_out             device int32 [batch, n_kv_heads]
 *   workspace              wkv_workspace_bytes(problem, 1) bytes
 */
wkv_status wkv_compress_group(const wkv_problem *problem, int32_t gamma, const void *q_obs,
                              const float *lse_obs, const void *const *k_layers,
                              const void *const *v_layers, void *const *k_out_layers,
                              void *const *v_out_layers, int32_t *win_idx_out,
                              int32_t *tok_idx_out, int32_t *n_keep_out, void *workspace,
                              size_t workspace_bytes, void *hip_stream);

/*
 * The whole path (Eq. 1-4, selection, sharing, gather) for n_groups layer groups of gamma
 * layers each, batched so that every stage is one launch over all groups.
 *   q_obs_groups   host array [n_groups] of device pointers: q_obs of each group's first layer
 *   lse_obs_groups NULL, or host array [n_groups] of device pointers: lse_obs of each group's
 *                  first layer as described at wkv_score (all groups or none)
 *   k_windows_groups  NULL, or host int32 [n_groups, batch]: windows to keep for sequence b in
 *                  group g when the groups have budgets of their own (Section 2.2.3, Eq. 5-7;
 *                  see wkv_group_budgets), 0 <= k <= problem->k_windows[b].  problem->k_windows
 *                  then only sizes the outputs (k_max, nkeep_max); rows are padded as usual.
 *                  Needs n_groups*batch <= 1024.  With NULL every group keeps k_windows[b].
 *   k_layers, v_layers, k_out_layers, v_out_layers
 *                  host arrays [n_groups*gamma] of device pointers, layer l of group g at
 *                  index g*gamma + l; group g is scored on k_layers[g*gamma] only
 *   win_idx_out    device int32 [n_groups, batch, n_kv_heads, k_max]
 *   tok_idx_out    device int32 [n_groups, batch, n_kv_heads, nkeep_max]
 *   n_keep_out     device int32 [n_groups, batch, n_kv_heads]
 * Results equal those of the four stage calls run group by group, except that the fp32
 * summation order of the softmax normalisers depends on how a launch splits the keys over
 * workgroups: token scores can differ in their last bits, hence selections only between windows
 * whose scores agree to fp32 rounding.
 * n_groups <= WKV_MAX_GROUPS, n_groups*gamma <= WKV_MAX_LAYERS.
 */
wkv_status wkv_compress_groups(const wkv_problem *problem, int32_t n_groups, int32_t gamma,
                               const void *const *q_obs_groups, const float *const *lse_obs_groups,
                               const int32_t *k_windows_groups,
                               const void *const *k_layers, const void *const *v_layers,
                               void *const *k_out_layers, void *const *v_out_layers,
                               int32_t *win_idx_out, int32_t *tok_idx_out, int32_t *n_keep_out,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Diagnostic twin of wkv_compress_groups (same arguments, same results, same launches): it
 * brackets every kernel of the path with HIP events on the caller's stream, waits for the
 * stream, and reports each kernel's duration.  It creates and destroys HIP events and blocks
 * the calling thread, so it is for benchmarks and profiling, not for serving.
 *   stage_ms_out  host float [WKV_N_STAGES]: milliseconds of, in order, the softmax-statistics
 *                 pass (Eq. 1; 0 with lse_obs_groups; with WKV_SCORE_SINGLE_READ the single-read
 *                 kernel, which then covers Eq. 1-2), the score pass (Eq. 1-2, and Eq. 3-4 where it
 *                 pools its own windows), the selection kernel (2.2.1, and Eq. 3-4 otherwise) and
 *                 the shared-index gather (2.2.2).
 */
#define WKV_N_STAGES 4
wkv_status wkv_compress_groups_profiled(const wkv_problem *problem, int32_t n_groups, int32_t gamma,
                                        const void *const *q_obs_groups,
                                        const float *const *lse_obs_groups,
                                        const int32_t *k_windows_groups,
                                        const void *const *k_layers, const void *const *v_layers,
                                        void *const *k_out_layers, void *const *v_out_layers,
                                        int32_t *win_idx_out, int32_t *tok_idx_out,
                                        int32_t *n_keep_out, void *workspace, size_t workspace_bytes,
                                        void *hip_stream, float *stage_ms_out);

/*
 * Section 2.2.3, Eq. 5-7 (host only): arithmetic-sequence budgets for n_groups groups,
 * b^{H-1} = b_total/(lambda*H), b^0 = 2*b_total/H - b^{H-1}, linear in between.
 *   budgets_out  host double [n_groups], real-valued as in the paper; turning a budget into
 *                a whole number of windows is left to the caller.
 */
wkv_status wkv_group_budgets(double b_total, int32_t n_groups, double lambda,
                             double *budgets_out);

/*
 * Section 3.2 (how alike the selections of different layers are): Jaccard similarity
 * |A n B| / |A u B| of the retained token positions of every pair of index sets, e.g. of the
 * layers of a model each selected on its own (wkv_compress_groups with gamma = 1).
 *   n_sets        1 .. WKV_MAX_GROUPS
 *   tok_idx       device int32 [n_sets, batch, n_kv_heads, nkeep_max], rows ascending
 *   n_keep        device int32 [n_sets, batch, n_kv_heads]       (both as written by the
 *                 selection calls; values outside [0, nkeep_max] are clamped)
 *   jaccard_out   device float32 [n_sets, n_sets, batch, n_kv_heads]; 1 for two empty sets
 */
wkv_status wkv_index_jaccard(const wkv_problem *problem, int32_t n_sets, const int32_t *tok_idx,
                             const int32_t *n_keep, float *jaccard_out, void *hip_stream);

/* wkv_decode_shape.flags.  The gamma layers of a group share one index set (Section 2.2.2), hence
 * one n_keep row per (sequence, KV head): a caller that keeps ONE row counter per group runs the
 * decode step of the group's first gamma-1 layers with WKV_DECODE_KEEP_COUNT (the counter is read
 * but not changed) and the last layer's without it (the counter advances once per token).  A
 * caller with a counter per layer never sets it. */
#define WKV_DECODE_KEEP_COUNT 1

/*
 * Generation over the compact cache (what the throughput test of Section 3.5 runs): one decode
 * step of one layer.  For every (sequence b, KV head h) with n = n_valid[b,h] retained rows, the
 * new token's key and value rows are appended at row n of the compact caches, and each of the
 * G = n_q_heads / n_kv_heads query heads of h attends to rows 0 .. n (the new one included):
 *     out = softmax(q . K^T * scale) . V      (Eq. 1 with one query row; nothing is masked)
 * with fp32 accumulation and an fp32 result.
 */
typedef struct {
  int32_t batch;            /* >= 1; batch * n_kv_heads <= 65535                               */
  int32_t n_q_heads;        /* multiple of n_kv_heads, at most 8 query heads per KV head       */
  int32_t n_kv_heads;
  int32_t head_dim;         /* 64 or 128                                                       */
  int32_t dtype;            /* wkv_dtype of q_new, k_new, v_new and the caches                 */
  float   scale;            /* logit scale; 0 selects 1/sqrt(head_dim)                         */
  int32_t capacity;         /* token rows per (b, h) in the caches (nkeep_max + tokens to come) */
  int64_t cache_stride_b, cache_stride_h, cache_stride_t;   /* elements; head_dim contiguous   */
  int32_t flags;            /* 0, or WKV_DECODE_KEEP_COUNT                                     */
} wkv_decode_shape;

/* Bytes of 256-byte-aligned device workspace wkv_decode_step needs; 0 for an invalid shape. */
size_t wkv_decode_workspace_bytes(const wkv_decode_shape *shape);

/*
 *   q_new          device [batch, n_q_heads, head_dim], contiguous
 *   k_new, v_new   device [batch, n_kv_heads, head_dim], contiguous
 *   k_cache,
 *   v_cache        device [batch, n_kv_heads, capacity, head_dim] by the strides above; rows
 *                  0 .. n_valid[b,h]-1 are read, row n_valid[b,h] is written
 *   n_valid        device int32 [batch, n_kv_heads]; read, then incremented by one unless
 *                  WKV_DECODE_KEEP_COUNT is set.  It counts the rows of THIS layer's caches: the
 *                  n_keep row of a group describes all gamma layers of the group, so pass either a
 *                  copy per layer, or the shared row with WKV_DECODE_KEEP_COUNT on all but the
 *                  group's last layer (otherwise the second layer would find the counter already
 *                  advanced and attend to a row its cache does not hold yet)
 *   out            device float32 [batch, n_q_heads, head_dim]
 * A (b, h) whose n_valid is negative or already equals capacity cannot take the new row: its
 * caches and n_valid are left untouched and its rows of `out` are set to NaN.
 */
wkv_status wkv_decode_step(const wkv_decode_shape *shape, const void *q_new, const void *k_new,
                           const void *v_new, void *k_cache, void *v_cache, int32_t *n_valid,
                           float *out, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * wkv_decode_step for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the
 * workspace), same kernels, same results; the partial results of the key ranges go to a scratch
 * array that is part of the library's device image (WKV_DECODE_STATIC_SCRATCH_BYTES, held by every
 * GPU the library runs on until the process ends) instead of caller memory.  The call allocates
 * and frees nothing.
 *   - A shape whose wkv_decode_workspace_bytes exceeds WKV_DECODE_STATIC_SCRATCH_BYTES is refused
 *     with WKV_ERR_WORKSPACE before anything is launched (use wkv_decode_step with a workspace).
 *   - All calls on one GPU share that GPU's scratch array: calls that may overlap in time on one
 *     GPU (different streams, different threads) race on it and must be serialised by the caller.
 *     Nothing in it needs to survive from one call to the next.
 *   - The first call on a device looks up the array's address (no stream work, no allocation);
 *     make that first call outside graph capture.
 */
#define WKV_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
wkv_status wkv_decode_step_static(const wkv_decode_shape *shape, const void *q_new, const void *k_new,
                                  const void *v_new, void *k_cache, void *v_cache, int32_t *n_valid,
                                  float *out, void *hip_stream);

const char *wkv_status_string(wkv_status status);

/* Message describing the most recent failure on the calling thread ("" if none). */
const char *wkv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* WKV_H */
