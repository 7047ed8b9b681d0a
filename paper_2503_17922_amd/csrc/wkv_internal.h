// Internal declarations shared by the translation units of libwkv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wkv.h"

namespace wkv {

inline int64_t elem_bytes(int32_t dtype) { return dtype == WKV_F32 ? 4 : 2; }

// Per-sequence parameters, passed to kernels by value inside the kernel argument block so
// that no host-to-device copy (and no allocation) is ever needed for metadata.
struct SeqParam {
  int32_t L;    // prefix length
  int32_t win;  // review-window size (omega)
  int32_t p;    // top-p, already clamped to [1, win]
  int32_t k;    // windows to keep
};
struct BatchParams {
  SeqParam seq[WKV_MAX_BATCH];
  // The sequences in ascending length: the statistics pass dispatches the rows of short sequences
  // first (in a batch of mixed lengths that shortens the launch; measured 6 % on a batch of eight
  // prefixes between 4.8K and 31K tokens).  A permutation of 0 .. batch-1; identity beyond.
  uint8_t by_length[WKV_MAX_BATCH];
};

// Windows to keep per (group, sequence) when the groups have budgets of their own (Section
// 2.2.3); index g * B + b.  Not in use: every group keeps SeqParam::k windows.
constexpr int32_t MAX_GROUP_K = 1024;
struct GroupK {
  int32_t in_use;
  uint16_t k[MAX_GROUP_K];
};

// Per-group device pointers of the scored layer.
struct GroupPtrs {
  const void *q[WKV_MAX_GROUPS];
  const void *k[WKV_MAX_GROUPS];
  const float *lse[WKV_MAX_GROUPS];   // caller's softmax log-sum-exp of the observation rows, or all null
};

// Per-layer device pointers for the gather.
struct LayerPtrs {
  const void *k_in[WKV_MAX_LAYERS];
  const void *v_in[WKV_MAX_LAYERS];
  void *k_out[WKV_MAX_LAYERS];
  void *v_out[WKV_MAX_LAYERS];
};

// Problem shape as the kernels see it.
struct Shape {
  int32_t B, Hq, Hkv, d, w_obs, G;
  int32_t M;          // G * w_obs softmax rows per KV head
  int32_t t_stride, nw_max, k_max, nkeep_max;
  int32_t dtype;
  int32_t fill_padding;   // gather: zero the compact-cache rows past n_keep
  float c1;           // logit scale * log2(e): logits are handled in base-2 units
  int64_t q_sb, q_sh, q_st;
  int64_t kv_sb, kv_sh, kv_st;
  int64_t o_sb, o_sh, o_st;
};

// How the score passes split the key axis into workgroup chunks.
// Longest key chunk of one workgroup: pass 1 keeps nothing per key; pass 2 stages the chunk's
// token scores in LDS (4 bytes per key).
constexpr int32_t MAX_CHUNK1 = 8192;
constexpr int32_t MAX_CHUNK2 = 4096;

struct ScorePlan {
  int32_t chunk1, n_chunks1;   // stats pass
  int32_t chunk2, n_chunks2;   // score pass (over t_stride)
  int32_t m_pad;               // rows padded to a multiple of 16
  bool mfma;                   // bf16 MFMA kernels (else the generic ones)
  bool fold_in_pass2;          // MFMA path: pass 2 folds the pass-1 partials itself (few chunks per row)
  bool pool_in_pass2;          // MFMA path: pass 2 can pool its chunk's windows (every window size divides 128)
};

// ---- single-read score kernel ("resident keys") ----------------------------------------------------
constexpr int32_t RK_SLICE = 256;        // keys a workgroup holds in registers between its two phases
// Synchronisation words in the workspace (uint32, cleared at the start of every call): a few
// global ones, then RK_SYNC_WORDS per (group, sequence, KV head) row.
constexpr int32_t RK_GLOBAL_WORDS = 4;
constexpr int32_t RK_FAIL = 0;           // global: a bounded wait ran out; the two-pass kernels redo the scores
constexpr int32_t RK_SYNC_WORDS = 4;
constexpr int32_t RK_ARRIVED = 0;        // per row: slices whose phase-1 partials are in the workspace
constexpr int32_t RK_READY = 1;          // per row: the normalisers of the row are published

struct ResidentPlan {
  int32_t use;                           // the call takes the single-read kernel
  int32_t n_items, items_per_group;      // slices in the call / in one group
  int32_t nsl_max;                       // most slices of any row
  int32_t m_pad;
  int32_t spin_limit;                    // polls before a waiting workgroup gives up
};

struct Workspace {
  float2 *partials;   // [n_groups][B][Hkv][m_pad][n_chunks1] (running max, sum) in base 2
  float *lse;         // [n_groups][B][Hkv][m_pad] base-2 log-sum-exp of every softmax row
  float *t;           // [n_groups][B][Hkv][t_stride]
  float *s;           // [n_groups][B][Hkv][nw_max]
  unsigned long long *rk_partials;   // [rows][nsl_max][m_pad] (m, z) of every slice (single-read kernel)
  uint32_t *rk_sync;                 // [RK_GLOBAL_WORDS + rows * RK_SYNC_WORDS]
  size_t t_offset, s_offset;   // byte offsets of t and s from the base
  size_t bytes;
};

// ---- host-side helpers (wkv_host.cpp) ---------------------------------------------------
void set_error(const char *fmt, ...);
wkv_status validate(const wkv_problem *p, wkv_dims *dims);
void fill_shape(const wkv_problem *p, const wkv_dims &dims, Shape *s, BatchParams *bp);
ScorePlan plan_score(const Shape &s, const BatchParams &bp, int32_t n_groups);
ResidentPlan plan_resident(const Shape &s, const BatchParams &bp, const ScorePlan &plan, int32_t n_groups, int32_t flags);
Workspace carve_workspace(const Shape &s, const ScorePlan &plan, const ResidentPlan &rp, int32_t n_groups, void *base);

// ---- launchers (one per kernel family) ----------------------------------------------------
// All return hipSuccess or the launch error. Pointers are device pointers unless noted.
// `mid`, if not null, is recorded between the stats pass and the score pass.
// `only_if`, if not null, points to a device word: the kernels return at once unless it is non-zero.
hipError_t launch_score(const Shape &s, const BatchParams &bp, const ScorePlan &plan,
                        const GroupPtrs &gp, int32_t n_groups, bool have_lse, float2 *partials, float *lse,
                        float *t_out, float *s_pool, hipStream_t stream, hipEvent_t mid = nullptr,
                        const uint32_t *only_if = nullptr);
// Clears the synchronisation words, then the single-read score kernel (Eq. 1-2, pooled if s_pool).
hipError_t launch_resident(const Shape &s, const BatchParams &bp, const ResidentPlan &rp, const GroupPtrs &gp,
                           int32_t n_groups, unsigned long long *partials, float *lse, uint32_t *sync, float *t_out,
                           float *s_pool, hipStream_t stream);
hipError_t launch_pool(const Shape &s, const BatchParams &bp, int32_t n_groups, const float *t,
                       float *s_out, hipStream_t stream);
hipError_t launch_topk(const Shape &s, const BatchParams &bp, const GroupK &gk, int32_t n_groups, const float *sc,
                       int32_t *win_idx, int32_t *tok_idx, int32_t *n_keep, hipStream_t stream);
// Pooling and selection in one launch (same results as launch_pool followed by launch_topk).
hipError_t launch_select(const Shape &s, const BatchParams &bp, const GroupK &gk, int32_t n_groups, const float *t,
                         int32_t *win_idx, int32_t *tok_idx, int32_t *n_keep, hipStream_t stream);
hipError_t launch_gather(const Shape &s, const LayerPtrs &lp, int32_t n_layers, int32_t gamma,
                         const int32_t *tok_idx, const int32_t *n_keep, hipStream_t stream);

hipError_t launch_jaccard(const Shape &s, int32_t n_sets, const int32_t *tok_idx, const int32_t *n_keep, float *out,
                          hipStream_t stream);

// ---- decode over the compact cache --------------------------------------------------------
struct DecodeShape {
  int32_t B, Hq, Hkv, d, G, dtype;
  int32_t capacity;          // token rows per (sequence, KV head) in the caches
  int32_t n_splits, chunk;   // key ranges per (sequence, KV head) and their length
  int32_t keep_count;        // leave n_valid as it is (the caller advances it after the group's last layer)
  float c1;                  // scale * log2(e)
  int64_t sb, sh, st;        // cache strides in elements
};
struct Decode {
  DecodeShape shape;
  size_t ws_bytes;           // partial results: [B*Hkv][n_splits][G][d + 2] floats
};
wkv_status validate_decode(const wkv_decode_shape *p, Decode *out);
hipError_t launch_decode(const DecodeShape &s, const void *q_new, const void *k_new, const void *v_new, void *k_cache,
                         void *v_cache, int32_t *n_valid, float *out, float *part, hipStream_t stream);

// The same launches with the partial results in the library's own static scratch array of the
// current device (no workspace argument; the caller has checked that the shape fits).
hipError_t launch_decode_static(const DecodeShape &s, const void *q_new, const void *k_new, const void *v_new,
                                void *k_cache, void *v_cache, int32_t *n_valid, float *out, hipStream_t stream);

}  // namespace wkv
