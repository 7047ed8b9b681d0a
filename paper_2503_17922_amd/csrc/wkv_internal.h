// Internal declarations shared by the translation units of libwkv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wkv.h"

namespace wkv {

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
};

// Per-group device pointers of the scored layer.
struct GroupPtrs {
  const void *q[WKV_MAX_GROUPS];
  const void *k[WKV_MAX_GROUPS];
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
  float c1;           // logit scale * log2(e): logits are handled in base-2 units
  int64_t q_sb, q_sh, q_st;
  int64_t kv_sb, kv_sh, kv_st;
  int64_t o_sb, o_sh, o_st;
};

// How the score passes split the key axis into workgroup chunks.
struct ScorePlan {
  int32_t chunk1, n_chunks1;   // stats pass
  int32_t chunk2, n_chunks2;   // score pass (over t_stride)
  int32_t m_pad;               // rows padded to a multiple of 16
  bool mfma;                   // bf16 MFMA kernels (else the generic ones)
};

// Single-pass score kernel: key chunk of one workgroup, and the layout of the sync block through
// which the workgroups of one (group, sequence, KV head) exchange row maxima and row sums.
constexpr int FUSED_CHUNK = 256;
constexpr int SYNC_HEADER_WORDS = 64;     // 32-bit words; [SYNC_TICKET] work counter, [SYNC_ERROR] spin ran out
constexpr int SYNC_TICKET = 0, SYNC_ERROR = 16;
constexpr int SYNC_PROBLEM_WORDS = 512;   // per (group, sequence, KV head)
constexpr int SYNC_ROWMAX = 0;            // 128 x u32  order-preserving keys of the raw row maxima
constexpr int SYNC_ZFIX = 128;            // 128 x u64  row sums in units of 2^-40
constexpr int SYNC_CNT1 = 384, SYNC_CNT2 = 400;   // arrival counters (own cache lines)

struct FusedPlan {
  int32_t eligible;                       // shape allows the single-pass kernel
  int32_t tickets_per_group;              // Hkv * sum_b nch[b]
  int32_t total_tickets;
  int32_t nch[WKV_MAX_BATCH];             // key chunks of sequence b
  int32_t first[WKV_MAX_BATCH + 1];       // first ticket (within a group) of sequence b
};

struct Workspace {
  float2 *partials;   // [n_groups][B][Hkv][m_pad][n_chunks1] (running max, sum) in base 2
  float *t;           // [n_groups][B][Hkv][t_stride]
  float *s;           // [n_groups][B][Hkv][nw_max]
  uint32_t *sync;     // sync block of the single-pass score kernel
  size_t sync_words;
  size_t bytes;
};

// ---- host-side helpers (wkv_host.cpp) ---------------------------------------------------
void set_error(const char *fmt, ...);
wkv_status validate(const wkv_problem *p, wkv_dims *dims);
void fill_shape(const wkv_problem *p, const wkv_dims &dims, Shape *s, BatchParams *bp);
ScorePlan plan_score(const Shape &s, int32_t n_groups);
FusedPlan plan_fused(const Shape &s, const BatchParams &bp, const ScorePlan &pl, int32_t n_groups);
int score_path_override();   // 0 = automatic, 1 = two passes, 2 = single pass where possible
Workspace carve_workspace(const Shape &s, const ScorePlan &plan, int32_t n_groups, void *base);

// ---- launchers (one per kernel family) ----------------------------------------------------
// All return hipSuccess or the launch error. Pointers are device pointers unless noted.
// `mid`, if not null, is recorded between the stats pass and the score pass.
hipError_t launch_score(const Shape &s, const BatchParams &bp, const ScorePlan &plan,
                        const GroupPtrs &gp, int32_t n_groups, float2 *partials, float *t_out,
                        hipStream_t stream, hipEvent_t mid = nullptr);
// Single-pass variant.  *used is false (and nothing was launched) when the device cannot keep a
// problem's workgroups resident together; the caller then runs launch_score instead.
hipError_t launch_score_fused(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const FusedPlan &fp,
                              const GroupPtrs &gp, uint32_t *sync, size_t sync_words, float *t_out,
                              hipStream_t stream, hipEvent_t mid, bool *used);
hipError_t launch_pool(const Shape &s, const BatchParams &bp, int32_t n_groups, const float *t,
                       float *s_out, hipStream_t stream);
hipError_t launch_topk(const Shape &s, const BatchParams &bp, int32_t n_groups, const float *sc,
                       int32_t *win_idx, int32_t *tok_idx, int32_t *n_keep, hipStream_t stream);
hipError_t launch_gather(const Shape &s, const LayerPtrs &lp, int32_t n_layers, int32_t gamma,
                         const int32_t *tok_idx, const int32_t *n_keep, hipStream_t stream);

}  // namespace wkv
