// The exported entry points: validate on the host, then enqueue the kernels on the caller's
// stream.  No allocation, no synchronisation, no state.
#include <cstring>

#include "wkv_internal.h"

using namespace wkv;

namespace {

inline bool misaligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

wkv_status hip_fail(hipError_t e, const char *what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return WKV_ERR_HIP;
}

struct Prepared {
  wkv_dims dims;
  Shape shape;
  BatchParams bp;
};

wkv_status prepare(const wkv_problem *problem, Prepared *out) {
  wkv_status st = validate(problem, &out->dims);
  if (st != WKV_OK) return st;
  fill_shape(problem, out->dims, &out->shape, &out->bp);
  return WKV_OK;
}

wkv_status check_workspace(const Shape &s, const ScorePlan &pl, const ResidentPlan &rp, int32_t n_groups, void *ws,
                           size_t bytes, Workspace *out) {
  if (!ws) { set_error("workspace is NULL"); return WKV_ERR_WORKSPACE; }
  if (misaligned(ws, 256)) { set_error("workspace must be 256-byte aligned"); return WKV_ERR_WORKSPACE; }
  *out = carve_workspace(s, pl, rp, n_groups, ws);
  if (bytes < out->bytes) {
    set_error("workspace has %zu bytes, %zu needed", bytes, out->bytes);
    return WKV_ERR_WORKSPACE;
  }
  return WKV_OK;
}

}  // namespace

extern "C" {

wkv_status wkv_score(const wkv_problem *problem, const void *q_obs, const void *k_first, const float *lse_obs,
                     float *t_out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Prepared pr;
  wkv_status st = prepare(problem, &pr);
  if (st != WKV_OK) return st;
  if (!q_obs || !k_first || !t_out) { set_error("q_obs / k_first / t_out is NULL"); return WKV_ERR_INVALID_ARG; }
  if (misaligned(q_obs, 16) || misaligned(k_first, 16)) { set_error("q_obs and k_first must be 16-byte aligned"); return WKV_ERR_INVALID_ARG; }
  if (misaligned(lse_obs, 4)) { set_error("lse_obs must be 4-byte aligned"); return WKV_ERR_INVALID_ARG; }
  const ScorePlan pl = plan_score(pr.shape, pr.bp, 1);
  const ResidentPlan rp = plan_resident(pr.shape, pr.bp, pl, 1, problem->flags);
  Workspace ws;
  st = check_workspace(pr.shape, pl, rp, 1, workspace, workspace_bytes, &ws);
  if (st != WKV_OK) return st;
  GroupPtrs gp;
  std::memset(&gp, 0, sizeof(gp));
  gp.q[0] = q_obs; gp.k[0] = k_first; gp.lse[0] = lse_obs;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipError_t e = hipSuccess;
  const uint32_t *only_if = nullptr;
  if (rp.use && !lse_obs) {
    // one read of the keys; the two-pass kernels behind it run only if a wait of it gave up
    e = launch_resident(pr.shape, pr.bp, rp, gp, 1, ws.rk_partials, ws.lse, ws.rk_sync, t_out, nullptr, stream);
    if (e != hipSuccess) return hip_fail(e, "wkv_score launch (single read)");
    only_if = ws.rk_sync + RK_FAIL;
  }
  e = launch_score(pr.shape, pr.bp, pl, gp, 1, lse_obs != nullptr, ws.partials, ws.lse, t_out, nullptr, stream, nullptr, only_if);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_score launch");
}

wkv_status wkv_window_pool(const wkv_problem *problem, const float *t, float *s_out, void *hip_stream) {
  Prepared pr;
  wkv_status st = prepare(problem, &pr);
  if (st != WKV_OK) return st;
  if (!t || !s_out) { set_error("t / s_out is NULL"); return WKV_ERR_INVALID_ARG; }
  hipError_t e = launch_pool(pr.shape, pr.bp, 1, t, s_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_window_pool launch");
}

wkv_status wkv_topk_windows(const wkv_problem *problem, const float *s, int32_t *win_idx_out,
                            int32_t *tok_idx_out, int32_t *n_keep_out, void *hip_stream) {
  Prepared pr;
  wkv_status st = prepare(problem, &pr);
  if (st != WKV_OK) return st;
  if (!s || !win_idx_out || !tok_idx_out || !n_keep_out) {
    set_error("s / win_idx_out / tok_idx_out / n_keep_out is NULL"); return WKV_ERR_INVALID_ARG;
  }
  GroupK gk;
  std::memset(&gk, 0, sizeof(gk));
  hipError_t e = launch_topk(pr.shape, pr.bp, gk, 1, s, win_idx_out, tok_idx_out, n_keep_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_topk_windows launch");
}

static wkv_status fill_layers(int32_t n_layers, const void *const *k_layers, const void *const *v_layers,
                              void *const *k_out_layers, void *const *v_out_layers, LayerPtrs *lp) {
  if (!k_layers || !v_layers || !k_out_layers || !v_out_layers) {
    set_error("layer pointer arrays must be non-NULL"); return WKV_ERR_INVALID_ARG;
  }
  std::memset(lp, 0, sizeof(*lp));
  for (int32_t l = 0; l < n_layers; ++l) {
    if (!k_layers[l] || !v_layers[l] || !k_out_layers[l] || !v_out_layers[l]) {
      set_error("layer %d has a NULL tensor pointer", l); return WKV_ERR_INVALID_ARG;
    }
    if (misaligned(k_layers[l], 16) || misaligned(v_layers[l], 16) || misaligned(k_out_layers[l], 16) ||
        misaligned(v_out_layers[l], 16)) {
      set_error("layer %d: tensors must be 16-byte aligned", l); return WKV_ERR_INVALID_ARG;
    }
    lp->k_in[l] = k_layers[l]; lp->v_in[l] = v_layers[l];
    lp->k_out[l] = k_out_layers[l]; lp->v_out[l] = v_out_layers[l];
  }
  return WKV_OK;
}

wkv_status wkv_gather_group(const wkv_problem *problem, int32_t n_layers, const void *const *k_layers,
                            const void *const *v_layers, const int32_t *tok_idx, const int32_t *n_keep,
                            void *const *k_out_layers, void *const *v_out_layers, void *hip_stream) {
  Prepared pr;
  wkv_status st = prepare(problem, &pr);
  if (st != WKV_OK) return st;
  if (n_layers < 1 || n_layers > WKV_MAX_LAYERS) { set_error("n_layers outside [1, %d]", WKV_MAX_LAYERS); return WKV_ERR_INVALID_ARG; }
  if (!tok_idx || !n_keep) { set_error("tok_idx / n_keep is NULL"); return WKV_ERR_INVALID_ARG; }
  LayerPtrs lp;
  st = fill_layers(n_layers, k_layers, v_layers, k_out_layers, v_out_layers, &lp);
  if (st != WKV_OK) return st;
  // one group: every layer reads the same index rows (gamma = n_layers)
  hipError_t e = launch_gather(pr.shape, lp, n_layers, n_layers, tok_idx, n_keep, (hipStream_t)hip_stream);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_gather_group launch");
}

static wkv_status compress_impl(const wkv_problem *problem, int32_t n_groups, int32_t gamma,
                                const void *const *q_obs_groups, const float *const *lse_obs_groups,
                                const int32_t *k_windows_groups, const void *const *k_layers,
                                const void *const *v_layers, void *const *k_out_layers,
                                void *const *v_out_layers, int32_t *win_idx_out, int32_t *tok_idx_out,
                                int32_t *n_keep_out, void *workspace, size_t workspace_bytes, void *hip_stream,
                                hipEvent_t *ev /* null or [WKV_N_STAGES + 1] */) {
  Prepared pr;
  wkv_status st = prepare(problem, &pr);
  if (st != WKV_OK) return st;
  if (n_groups < 1 || n_groups > WKV_MAX_GROUPS) { set_error("n_groups outside [1, %d]", WKV_MAX_GROUPS); return WKV_ERR_INVALID_ARG; }
  if (gamma < 1 || (int64_t)n_groups * gamma > WKV_MAX_LAYERS) {
    set_error("need gamma >= 1 and n_groups*gamma <= %d", WKV_MAX_LAYERS); return WKV_ERR_INVALID_ARG;
  }
  if (!q_obs_groups || !win_idx_out || !tok_idx_out || !n_keep_out) {
    set_error("q_obs_groups / win_idx_out / tok_idx_out / n_keep_out is NULL"); return WKV_ERR_INVALID_ARG;
  }
  const int32_t n_layers = n_groups * gamma;
  LayerPtrs lp;
  st = fill_layers(n_layers, k_layers, v_layers, k_out_layers, v_out_layers, &lp);
  if (st != WKV_OK) return st;
  GroupPtrs gp;
  std::memset(&gp, 0, sizeof(gp));
  for (int32_t g = 0; g < n_groups; ++g) {
    if (!q_obs_groups[g] || misaligned(q_obs_groups[g], 16)) {
      set_error("q_obs_groups[%d] is NULL or not 16-byte aligned", g); return WKV_ERR_INVALID_ARG;
    }
    gp.q[g] = q_obs_groups[g];
    gp.k[g] = k_layers[(size_t)g * gamma];     // Section 2.2.2: the group's first layer is scored
    if (lse_obs_groups) {
      if (!lse_obs_groups[g] || misaligned(lse_obs_groups[g], 4)) {
        set_error("lse_obs_groups[%d] is NULL or not 4-byte aligned (pass a NULL array to have the statistics computed)", g);
        return WKV_ERR_INVALID_ARG;
      }
      gp.lse[g] = lse_obs_groups[g];
    }
  }
  GroupK gk;
  std::memset(&gk, 0, sizeof(gk));
  if (k_windows_groups) {
    // Section 2.2.3: groups with budgets of their own; problem->k_windows is then the capacity
    if ((int64_t)n_groups * problem->batch > MAX_GROUP_K) {
      set_error("per-group budgets support n_groups*batch <= %d", MAX_GROUP_K); return WKV_ERR_UNSUPPORTED;
    }
    gk.in_use = 1;
    for (int32_t g = 0; g < n_groups; ++g)
      for (int32_t b = 0; b < problem->batch; ++b) {
        const int32_t kgb = k_windows_groups[(size_t)g * problem->batch + b];
        if (kgb < 0 || kgb > problem->k_windows[b]) {
          set_error("k_windows_groups[%d][%d] = %d outside [0, k_windows[%d] = %d]", g, b, kgb, b, problem->k_windows[b]);
          return WKV_ERR_INVALID_ARG;
        }
        gk.k[(size_t)g * problem->batch + b] = (uint16_t)kgb;
      }
  }
  const ScorePlan pl = plan_score(pr.shape, pr.bp, n_groups);
  const ResidentPlan rp = plan_resident(pr.shape, pr.bp, pl, n_groups, problem->flags);
  Workspace ws;
  st = check_workspace(pr.shape, pl, rp, n_groups, workspace, workspace_bytes, &ws);
  if (st != WKV_OK) return st;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipError_t e;
#define WKV_MARK(i) if (ev && (e = hipEventRecord(ev[i], stream)) != hipSuccess) return hip_fail(e, "event record");
  WKV_MARK(0)
  // With window sizes that divide the chunk length the score kernel pools its own windows
  // (Eq. 3-4 on the scores still in LDS) and only the window scores reach memory.
  float *s_pool = pl.pool_in_pass2 ? ws.s : nullptr;
  const uint32_t *only_if = nullptr;
  if (rp.use && !lse_obs_groups) {
    // one read of the keys; the two-pass kernels behind it run only if a wait of it gave up
    e = launch_resident(pr.shape, pr.bp, rp, gp, n_groups, ws.rk_partials, ws.lse, ws.rk_sync, ws.t, s_pool, stream);
    if (e != hipSuccess) return hip_fail(e, "score launch (single read)");
    only_if = ws.rk_sync + RK_FAIL;
  }
  e = launch_score(pr.shape, pr.bp, pl, gp, n_groups, lse_obs_groups != nullptr, ws.partials, ws.lse, ws.t, s_pool,
                   stream, ev ? ev[1] : nullptr, only_if);
  if (e != hipSuccess) return hip_fail(e, "score launch");
  WKV_MARK(2)
  if (s_pool) e = launch_topk(pr.shape, pr.bp, gk, n_groups, ws.s, win_idx_out, tok_idx_out, n_keep_out, stream);
  else e = launch_select(pr.shape, pr.bp, gk, n_groups, ws.t, win_idx_out, tok_idx_out, n_keep_out, stream);
  if (e != hipSuccess) return hip_fail(e, "select launch");
  WKV_MARK(3)
  e = launch_gather(pr.shape, lp, n_layers, gamma, tok_idx_out, n_keep_out, stream);
  if (e != hipSuccess) return hip_fail(e, "gather launch");
  WKV_MARK(4)
#undef WKV_MARK
  return WKV_OK;
}

wkv_status wkv_compress_groups(const wkv_problem *problem, int32_t n_groups, int32_t gamma,
                               const void *const *q_obs_groups, const float *const *lse_obs_groups,
                               const int32_t *k_windows_groups, const void *const *k_layers,
                               const void *const *v_layers, void *const *k_out_layers,
                               void *const *v_out_layers, int32_t *win_idx_out, int32_t *tok_idx_out,
                               int32_t *n_keep_out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  return compress_impl(problem, n_groups, gamma, q_obs_groups, lse_obs_groups, k_windows_groups, k_layers, v_layers, k_out_layers,
                       v_out_layers, win_idx_out, tok_idx_out, n_keep_out, workspace, workspace_bytes, hip_stream,
                       nullptr);
}

wkv_status wkv_compress_group(const wkv_problem *problem, int32_t gamma, const void *q_obs, const float *lse_obs,
                              const void *const *k_layers, const void *const *v_layers, void *const *k_out_layers,
                              void *const *v_out_layers, int32_t *win_idx_out, int32_t *tok_idx_out,
                              int32_t *n_keep_out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  const void *q_groups[1] = {q_obs};
  const float *lse_groups[1] = {lse_obs};
  return compress_impl(problem, 1, gamma, q_groups, lse_obs ? lse_groups : nullptr, nullptr, k_layers, v_layers,
                       k_out_layers, v_out_layers, win_idx_out, tok_idx_out, n_keep_out, workspace, workspace_bytes,
                       hip_stream, nullptr);
}

wkv_status wkv_compress_groups_profiled(const wkv_problem *problem, int32_t n_groups, int32_t gamma,
                                        const void *const *q_obs_groups, const float *const *lse_obs_groups,
                                        const int32_t *k_windows_groups, const void *const *k_layers,
                                        const void *const *v_layers, void *const *k_out_layers,
                                        void *const *v_out_layers, int32_t *win_idx_out, int32_t *tok_idx_out,
                                        int32_t *n_keep_out, void *workspace, size_t workspace_bytes,
                                        void *hip_stream, float *stage_ms_out) {
  if (!stage_ms_out) { set_error("stage_ms_out is NULL"); return WKV_ERR_INVALID_ARG; }
  hipEvent_t ev[WKV_N_STAGES + 1];
  int made = 0;
  hipError_t e = hipSuccess;
  for (; made < WKV_N_STAGES + 1; ++made)
    if ((e = hipEventCreate(&ev[made])) != hipSuccess) break;
  wkv_status st = WKV_OK;
  if (e != hipSuccess) {
    st = hip_fail(e, "hipEventCreate");
  } else {
    st = compress_impl(problem, n_groups, gamma, q_obs_groups, lse_obs_groups, k_windows_groups, k_layers, v_layers, k_out_layers,
                       v_out_layers, win_idx_out, tok_idx_out, n_keep_out, workspace, workspace_bytes, hip_stream, ev);
    if (st == WKV_OK) {
      if ((e = hipEventSynchronize(ev[WKV_N_STAGES])) != hipSuccess) st = hip_fail(e, "hipEventSynchronize");
      for (int i = 0; st == WKV_OK && i < WKV_N_STAGES; ++i)
        if ((e = hipEventElapsedTime(&stage_ms_out[i], ev[i], ev[i + 1])) != hipSuccess) {
          // an event that was never recorded (a stage with nothing to launch) reads as 0
          stage_ms_out[i] = 0.0f;
          (void)hipGetLastError();
        }
    }
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return st;
}

wkv_status wkv_index_jaccard(const wkv_problem *problem, int32_t n_sets, const int32_t *tok_idx, const int32_t *n_keep,
                             float *jaccard_out, void *hip_stream) {
  Prepared pr;
  wkv_status st = prepare(problem, &pr);
  if (st != WKV_OK) return st;
  if (n_sets < 1 || n_sets > WKV_MAX_GROUPS) { set_error("n_sets outside [1, %d]", WKV_MAX_GROUPS); return WKV_ERR_INVALID_ARG; }
  if (!tok_idx || !n_keep || !jaccard_out) { set_error("tok_idx / n_keep / jaccard_out is NULL"); return WKV_ERR_INVALID_ARG; }
  hipError_t e = launch_jaccard(pr.shape, n_sets, tok_idx, n_keep, jaccard_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_index_jaccard launch");
}

wkv_status wkv_decode_step(const wkv_decode_shape *shape, const void *q_new, const void *k_new, const void *v_new,
                           void *k_cache, void *v_cache, int32_t *n_valid, float *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream) {
  Decode dc;
  wkv_status st = validate_decode(shape, &dc);
  if (st != WKV_OK) return st;
  if (!q_new || !k_new || !v_new || !k_cache || !v_cache || !n_valid || !out) {
    set_error("q_new / k_new / v_new / k_cache / v_cache / n_valid / out is NULL"); return WKV_ERR_INVALID_ARG;
  }
  if (misaligned(q_new, 16) || misaligned(k_new, 16) || misaligned(v_new, 16) || misaligned(k_cache, 16) ||
      misaligned(v_cache, 16)) {
    set_error("q_new, k_new, v_new and the caches must be 16-byte aligned"); return WKV_ERR_INVALID_ARG;
  }
  if (!workspace) { set_error("workspace is NULL"); return WKV_ERR_WORKSPACE; }
  if (misaligned(workspace, 256)) { set_error("workspace must be 256-byte aligned"); return WKV_ERR_WORKSPACE; }
  if (workspace_bytes < dc.ws_bytes) {
    set_error("workspace has %zu bytes, %zu needed", workspace_bytes, dc.ws_bytes); return WKV_ERR_WORKSPACE;
  }
  hipError_t e = launch_decode(dc.shape, q_new, k_new, v_new, k_cache, v_cache, n_valid, out, (float *)workspace,
                               (hipStream_t)hip_stream);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_decode_step launch");
}

wkv_status wkv_decode_step_static(const wkv_decode_shape *shape, const void *q_new, const void *k_new,
                                  const void *v_new, void *k_cache, void *v_cache, int32_t *n_valid, float *out,
                                  void *hip_stream) {
  Decode dc;
  wkv_status st = validate_decode(shape, &dc);
  if (st != WKV_OK) return st;
  if (!q_new || !k_new || !v_new || !k_cache || !v_cache || !n_valid || !out) {
    set_error("q_new / k_new / v_new / k_cache / v_cache / n_valid / out is NULL"); return WKV_ERR_INVALID_ARG;
  }
  if (misaligned(q_new, 16) || misaligned(k_new, 16) || misaligned(v_new, 16) || misaligned(k_cache, 16) ||
      misaligned(v_cache, 16)) {
    set_error("q_new, k_new, v_new and the caches must be 16-byte aligned"); return WKV_ERR_INVALID_ARG;
  }
  if (dc.ws_bytes > WKV_DECODE_STATIC_SCRATCH_BYTES) {
    set_error("this shape needs %zu bytes of scratch, the static array holds %u: use wkv_decode_step with a workspace",
              dc.ws_bytes, (unsigned)WKV_DECODE_STATIC_SCRATCH_BYTES);
    return WKV_ERR_WORKSPACE;
  }
  hipError_t e = launch_decode_static(dc.shape, q_new, k_new, v_new, k_cache, v_cache, n_valid, out, (hipStream_t)hip_stream);
  return e == hipSuccess ? WKV_OK : hip_fail(e, "wkv_decode_step_static launch");
}

}  // extern "C"
