// Host-side logic of libwkv: argument validation, derived sizes, launch planning and the
// scalar helpers.  Nothing in this file touches the GPU, so all of it is testable on a
// machine without one.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "wkv_internal.h"

namespace wkv {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

wkv_status validate(const wkv_problem *p, wkv_dims *dims) {
  g_err[0] = 0;
  if (!p) { set_error("problem is NULL"); return WKV_ERR_INVALID_ARG; }
  if (!p->seq_len || !p->win || !p->top_p || !p->k_windows) {
    set_error("seq_len / win / top_p / k_windows must be non-NULL host arrays");
    return WKV_ERR_INVALID_ARG;
  }
  if (p->batch < 1) { set_error("batch must be >= 1 (got %d)", p->batch); return WKV_ERR_INVALID_ARG; }
  if (p->batch > WKV_MAX_BATCH) {
    set_error("batch %d exceeds WKV_MAX_BATCH=%d; split the call", p->batch, WKV_MAX_BATCH);
    return WKV_ERR_UNSUPPORTED;
  }
  if (p->n_kv_heads < 1 || p->n_q_heads < 1 || p->n_q_heads % p->n_kv_heads != 0) {
    set_error("n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", p->n_q_heads, p->n_kv_heads);
    return WKV_ERR_INVALID_ARG;
  }
  if ((int64_t)p->batch * p->n_kv_heads > 65535) {
    set_error("batch * n_kv_heads exceeds 65535 (launch grid limit); split the call"); return WKV_ERR_UNSUPPORTED;
  }
  if (p->dtype != WKV_F32 && p->dtype != WKV_BF16 && p->dtype != WKV_F16) {
    set_error("unknown dtype %d", p->dtype); return WKV_ERR_INVALID_ARG;
  }
  if (p->head_dim != 64 && p->head_dim != 128) {
    set_error("head_dim %d is not supported (64 or 128)", p->head_dim); return WKV_ERR_UNSUPPORTED;
  }
  if (p->flags & ~(WKV_KEEP_PADDING | WKV_SCORE_TWO_PASS | WKV_SCORE_SINGLE_READ | WKV_DEBUG_WAIT_GIVES_UP)) {
    set_error("unknown bits in flags (0x%x)", p->flags); return WKV_ERR_INVALID_ARG;
  }
  if ((p->flags & WKV_SCORE_TWO_PASS) && (p->flags & WKV_SCORE_SINGLE_READ)) {
    set_error("WKV_SCORE_TWO_PASS and WKV_SCORE_SINGLE_READ exclude each other"); return WKV_ERR_INVALID_ARG;
  }
  if (p->w_obs < 1) { set_error("w_obs must be >= 1"); return WKV_ERR_INVALID_ARG; }
  const int64_t G = p->n_q_heads / p->n_kv_heads;
  if (G * p->w_obs > WKV_MAX_OBS_ROWS) {
    set_error("(Hq/Hkv)*w_obs = %lld exceeds WKV_MAX_OBS_ROWS=%d", (long long)(G * p->w_obs), WKV_MAX_OBS_ROWS);
    return WKV_ERR_UNSUPPORTED;
  }
  if (p->max_seq_len < p->w_obs) { set_error("max_seq_len < w_obs"); return WKV_ERR_INVALID_ARG; }
  if (!(p->scale >= 0.0f) || std::isinf(p->scale)) {
    set_error("scale must be finite and >= 0 (0 selects 1/sqrt(head_dim))"); return WKV_ERR_INVALID_ARG;
  }
  const int64_t d = p->head_dim;
  if (p->q_stride_t < d || p->kv_stride_t < d || p->out_stride_t < d) {
    set_error("token strides must be >= head_dim"); return WKV_ERR_INVALID_ARG;
  }
  // 16-byte vector loads: every row start must be 16-byte aligned relative to the base.
  const int64_t vec = 16 / elem_bytes(p->dtype);
  const int64_t strides[9] = {p->q_stride_b, p->q_stride_h, p->q_stride_t, p->kv_stride_b, p->kv_stride_h,
                              p->kv_stride_t, p->out_stride_b, p->out_stride_h, p->out_stride_t};
  for (int i = 0; i < 9; ++i) {
    if (strides[i] < 0 || strides[i] % vec != 0) {
      set_error("strides must be non-negative multiples of %lld elements (16 bytes)", (long long)vec);
      return WKV_ERR_INVALID_ARG;
    }
  }
  if (p->kv_stride_h < d || p->q_stride_h < d || p->out_stride_h < d) {
    set_error("head strides must be >= head_dim"); return WKV_ERR_INVALID_ARG;
  }

  wkv_dims dm;
  std::memset(&dm, 0, sizeof(dm));
  dm.obs_rows = (int32_t)(G * p->w_obs);
  dm.t_stride = p->max_seq_len - p->w_obs;
  for (int b = 0; b < p->batch; ++b) {
    const int64_t L = p->seq_len[b], w = p->win[b], tp = p->top_p[b], k = p->k_windows[b];
    if (L < p->w_obs || L > p->max_seq_len) {
      set_error("seq_len[%d]=%lld outside [w_obs=%d, max_seq_len=%d]", b, (long long)L, p->w_obs, p->max_seq_len);
      return WKV_ERR_INVALID_ARG;
    }
    if (w < 1) { set_error("win[%d] must be >= 1", b); return WKV_ERR_INVALID_ARG; }
    if (w > WKV_MAX_WIN) { set_error("win[%d]=%lld exceeds WKV_MAX_WIN=%d", b, (long long)w, WKV_MAX_WIN); return WKV_ERR_UNSUPPORTED; }
    if (tp < 1) { set_error("top_p[%d] must be >= 1", b); return WKV_ERR_INVALID_ARG; }
    const int64_t nw = ceil_div(L - p->w_obs, w);
    if (nw > WKV_MAX_WINDOWS) { set_error("sequence %d has %lld windows (> WKV_MAX_WINDOWS=%d)", b, (long long)nw, WKV_MAX_WINDOWS); return WKV_ERR_UNSUPPORTED; }
    if (k < 0 || k > nw) { set_error("k_windows[%d]=%lld outside [0, NW=%lld]", b, (long long)k, (long long)nw); return WKV_ERR_INVALID_ARG; }
    if (nw > dm.nw_max) dm.nw_max = (int32_t)nw;
    if (k > dm.k_max) dm.k_max = (int32_t)k;
    if (k * w + p->w_obs > dm.nkeep_max) dm.nkeep_max = (int32_t)(k * w + p->w_obs);
    dm.total_tokens += L;
  }
  if (dims) *dims = dm;
  return WKV_OK;
}

void fill_shape(const wkv_problem *p, const wkv_dims &dims, Shape *s, BatchParams *bp) {
  s->B = p->batch; s->Hq = p->n_q_heads; s->Hkv = p->n_kv_heads; s->d = p->head_dim;
  s->w_obs = p->w_obs; s->G = p->n_q_heads / p->n_kv_heads; s->M = dims.obs_rows;
  s->t_stride = dims.t_stride; s->nw_max = dims.nw_max; s->k_max = dims.k_max;
  s->nkeep_max = dims.nkeep_max; s->dtype = p->dtype;
  s->fill_padding = (p->flags & WKV_KEEP_PADDING) ? 0 : 1;
  const double scale = p->scale > 0.0f ? (double)p->scale : 1.0 / std::sqrt((double)p->head_dim);
  s->c1 = (float)(scale * 1.4426950408889634074);
  s->q_sb = p->q_stride_b; s->q_sh = p->q_stride_h; s->q_st = p->q_stride_t;
  s->kv_sb = p->kv_stride_b; s->kv_sh = p->kv_stride_h; s->kv_st = p->kv_stride_t;
  s->o_sb = p->out_stride_b; s->o_sh = p->out_stride_h; s->o_st = p->out_stride_t;
  std::memset(bp, 0, sizeof(*bp));
  for (int b = 0; b < p->batch; ++b) {
    bp->seq[b].L = p->seq_len[b];
    bp->seq[b].win = p->win[b];
    bp->seq[b].p = p->top_p[b] < p->win[b] ? p->top_p[b] : p->win[b];
    bp->seq[b].k = p->k_windows[b];
  }
  for (int b = 0; b < WKV_MAX_BATCH; ++b) bp->by_length[b] = (uint8_t)b;
  std::stable_sort(bp->by_length, bp->by_length + p->batch,
                   [&](uint8_t a, uint8_t c) { return p->seq_len[a] < p->seq_len[c]; });
}

// Number of (row, chunk) work items that hold at least one key, for chunks of `chunk` keys.
static int64_t count_items(const BatchParams &bp, int32_t B, int64_t rows_per_seq, int32_t drop, int32_t chunk) {
  int64_t n = 0;
  for (int32_t b = 0; b < B; ++b) n += ceil_div(std::max(bp.seq[b].L - drop, 0), chunk) * rows_per_seq;
  return n;
}

// Keys per workgroup.  The score kernels keep three workgroups resident on each of the 256
// compute units (one, with more than 128 softmax rows), and a workgroup's fixed cost (staging
// the query fragments, the first key load, the epilogue) is several microseconds: the launch is
// fastest when its non-empty work items fill those `slots` a whole number of times with chunks
// as long as the kernels allow.
// Chunks are multiples of 128 keys (one iteration of a workgroup); `drop` keys at the end of
// every sequence are not part of the pass.
static int32_t pick_chunk(const BatchParams &bp, int32_t B, int64_t rows_per_seq, int32_t drop, int32_t lo, int32_t hi,
                          int64_t slots) {
  int64_t total = 0;
  for (int32_t b = 0; b < B; ++b) total += (int64_t)std::max(bp.seq[b].L - drop, 0) * rows_per_seq;
  if (total <= 0) return lo;
  for (int64_t rounds = 1; rounds <= 64; ++rounds) {
    int64_t c = ceil_div(ceil_div(total, slots * rounds), 128) * 128;
    if (c < lo) return lo;
    while (c <= hi && count_items(bp, B, rows_per_seq, drop, (int32_t)c) > slots * rounds) c += 128;
    if (c <= hi) return (int32_t)c;
  }
  return hi;
}

ScorePlan plan_score(const Shape &s, const BatchParams &bp, int32_t n_groups) {
  ScorePlan pl;
  pl.m_pad = (s.M + 15) / 16 * 16;
  pl.mfma = s.dtype != WKV_F32;      // 16-bit inputs: matrix-pipe kernels (m_pad <= 256 always holds)
  const int64_t rows_per_seq = (int64_t)s.Hkv * n_groups;
  const int32_t Lmax = s.t_stride + s.w_obs;
  const int64_t slots = pl.m_pad <= 128 ? 768 : 256;
  pl.chunk1 = pick_chunk(bp, s.B, rows_per_seq, 0, 256, MAX_CHUNK1, slots);
  pl.n_chunks1 = (int32_t)ceil_div(Lmax, pl.chunk1);
  pl.chunk2 = pick_chunk(bp, s.B, rows_per_seq, s.w_obs, 256, MAX_CHUNK2, slots);
  pl.n_chunks2 = (int32_t)ceil_div(s.t_stride > 0 ? s.t_stride : 1, pl.chunk2);
  // every pass-2 workgroup re-reads rows * n_chunks1 partials when it folds them itself: worth
  // it (one launch less) only while that stays a few KB
  pl.fold_in_pass2 = pl.mfma && pl.n_chunks1 <= 16;
  // chunks are multiples of 128 keys: windows never straddle two workgroups when win divides 128
  pl.pool_in_pass2 = pl.mfma;
  for (int32_t b = 0; b < s.B; ++b) pl.pool_in_pass2 = pl.pool_in_pass2 && (128 % bp.seq[b].win == 0);
  return pl;
}

// The single-read kernel applies to 16-bit inputs with at most 128 softmax rows per KV head (its
// workgroups keep the row statistics of one row tile set in registers).  It is taken only when the
// caller asks for it: on MI355X the exchange of the row statistics between workgroups costs more
// than the second read of the keys it saves (measured at the 32K configuration: 0.57 ms against
// 0.21 ms for the two passes), so the library never chooses it by itself.
ResidentPlan plan_resident(const Shape &s, const BatchParams &bp, const ScorePlan &plan, int32_t n_groups, int32_t flags) {
  ResidentPlan rp;
  std::memset(&rp, 0, sizeof(rp));
  rp.m_pad = plan.m_pad;
  int64_t per_group = 0;
  for (int32_t b = 0; b < s.B; ++b) {
    const int64_t nsl = ceil_div(bp.seq[b].L, RK_SLICE);
    per_group += nsl * s.Hkv;
    if (nsl > rp.nsl_max) rp.nsl_max = (int32_t)nsl;
  }
  const int64_t items = per_group * n_groups;
  rp.items_per_group = (int32_t)per_group;
  rp.n_items = (int32_t)items;
  // a wait that is still unanswered after this many polls (tens of milliseconds) gives up
  rp.spin_limit = (flags & WKV_DEBUG_WAIT_GIVES_UP) ? 0 : (1 << 16);
  const bool can = plan.mfma && plan.m_pad <= 128 && s.t_stride > 0 && items < (int64_t)1 << 30;
  rp.use = can && (flags & WKV_SCORE_SINGLE_READ);
  return rp;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

Workspace carve_workspace(const Shape &s, const ScorePlan &plan, const ResidentPlan &rp, int32_t n_groups, void *base) {
  Workspace w;
  const size_t rows = (size_t)n_groups * s.B * s.Hkv;
  const size_t part = align256(rows * plan.m_pad * plan.n_chunks1 * sizeof(float2));
  const size_t tb = align256(rows * (size_t)(s.t_stride > 0 ? s.t_stride : 1) * sizeof(float));
  const size_t sb = align256(rows * (size_t)(s.nw_max > 0 ? s.nw_max : 1) * sizeof(float));
  const size_t lb = align256(rows * plan.m_pad * sizeof(float));
  // single-read kernel: the (m, z) partials of every slice and the synchronisation words
  const size_t rkp = rp.use ? align256(rows * (size_t)rp.nsl_max * rp.m_pad * sizeof(unsigned long long)) : 0;
  const size_t rks = rp.use ? align256((RK_GLOBAL_WORDS + rows * RK_SYNC_WORDS) * sizeof(uint32_t)) : 0;
  w.t_offset = part;
  w.s_offset = part + tb;
  w.bytes = part + tb + sb + lb + rkp + rks;
  char *b = (char *)base;          // a null base asks for the sizes only: no pointer is formed from it
  w.partials = b ? (float2 *)b : nullptr;
  w.t = b ? (float *)(b + w.t_offset) : nullptr;
  w.s = b ? (float *)(b + w.s_offset) : nullptr;
  w.lse = b ? (float *)(b + part + tb + sb) : nullptr;
  w.rk_partials = b && rp.use ? (unsigned long long *)(b + part + tb + sb + lb) : nullptr;
  w.rk_sync = b && rp.use ? (uint32_t *)(b + part + tb + sb + lb + rkp) : nullptr;
  return w;
}

wkv_status validate_decode(const wkv_decode_shape *p, Decode *out) {
  g_err[0] = 0;
  if (!p) { set_error("shape is NULL"); return WKV_ERR_INVALID_ARG; }
  if (p->batch < 1) { set_error("batch must be >= 1 (got %d)", p->batch); return WKV_ERR_INVALID_ARG; }
  if (p->n_kv_heads < 1 || p->n_q_heads < 1 || p->n_q_heads % p->n_kv_heads != 0) {
    set_error("n_q_heads (%d) must be a positive multiple of n_kv_heads (%d)", p->n_q_heads, p->n_kv_heads);
    return WKV_ERR_INVALID_ARG;
  }
  if ((int64_t)p->batch * p->n_kv_heads > 65535) {
    set_error("batch * n_kv_heads exceeds 65535 (launch grid limit); split the call"); return WKV_ERR_UNSUPPORTED;
  }
  const int32_t G = p->n_q_heads / p->n_kv_heads;
  if (G > 8) { set_error("n_q_heads / n_kv_heads = %d is not supported by the decode step (at most 8)", G); return WKV_ERR_UNSUPPORTED; }
  if (p->dtype != WKV_F32 && p->dtype != WKV_BF16 && p->dtype != WKV_F16) { set_error("unknown dtype %d", p->dtype); return WKV_ERR_INVALID_ARG; }
  if (p->head_dim != 64 && p->head_dim != 128) {
    set_error("head_dim %d is not supported (64 or 128)", p->head_dim); return WKV_ERR_UNSUPPORTED;
  }
  if (!(p->scale >= 0.0f) || std::isinf(p->scale)) {
    set_error("scale must be finite and >= 0 (0 selects 1/sqrt(head_dim))"); return WKV_ERR_INVALID_ARG;
  }
  if (p->capacity < 1) { set_error("capacity must be >= 1"); return WKV_ERR_INVALID_ARG; }
  if (p->flags & ~WKV_DECODE_KEEP_COUNT) { set_error("unknown bits in flags (0x%x)", p->flags); return WKV_ERR_INVALID_ARG; }
  const int64_t vec = 16 / elem_bytes(p->dtype);
  const int64_t strides[3] = {p->cache_stride_b, p->cache_stride_h, p->cache_stride_t};
  for (int i = 0; i < 3; ++i)
    if (strides[i] < 0 || strides[i] % vec != 0) {
      set_error("cache strides must be non-negative multiples of %lld elements (16 bytes)", (long long)vec);
      return WKV_ERR_INVALID_ARG;
    }
  if (p->cache_stride_t < p->head_dim || p->cache_stride_h < p->head_dim) {
    set_error("cache token and head strides must be >= head_dim"); return WKV_ERR_INVALID_ARG;
  }
  DecodeShape &s = out->shape;
  s.B = p->batch; s.Hq = p->n_q_heads; s.Hkv = p->n_kv_heads; s.d = p->head_dim; s.G = G; s.dtype = p->dtype;
  s.capacity = p->capacity;
  s.keep_count = (p->flags & WKV_DECODE_KEEP_COUNT) ? 1 : 0;
  const double scale = p->scale > 0.0f ? (double)p->scale : 1.0 / std::sqrt((double)p->head_dim);
  s.c1 = (float)(scale * 1.4426950408889634074);
  s.sb = p->cache_stride_b; s.sh = p->cache_stride_h; s.st = p->cache_stride_t;
  // about 1024 workgroups over the launch, key ranges of at least 256 rows (multiples of 64)
  const int64_t rows = (int64_t)s.B * s.Hkv;
  int64_t splits = std::min<int64_t>(std::max<int64_t>(ceil_div(1024, rows), 1), 64);
  int64_t chunk = std::max<int64_t>(ceil_div(ceil_div(s.capacity, splits), 64) * 64, 256);
  s.chunk = (int32_t)chunk;
  s.n_splits = (int32_t)ceil_div(s.capacity, chunk);
  out->ws_bytes = (size_t)rows * s.n_splits * s.G * (s.d + 2) * sizeof(float);
  return WKV_OK;
}

}  // namespace wkv

using namespace wkv;

extern "C" {

wkv_status wkv_get_dims(const wkv_problem *problem, wkv_dims *dims) {
  if (!dims) { set_error("dims is NULL"); return WKV_ERR_INVALID_ARG; }
  return validate(problem, dims);
}

size_t wkv_workspace_bytes(const wkv_problem *problem, int32_t n_groups) {
  wkv_dims dm;
  if (validate(problem, &dm) != WKV_OK) return 0;
  if (n_groups < 1 || n_groups > WKV_MAX_GROUPS) { set_error("n_groups outside [1, %d]", WKV_MAX_GROUPS); return 0; }
  Shape s; BatchParams bp;
  fill_shape(problem, dm, &s, &bp);
  ScorePlan pl = plan_score(s, bp, n_groups);
  return carve_workspace(s, pl, plan_resident(s, bp, pl, n_groups, problem->flags), n_groups, nullptr).bytes;
}

wkv_status wkv_get_workspace_layout(const wkv_problem *problem, int32_t n_groups, wkv_workspace_layout *layout) {
  if (!layout) { set_error("layout is NULL"); return WKV_ERR_INVALID_ARG; }
  wkv_dims dm;
  wkv_status st = validate(problem, &dm);
  if (st != WKV_OK) return st;
  if (n_groups < 1 || n_groups > WKV_MAX_GROUPS) { set_error("n_groups outside [1, %d]", WKV_MAX_GROUPS); return WKV_ERR_INVALID_ARG; }
  Shape s; BatchParams bp;
  fill_shape(problem, dm, &s, &bp);
  const ScorePlan pl = plan_score(s, bp, n_groups);
  const Workspace w = carve_workspace(s, pl, plan_resident(s, bp, pl, n_groups, problem->flags), n_groups, nullptr);
  layout->t_offset = w.t_offset;
  layout->s_offset = w.s_offset;
  layout->s_written = pl.pool_in_pass2 ? 1 : 0;
  layout->t_written = pl.pool_in_pass2 ? 0 : 1;
  return WKV_OK;
}

size_t wkv_decode_workspace_bytes(const wkv_decode_shape *shape) {
  Decode dc;
  if (validate_decode(shape, &dc) != WKV_OK) return 0;
  return dc.ws_bytes;
}

wkv_status wkv_group_budgets(double b_total, int32_t n_groups, double lambda, double *budgets_out) {
  if (!budgets_out) { set_error("budgets_out is NULL"); return WKV_ERR_INVALID_ARG; }
  if (n_groups < 1 || !(lambda > 0.0) || !(b_total >= 0.0)) {
    set_error("need n_groups >= 1, lambda > 0, b_total >= 0"); return WKV_ERR_INVALID_ARG;
  }
  const double H = (double)n_groups;
  if (n_groups == 1) { budgets_out[0] = b_total; return WKV_OK; }
  const double top = b_total / (lambda * H);          // Eq. 6, group H-1
  const double bottom = 2.0 * b_total / H - top;      // Eq. 6, group 0
  const double step = (bottom - top) / (H - 1.0);     // Eq. 7
  for (int32_t h = 0; h < n_groups; ++h) budgets_out[h] = bottom - step * (double)h;
  return WKV_OK;
}

const char *wkv_status_string(wkv_status st) {
  switch (st) {
    case WKV_OK: return "ok";
    case WKV_ERR_INVALID_ARG: return "invalid argument";
    case WKV_ERR_UNSUPPORTED: return "unsupported problem";
    case WKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case WKV_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

const char *wkv_last_error(void) { return g_err; }

}  // extern "C"
