// Window pooling (WindowKV Eq. 3-4) and top-k window selection (Section 2.2.1).
//
// Both stages touch only the token-score array (4 bytes per prefix token and KV head), about
// 1/64 of the bytes of the key stream that produced it, so they are latency bound rather than
// bandwidth bound: the design goal is few launches and no serial host involvement.
#include "wkv_internal.h"
#include "wkv_pool.h"
#include "wkv_topk.h"

namespace wkv {

constexpr int POOL_THREADS = 256;

// One thread per window.
__global__ __launch_bounds__(POOL_THREADS) void pool_kernel(Shape s, BatchParams bp, const float *__restrict__ t,
                                                                 float *__restrict__ s_out) {
  const int bh = blockIdx.y, b = bh / s.Hkv, g = blockIdx.z;
  const SeqParam sp = bp.seq[b];
  const int n_review = sp.L - s.w_obs;
  const int nw = (n_review + sp.win - 1) / sp.win;
  const int64_t row = (int64_t)g * s.B * s.Hkv + bh;
  const int w = blockIdx.x * POOL_THREADS + threadIdx.x;
  if (w >= s.nw_max) return;
  s_out[row * s.nw_max + w] = w < nw ? pool_window(t + row * s.t_stride, w, sp.win, n_review, sp.p) : -INFINITY;
}

hipError_t launch_pool(const Shape &s, const BatchParams &bp, int32_t n_groups, const float *t,
                       float *s_out, hipStream_t stream) {
  if (s.nw_max <= 0) return hipSuccess;
  dim3 grid((s.nw_max + POOL_THREADS - 1) / POOL_THREADS, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL(pool_kernel, grid, dim3(POOL_THREADS), 0, stream, s, bp, t, s_out);
  return hipGetLastError();
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(Shape s, BatchParams bp, GroupK gk,
                                                            const float *__restrict__ sc,
                                                            int32_t *__restrict__ win_idx,
                                                            int32_t *__restrict__ tok_idx,
                                                            int32_t *__restrict__ n_keep) {
  extern __shared__ uint32_t keys[];            // [nw_max], later reused for the selected list
  const int bh = blockIdx.x, b = bh / s.Hkv, g = blockIdx.y;
  SeqParam sp = bp.seq[b];
  if (gk.in_use) sp.k = gk.k[g * s.B + b];      // the group's own budget
  const int nw = (sp.L - s.w_obs + sp.win - 1) / sp.win;
  const int64_t row = (int64_t)g * s.B * s.Hkv + bh;
  const float *srow = sc + row * s.nw_max;
  for (int w = threadIdx.x; w < nw; w += TOPK_THREADS) keys[w] = float_to_key(srow[w]);
  __syncthreads();
  topk_body<TOPK_THREADS>(s, sp, keys, row, win_idx, tok_idx, n_keep);
}

// Pooling and selection in one launch (the path wkv_compress_groups takes): the window scores
// go straight from registers into the LDS key array and never touch global memory.
__global__ __launch_bounds__(TOPK_THREADS) void select_kernel(Shape s, BatchParams bp, GroupK gk,
                                                              const float *__restrict__ t,
                                                              int32_t *__restrict__ win_idx,
                                                              int32_t *__restrict__ tok_idx,
                                                              int32_t *__restrict__ n_keep) {
  extern __shared__ uint32_t keys[];
  const int bh = blockIdx.x, b = bh / s.Hkv, g = blockIdx.y;
  SeqParam sp = bp.seq[b];
  if (gk.in_use) sp.k = gk.k[g * s.B + b];      // the group's own budget
  const int n_review = sp.L - s.w_obs;
  const int nw = (n_review + sp.win - 1) / sp.win;
  const int64_t row = (int64_t)g * s.B * s.Hkv + bh;
  const float *trow = t + row * s.t_stride;
  for (int w = threadIdx.x; w < nw; w += TOPK_THREADS)
    keys[w] = float_to_key(pool_window(trow, w, sp.win, n_review, sp.p));
  __syncthreads();
  topk_body<TOPK_THREADS>(s, sp, keys, row, win_idx, tok_idx, n_keep);
}

hipError_t launch_topk(const Shape &s, const BatchParams &bp, const GroupK &gk, int32_t n_groups, const float *sc,
                       int32_t *win_idx, int32_t *tok_idx, int32_t *n_keep, hipStream_t stream) {
  const size_t lds = (size_t)(s.nw_max > 0 ? s.nw_max : 1) * sizeof(uint32_t);
  if (lds > 48 * 1024) {     // beyond the default dynamic-LDS limit: raise it (per device, any thread)
    hipError_t e = hipFuncSetAttribute((const void *)topk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       WKV_MAX_WINDOWS * (int)sizeof(uint32_t));
    if (e != hipSuccess) return e;
  }
  dim3 grid(s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL(topk_kernel, grid, dim3(TOPK_THREADS), lds, stream, s, bp, gk, sc, win_idx, tok_idx, n_keep);
  return hipGetLastError();
}

hipError_t launch_select(const Shape &s, const BatchParams &bp, const GroupK &gk, int32_t n_groups, const float *t,
                         int32_t *win_idx, int32_t *tok_idx, int32_t *n_keep, hipStream_t stream) {
  const size_t lds = (size_t)(s.nw_max > 0 ? s.nw_max : 1) * sizeof(uint32_t);
  if (lds > 48 * 1024) {     // beyond the default dynamic-LDS limit: raise it (per device, any thread)
    hipError_t e = hipFuncSetAttribute((const void *)select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       WKV_MAX_WINDOWS * (int)sizeof(uint32_t));
    if (e != hipSuccess) return e;
  }
  dim3 grid(s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL(select_kernel, grid, dim3(TOPK_THREADS), lds, stream, s, bp, gk, t, win_idx, tok_idx, n_keep);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Jaccard similarity of the retained positions of every pair of index sets (Section 3.2).
// One workgroup per (set i, set j, sequence, KV head): both rows are ascending, so each thread
// looks its elements of row i up in row j by binary search; |A u B| = |A| + |B| - |A n B|.
// ------------------------------------------------------------------------------------------
constexpr int JAC_THREADS = 256;

__global__ __launch_bounds__(JAC_THREADS) void jaccard_kernel(Shape s, int32_t n_sets, const int32_t *__restrict__ tok_idx,
                                                              const int32_t *__restrict__ n_keep,
                                                              float *__restrict__ out) {
  __shared__ int wave_hits[JAC_THREADS / 64];
  const int bh = blockIdx.x, i = blockIdx.y, j = blockIdx.z;
  const int64_t rows = (int64_t)s.B * s.Hkv;
  const int32_t *a = tok_idx + ((int64_t)i * rows + bh) * s.nkeep_max;
  const int32_t *b = tok_idx + ((int64_t)j * rows + bh) * s.nkeep_max;
  const int na = min(max(n_keep[(int64_t)i * rows + bh], 0), s.nkeep_max);
  const int nb = min(max(n_keep[(int64_t)j * rows + bh], 0), s.nkeep_max);
  int hits = 0;
  for (int k = threadIdx.x; k < na; k += JAC_THREADS) {
    const int32_t x = a[k];
    int lo = 0, hi = nb;                       // first position of row j not below x
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (b[mid] < x) lo = mid + 1; else hi = mid;
    }
    hits += lo < nb && b[lo] == x;
  }
  for (int off = 32; off > 0; off >>= 1) hits += __shfl_xor(hits, off);
  if ((threadIdx.x & 63) == 0) wave_hits[threadIdx.x >> 6] = hits;
  __syncthreads();
  if (threadIdx.x == 0) {
    int inter = 0;
    for (int w = 0; w < JAC_THREADS / 64; ++w) inter += wave_hits[w];
    const int uni = na + nb - inter;
    out[((int64_t)i * n_sets + j) * rows + bh] = uni == 0 ? 1.0f : (float)inter / (float)uni;
  }
}

hipError_t launch_jaccard(const Shape &s, int32_t n_sets, const int32_t *tok_idx, const int32_t *n_keep, float *out,
                          hipStream_t stream) {
  dim3 grid(s.B * s.Hkv, n_sets, n_sets);
  hipLaunchKernelGGL(jaccard_kernel, grid, dim3(JAC_THREADS), 0, stream, s, n_sets, tok_idx, n_keep, out);
  return hipGetLastError();
}

}  // namespace wkv
