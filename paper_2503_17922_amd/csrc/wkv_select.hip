// Window pooling (WindowKV Eq. 3-4) and top-k window selection (Section 2.2.1).
//
// Both stages touch only the token-score array (4 bytes per prefix token and KV head), about
// 1/64 of the bytes of the key stream that produced it, so they are latency bound rather than
// bandwidth bound: the design goal is few launches and no serial host involvement.
#include "wkv_internal.h"
#include "wkv_pool.h"

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

// ------------------------------------------------------------------------------------------
// Top-k windows.  One 1024-thread workgroup per (group, sequence, KV head).
//   1. window scores -> order-preserving uint32 keys in LDS
//   2. radix select (4 passes of 8 bits, LDS histogram) for the k-th largest key T and the
//      number `take_eq` of windows equal to T that still fit
//   3. one ordered sweep: window w is kept iff key > T, or key == T and fewer than take_eq
//      equal windows precede it (=> lower index wins ties).  Its output slot is
//      (#greater before w) + min(#equal before w, take_eq), found with ballot/popcount
//      prefix sums, so the list comes out ascending without a sort.
//   4. expansion to token positions, the observation window appended, -1 padding.
// ------------------------------------------------------------------------------------------
constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;

__device__ __forceinline__ uint32_t float_to_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Steps 2-4 on the keys already in LDS; `row` is the (group, sequence, KV head) index.
__device__ __forceinline__ void topk_body(const Shape &s, const SeqParam sp, uint32_t *keys, int64_t row,
                                          int32_t *__restrict__ win_idx, int32_t *__restrict__ tok_idx,
                                          int32_t *__restrict__ n_keep) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_remaining;
  __shared__ int wave_gt[TOPK_WAVES], wave_eq[TOPK_WAVES];
  __shared__ int run_gt, run_eq;

  const int n_review = sp.L - s.w_obs;
  const int nw = (n_review + sp.win - 1) / sp.win;
  const int k = sp.k;
  int32_t *wrow = win_idx + row * s.k_max;
  int32_t *trow = tok_idx + row * s.nkeep_max;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  if (tid == 0) { sh_prefix = 0u; sh_remaining = (uint32_t)k; }
  __syncthreads();
  // ---- 2. radix select -------------------------------------------------------------------
  uint32_t T = 0u, take_eq = 0u;
  if (k > 0) {
    uint32_t mask = 0u;
    for (int pass = 3; pass >= 0; --pass) {
      const int shift = pass * 8;
      if (tid < 256) hist[tid] = 0u;
      __syncthreads();
      const uint32_t prefix = sh_prefix;
      for (int w = tid; w < nw; w += TOPK_THREADS) {
        const uint32_t key = keys[w];
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (wave == 0) {
        // suffix sums over the 256 bins, 4 bins per lane, highest bins first
        const uint32_t remaining = sh_remaining;
        uint32_t c[4];
        uint32_t local = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) { c[i] = hist[255 - (lane * 4 + i)]; local += c[i]; }
        uint32_t incl = local;                     // inclusive scan over lanes
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const uint32_t o = __shfl_up(incl, off);
          if (lane >= off) incl += o;
        }
        uint32_t above = incl - local;             // windows in strictly higher bins
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (above < remaining && above + c[i] >= remaining) {
            sh_prefix = prefix | ((uint32_t)(255 - (lane * 4 + i)) << shift);
            sh_remaining = remaining - above;
          }
          above += c[i];
        }
      }
      mask |= 255u << shift;
      __syncthreads();
    }
    T = sh_prefix;
    take_eq = sh_remaining;
  }

  // ---- 3. ordered compaction -------------------------------------------------------------
  if (tid == 0) { run_gt = 0; run_eq = 0; }
  __syncthreads();
  for (int base = 0; base < nw; base += TOPK_THREADS) {
    const int w = base + tid;
    const bool valid = w < nw && k > 0;
    const uint32_t key = valid ? keys[w] : 0u;
    const bool gt = valid && key > T;
    const bool eq = valid && key == T;
    const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    const int gt_in_wave = __popcll(bgt & below), eq_in_wave = __popcll(beq & below);
    if (lane == 0) { wave_gt[wave] = __popcll(bgt); wave_eq[wave] = __popcll(beq); }
    __syncthreads();                              // also orders the key reads before the writes below
    int gt_before = run_gt + gt_in_wave, eq_before = run_eq + eq_in_wave;
    for (int i = 0; i < wave; ++i) { gt_before += wave_gt[i]; eq_before += wave_eq[i]; }
    const bool keep = gt || (eq && (uint32_t)eq_before < take_eq);
    if (keep) {
      const int slot = gt_before + min(eq_before, (int)take_eq);
      keys[slot] = (uint32_t)w;                   // slot <= w < base + TOPK_THREADS: already consumed
      wrow[slot] = w;
    }
    __syncthreads();
    if (tid == 0) {
      int a = 0, e = 0;
      for (int i = 0; i < TOPK_WAVES; ++i) { a += wave_gt[i]; e += wave_eq[i]; }
      run_gt += a; run_eq += e;
    }
    __syncthreads();
  }
  for (int i = k + tid; i < s.k_max; i += TOPK_THREADS) wrow[i] = -1;

  // ---- 4. token positions ------------------------------------------------------------------
  // Only the last window of the sequence can be partial, and if selected it is the last of
  // the ascending list, so slot m < k starts at m*win.
  int n_rev_kept = k * sp.win;
  if (k > 0) {
    const int last = (int)keys[k - 1];
    const int missing = (last + 1) * sp.win - n_review;
    if (missing > 0) n_rev_kept -= missing;
  }
  const int nk = n_rev_kept + s.w_obs;
  for (int r = tid; r < s.nkeep_max; r += TOPK_THREADS) {
    int tok = -1;
    if (r < n_rev_kept) {
      const int m = r / sp.win;
      tok = (int)keys[m] * sp.win + (r - m * sp.win);
    } else if (r < nk) {
      tok = n_review + (r - n_rev_kept);
    }
    trow[r] = tok;
  }
  if (tid == 0) n_keep[row] = nk;
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
  topk_body(s, sp, keys, row, win_idx, tok_idx, n_keep);
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
  topk_body(s, sp, keys, row, win_idx, tok_idx, n_keep);
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
