// Top-k window selection (WindowKV Section 2.2.1) on window scores that sit in LDS as
// order-preserving keys; shared by the selection kernels and by the score kernel's tail (the
// workgroup that finishes a row last selects for it).
#pragma once

#include "wkv_internal.h"

namespace wkv {

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
constexpr int TOPK_THREADS = 1024;       // of the stand-alone selection kernels

__device__ __forceinline__ uint32_t float_to_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Steps 2-4 on the keys already in LDS (all NT threads of the workgroup take part and must have
// passed a barrier after the keys were written); `row` is the (group, sequence, KV head) index.
template <int NT>
__device__ __forceinline__ void topk_body(const Shape &s, const SeqParam sp, uint32_t *keys, int64_t row,
                                          int32_t *__restrict__ win_idx, int32_t *__restrict__ tok_idx,
                                          int32_t *__restrict__ n_keep) {
  constexpr int TOPK_WAVES = NT / 64;
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
      for (int w = tid; w < nw; w += NT) {
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
  for (int base = 0; base < nw; base += NT) {
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
      keys[slot] = (uint32_t)w;                   // slot <= w < base + NT: already consumed
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
  for (int i = k + tid; i < s.k_max; i += NT) wrow[i] = -1;

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
  for (int r = tid; r < s.nkeep_max; r += NT) {
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

}  // namespace wkv
