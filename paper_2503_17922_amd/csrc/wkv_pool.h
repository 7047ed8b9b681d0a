// Window pooling (WindowKV Eq. 3-4) of one window by one thread; shared by the pooling kernel,
// the fused selection kernel and the score kernel's epilogue, so that all three give the same bits.
#pragma once

#include "wkv_internal.h"

namespace wkv {

// ------------------------------------------------------------------------------------------
// Eq. 3-4: s_w = sum(Top-p(W_w)) / min(p, win), one thread per window.
// Register-resident pooling for the common window sizes.  The window's token scores sit in
// registers (loaded as float4s: a lane reads its window's 4*WIN contiguous bytes) and are put
// in descending order by a fully unrolled bitonic network (min/max pairs, nothing indexed
// dynamically); the score is the sum of the first p.  Which of several equal values counts
// as "in the top p" does not change that sum.
// ------------------------------------------------------------------------------------------
template <int WIN>
__device__ __forceinline__ float pool_window_regs(const float *__restrict__ trow, int w, int n_review, int p) {
  float v[WIN];
  const int tok0 = w * WIN;
  const int size = min(WIN, n_review - tok0);
  if (size == WIN && ((uintptr_t)(trow + tok0) & 15) == 0) {
#pragma unroll
    for (int i = 0; i < WIN; i += 4) {
      const float4 q = *(const float4 *)(trow + tok0 + i);
      v[i] = q.x; v[i + 1] = q.y; v[i + 2] = q.z; v[i + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < WIN; ++i) v[i] = i < size ? trow[tok0 + i] : -INFINITY;
  }
  float acc = 0.0f;
  if (p >= size) {
#pragma unroll
    for (int i = 0; i < WIN; ++i) acc += i < size ? v[i] : 0.0f;
  } else {
#pragma unroll
    for (int k = 2; k <= WIN; k <<= 1)
#pragma unroll
      for (int j = k >> 1; j > 0; j >>= 1)
#pragma unroll
        for (int i = 0; i < WIN; ++i) {
          const int l = i ^ j;
          if (l > i) {
            const float lo = fminf(v[i], v[l]), hi = fmaxf(v[i], v[l]);
            const bool descending = (i & k) == 0;
            v[i] = descending ? hi : lo;
            v[l] = descending ? lo : hi;
          }
        }
#pragma unroll
    for (int i = 0; i < WIN; ++i) acc += i < p ? v[i] : 0.0f;     // p < size: none of these is padding
  }
  return acc / (float)p;
}

// Any window size: plain loops over global memory (cached; O(size^2) compares).  Element i is
// kept when fewer than p elements are larger, equal values ordered by position.
__device__ __forceinline__ float pool_window_any(const float *__restrict__ trow, int w, int win, int n_review, int p) {
  const int tok0 = w * win;
  const int size = min(win, n_review - tok0);
  float acc = 0.0f;
  if (p >= size) {
    for (int i = 0; i < size; ++i) acc += trow[tok0 + i];
  } else {
    for (int i = 0; i < size; ++i) {
      const float vi = trow[tok0 + i];
      int rank = 0;
      for (int j = 0; j < size; ++j) {
        const float vj = trow[tok0 + j];
        rank += (vj > vi) || (vj == vi && j < i);
      }
      if (rank < p) acc += vi;
    }
  }
  return acc / (float)p;
}

// Window score by whichever of the two fits the window size (uniform per workgroup).
__device__ __forceinline__ float pool_window(const float *__restrict__ trow, int w, int win, int n_review, int p) {
  switch (win) {
    case 8: return pool_window_regs<8>(trow, w, n_review, p);
    case 16: return pool_window_regs<16>(trow, w, n_review, p);
    case 32: return pool_window_regs<32>(trow, w, n_review, p);
    default: return pool_window_any(trow, w, win, n_review, p);
  }
}

}  // namespace wkv
