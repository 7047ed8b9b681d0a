// Device-side helpers shared by the score kernels (not part of the ABI).
#pragma once

#include "wkv_internal.h"

namespace wkv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;

// D = A (16 x 32) * B (32 x 16) + C on the matrix pipe; the 16-byte operands hold 8 bfloat16 or
// (F16) 8 IEEE half values and travel as bf16x8 either way.
template <bool F16>
__device__ __forceinline__ f32x4 mfma_16x16x32(bf16x8 a, bf16x8 b, f32x4 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Merge (m2, z2) into (m, z): both describe sum 2^(v - m) over disjoint key sets.
__device__ __forceinline__ void merge_stats(float &m, float &z, float m2, float z2) {
  const float mn = fmaxf(m, m2);
  if (mn == -INFINITY) { m = mn; z = 0.0f; return; }
  z = z * fast_exp2(m - mn) + z2 * fast_exp2(m2 - mn);
  m = mn;
}

// (m, z) of one row over the partials c = first, first + step, ... < n_chunks.  Loads are
// issued four at a time so that their latencies overlap.
__device__ __forceinline__ void fold_partials_strided(const float2 *__restrict__ part, int n_chunks, int first,
                                                      int step, float &m, float &z) {
  m = -INFINITY;
  z = 0.0f;
  int c = first;
  for (; c + 3 * step < n_chunks; c += 4 * step) {
    const float2 p0 = part[c], p1 = part[c + step], p2 = part[c + 2 * step], p3 = part[c + 3 * step];
    const float mn = fmaxf(fmaxf(fmaxf(p0.x, p1.x), fmaxf(p2.x, p3.x)), m);
    if (mn != -INFINITY) {
      z = z * fast_exp2(m - mn) + p0.y * fast_exp2(p0.x - mn) + p1.y * fast_exp2(p1.x - mn) +
          p2.y * fast_exp2(p2.x - mn) + p3.y * fast_exp2(p3.x - mn);
      m = mn;
    }
  }
  for (; c < n_chunks; c += step) merge_stats(m, z, part[c].x, part[c].y);
}

// lse2 of one row from its per-chunk partials (single thread).
__device__ __forceinline__ float fold_partials(const float2 *__restrict__ part, int n_chunks) {
  float m, z;
  fold_partials_strided(part, n_chunks, 0, 1, m, z);
  return m + fast_log2(z);
}

// ---- MFMA building blocks (bf16, v_mfma_f32_16x16x32_bf16) ----------------------------------
constexpr int MF_THREADS = 256;           // per row half (see score_mfma_kernel)
constexpr int MF_WAVES = 4;              // waves that share the key tiles of an iteration
constexpr int MF_KT = 2;                 // key tiles of 16 per wave iteration (share each B fragment)
constexpr float MF_BIG = 1.0e30f;        // a tile sum above this re-references the row (2^100)

// Arrange the M query rows of KV head h as MFMA B fragments in LDS.
// Fragment (mt, ks) is 64 x 16 bytes: lane l holds row 16*mt + l%16, channels 32*ks + 8*(l/16)..+7.
template <int D, int MT, int NT>                          // NT threads stage MT row tiles
struct QStage {
  static constexpr int KS = D / 32;
  static constexpr int TOTAL = MT * KS * 64;               // 16-byte pieces of the fragments
  static constexpr int N = (TOTAL + NT - 1) / NT;          // per thread
  uint4 v[N];
  // Issue every load of this thread at once (independent of each other, so their latencies
  // overlap; a load-then-store loop would pay one round trip per piece).
  __device__ __forceinline__ void load(const Shape &s, const void *qbase, int b, int h, int tid = threadIdx.x) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int i = tid + k * NT;
      const int l = i & 63, f = i >> 6, ks = f % KS, mt = f / KS;
      const int r = mt * 16 + (l & 15);
      v[k] = make_uint4(0u, 0u, 0u, 0u);
      if (i < TOTAL && r < s.M) {
        const int hq = h * s.G + r / s.w_obs, io = r % s.w_obs;
        const int64_t off = (int64_t)b * s.q_sb + (int64_t)hq * s.q_sh + (int64_t)io * s.q_st + ks * 32 + (l >> 4) * 8;
        v[k] = *(const uint4 *)((const uint16_t *)qbase + off);
      }
    }
  }
  __device__ __forceinline__ void store(uint4 *qfrag, int tid = threadIdx.x) const {
#pragma unroll
    for (int k = 0; k < N; ++k)
      if (tid + k * NT < TOTAL) qfrag[tid + k * NT] = v[k];
  }
};

// Sum over the 16 lanes of a DPP row (lanes with equal l/16); every lane gets the total.
__device__ __forceinline__ float row16_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, false)); // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, false)); // row_mirror
  return x;
}

template <int KS>
struct KFrags {
  bf16x8 f[MF_KT][KS];
};

// Loads the A fragments of MF_KT key tiles starting at key j0 (rows clamped into [0, L-1];
// callers pass L >= 1).
template <int KS>
__device__ __forceinline__ void load_k(KFrags<KS> &kf, const uint16_t *kbase, int64_t st, int j0, int col, int L) {
#pragma unroll
  for (int n = 0; n < MF_KT; ++n) {
    const int j = min(j0 + n * 16 + col, L - 1);
    const uint16_t *kp = kbase + (int64_t)j * st;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf.f[n][ks] = *(const bf16x8 *)(kp + ks * 32);
  }
}

}  // namespace wkv
