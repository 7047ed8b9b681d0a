// Observation-window token scores (WindowKV Eq. 1-2) for one or more layer groups.
//
//   t[b,h,j] = sum_{g<G} sum_{i<w_obs} softmax_j( q_{g,i} . k_j * scale )      j < L - w_obs
//
// The G*w_obs query rows that share a KV head are stacked into one M-row operand, so the
// logits of a KV head are one [M x d] x [d x L] contraction.  The softmax normaliser of a row
// needs every key of the prefix before any column sum can be finished, hence two passes over
// the keys of the scored layer:
//
//   pass 1 (stats)  per (row, key chunk): running maximum m and sum z = sum 2^(v - m) of the
//                   base-2 logits v = (q.k) * scale * log2(e), with the causal mask of the
//                   observation block applied.  Partials go to the workspace.
//   pass 2 (score)  each workgroup folds the partials of its KV head into one
//                   lse2_i = m_i + log2(z_i) per row, recomputes its logits and writes
//                   t_j = sum_i 2^(v_ij - lse2_i).
//
// Two kernel families implement the passes:
//   * MFMA (bf16 inputs, M <= 128): v_mfma_f32_16x16x32_bf16 with the query rows as the A
//     operand (fragments pre-arranged in LDS, one conflict-free ds_read_b128 per fragment) and
//     the keys as the B operand, loaded straight from global memory into registers in
//     operand layout (lane = key l%16, 16-byte piece l/16 of a 64-byte run), so K never
//     passes through LDS and the four waves of a workgroup never synchronise in the loop.
//     In the 16x16 result layout a lane holds 4 rows of one key column: the column sums of
//     Eq. 2 are in-lane adds plus two cross-lane steps, and per-row statistics are kept
//     per lane and only merged once per chunk.
//   * generic (fp32 inputs, or M > 128): plain fp32 FMAs, thread-per-row for the stats,
//     thread-per-key for the scores, the other operand broadcast from LDS.
#include "wkv_internal.h"

namespace wkv {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

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

// lse2 of one row from its per-chunk partials.
__device__ __forceinline__ float fold_partials(const float2 *__restrict__ part, int n_chunks) {
  float m = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) m = fmaxf(m, part[c].x);
  float z = 0.0f;
  for (int c = 0; c < n_chunks; ++c) {
    const float2 pz = part[c];
    if (pz.x != -INFINITY) z += pz.y * fast_exp2(pz.x - m);
  }
  return m + fast_log2(z);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const void *p, int64_t i) { return ((const float *)p)[i]; }
};
template <> struct Elem<uint16_t> {
  static __device__ __forceinline__ float load(const void *p, int64_t i) { return bf16_to_float(((const uint16_t *)p)[i]); }
};

// =========================================================================================
// generic kernels
// =========================================================================================
constexpr int GEN_THREADS = 256;
constexpr int GEN_KT = 32;   // keys staged per LDS tile in the stats kernel

// Pass 1, generic.  Thread (row r = tid % R, key lane kl = tid / R); R = rows rounded up to a
// power of two <= 256, KL = 256 / R.  Each thread keeps its query row in registers and walks
// the staged key tile with broadcast LDS reads.
template <typename T, int D>
__global__ __launch_bounds__(GEN_THREADS) void stats_generic_kernel(Shape s, BatchParams bp, GroupPtrs gp,
                                                                    ScorePlan pl, float2 *__restrict__ partials,
                                                                    int R) {
  __shared__ float ktile[GEN_KT][D + 1];
  __shared__ float2 red[GEN_THREADS];
  const int bh = blockIdx.y, b = bh / s.Hkv, h = bh % s.Hkv, g = blockIdx.z;
  const int L = bp.seq[b].L;
  const int c0 = blockIdx.x * pl.chunk1;
  const int64_t prow = (((int64_t)g * s.B * s.Hkv + bh) * pl.m_pad) * pl.n_chunks1 + blockIdx.x;
  const int r = threadIdx.x % R, kl = threadIdx.x / R, KL = GEN_THREADS / R;
  const bool row_ok = r < s.M;
  // query row r: head h*G + r / w_obs, observation index r % w_obs
  float q[D];
  const int io = r % s.w_obs;
  if (row_ok) {
    const int hq = h * s.G + r / s.w_obs;
    const int64_t qoff = (int64_t)b * s.q_sb + (int64_t)hq * s.q_sh + (int64_t)io * s.q_st;
#pragma unroll
    for (int c = 0; c < D; ++c) q[c] = Elem<T>::load(gp.q[g], qoff + c);
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) q[c] = 0.0f;
  }
  const int last_visible = L - s.w_obs + io;   // causal: key j visible iff j <= last_visible
  const int c1 = min(c0 + pl.chunk1, L);
  float m = -INFINITY, z = 0.0f;
  const int64_t koff = (int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh;
  for (int j0 = c0; j0 < c1; j0 += GEN_KT) {
    __syncthreads();
    for (int i = threadIdx.x; i < GEN_KT * D; i += GEN_THREADS) {
      const int jj = i / D, c = i % D;
      const int j = j0 + jj;
      ktile[jj][c] = j < c1 ? Elem<T>::load(gp.k[g], koff + (int64_t)j * s.kv_st + c) : 0.0f;
    }
    __syncthreads();
    for (int jj = kl; jj < GEN_KT; jj += KL) {
      const int j = j0 + jj;
      if (j < c1 && j <= last_visible && row_ok) {
        float dot = 0.0f;
#pragma unroll
        for (int c = 0; c < D; ++c) dot = fmaf(q[c], ktile[jj][c], dot);
        merge_stats(m, z, dot * s.c1, 1.0f);
      }
    }
  }
  red[threadIdx.x] = make_float2(m, z);
  __syncthreads();
  if (kl == 0 && r < pl.m_pad) {
    for (int i = 1; i < KL; ++i) merge_stats(m, z, red[i * R + r].x, red[i * R + r].y);
    partials[prow + (int64_t)r * pl.n_chunks1] = make_float2(m, z);
  }
}

// Pass 2, generic.  One thread per key of the chunk; query rows and their lse2 are broadcast
// from LDS; the key row lives in registers.
template <typename T, int D>
__global__ __launch_bounds__(GEN_THREADS) void score_generic_kernel(Shape s, BatchParams bp, GroupPtrs gp,
                                                                    ScorePlan pl,
                                                                    const float2 *__restrict__ partials,
                                                                    float *__restrict__ t_out) {
  extern __shared__ float smem[];            // q [M][D], then lse2 [M]
  float *qs = smem;
  float *lse = smem + (size_t)s.M * D;
  const int bh = blockIdx.y, b = bh / s.Hkv, h = bh % s.Hkv, g = blockIdx.z;
  const int n_review = bp.seq[b].L - s.w_obs;
  const int64_t row = (int64_t)g * s.B * s.Hkv + bh;
  float *trow = t_out + row * s.t_stride;
  const int c0 = blockIdx.x * pl.chunk2;
  const int cend = min(c0 + pl.chunk2, s.t_stride);
  if (c0 >= n_review) {                      // nothing to score here: only the zero fill
    for (int j = c0 + threadIdx.x; j < cend; j += GEN_THREADS) trow[j] = 0.0f;
    return;
  }
  for (int i = threadIdx.x; i < s.M * D; i += GEN_THREADS) {
    const int r = i / D, c = i % D;
    const int hq = h * s.G + r / s.w_obs, io = r % s.w_obs;
    qs[i] = Elem<T>::load(gp.q[g], (int64_t)b * s.q_sb + (int64_t)hq * s.q_sh + (int64_t)io * s.q_st + c);
  }
  for (int r = threadIdx.x; r < s.M; r += GEN_THREADS)
    lse[r] = fold_partials(partials + (row * pl.m_pad + r) * pl.n_chunks1, pl.n_chunks1);
  __syncthreads();
  const int64_t koff = (int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh;
  for (int j = c0 + threadIdx.x; j < cend; j += GEN_THREADS) {
    float tj = 0.0f;
    if (j < n_review) {
      float kr[D];
#pragma unroll
      for (int c = 0; c < D; ++c) kr[c] = Elem<T>::load(gp.k[g], koff + (int64_t)j * s.kv_st + c);
      for (int r = 0; r < s.M; ++r) {
        float dot = 0.0f;
#pragma unroll
        for (int c = 0; c < D; ++c) dot = fmaf(qs[r * D + c], kr[c], dot);
        tj += fast_exp2(fmaf(dot, s.c1, -lse[r]));
      }
    }
    trow[j] = tj;
  }
}

// =========================================================================================
// MFMA kernels (bf16)
// =========================================================================================
constexpr int MF_THREADS = 256;
constexpr int MF_WAVES = 4;
constexpr int MF_NT = 2;        // key tiles of 16 that share one A-fragment read
constexpr float MF_RESCALE = 16.0f;   // re-reference a row when a logit exceeds its reference by 2^16

// Arrange the M query rows of KV head h as MFMA A fragments in LDS.
// Fragment (mt, ks) is 64 x 16 bytes: lane l holds row 16*mt + l%16, channels 32*ks + 8*(l/16)..+7.
template <int D, int MT>
__device__ __forceinline__ void stage_q_fragments(const Shape &s, const void *qbase, int b, int h, uint4 *qfrag) {
  constexpr int KS = D / 32;
  for (int i = threadIdx.x; i < MT * KS * 64; i += MF_THREADS) {
    const int l = i & 63, f = i >> 6, ks = f % KS, mt = f / KS;
    const int r = mt * 16 + (l & 15);
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r < s.M) {
      const int hq = h * s.G + r / s.w_obs, io = r % s.w_obs;
      const int64_t off = (int64_t)b * s.q_sb + (int64_t)hq * s.q_sh + (int64_t)io * s.q_st + ks * 32 + (l >> 4) * 8;
      v = *(const uint4 *)((const uint16_t *)qbase + off);
    }
    qfrag[i] = v;
  }
}

// PASS 1: stats.  PASS 2: scores.
template <int D, int MT, int PASS>
__global__ __launch_bounds__(MF_THREADS, 2) void score_mfma_kernel(Shape s, BatchParams bp, GroupPtrs gp,
                                                                   ScorePlan pl, float2 *__restrict__ partials,
                                                                   float *__restrict__ t_out) {
  constexpr int KS = D / 32;
  __shared__ uint4 qfrag[MT * KS * 64];
  __shared__ float lse_s[MT * 16];
  __shared__ float2 wave_part[MF_WAVES][MT * 16];

  const int bh = blockIdx.y, b = bh / s.Hkv, h = bh % s.Hkv, g = blockIdx.z;
  const int L = bp.seq[b].L;
  const int n_review = L - s.w_obs;
  const int64_t row = (int64_t)g * s.B * s.Hkv + bh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;

  const int chunk = PASS == 1 ? pl.chunk1 : pl.chunk2;
  const int c0 = blockIdx.x * chunk;
  const int limit = PASS == 1 ? L : n_review;       // keys that matter to this pass
  float *trow = PASS == 2 ? t_out + row * s.t_stride : nullptr;

  if (PASS == 2) {
    const int cend = min(c0 + chunk, s.t_stride);
    if (c0 >= n_review) {
      for (int j = c0 + threadIdx.x; j < cend; j += MF_THREADS) trow[j] = 0.0f;
      return;
    }
    // zero fill of the part of this chunk that lies beyond the review context
    for (int j = max(c0, n_review) + threadIdx.x; j < cend; j += MF_THREADS) trow[j] = 0.0f;
    for (int r = threadIdx.x; r < MT * 16; r += MF_THREADS)
      lse_s[r] = r < s.M ? fold_partials(partials + (row * pl.m_pad + r) * pl.n_chunks1, pl.n_chunks1) : INFINITY;
  }
  stage_q_fragments<D, MT>(s, gp.q[g], b, h, qfrag);
  __syncthreads();

  // per-lane row constants: rows 16*mt + 4*quad + e
  float lse_r[MT][4];
  float mref[MT][4], zsum[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int r = mt * 16 + quad * 4 + e;
      if (PASS == 2) lse_r[mt][e] = lse_s[r];
      mref[mt][e] = -INFINITY;
      zsum[mt][e] = 0.0f;
    }

  const int cend = min(c0 + chunk, limit);
  const uint16_t *kbase = (const uint16_t *)gp.k[g] + (int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh + quad * 8;
  constexpr int STEP = 16 * MF_NT;                    // keys per wave iteration

  for (int j0 = c0 + wave * STEP; j0 < cend; j0 += MF_WAVES * STEP) {
    // ---- load the key fragments of MF_NT tiles (rows clamped into the sequence) ----------
    bf16x8 kf[MF_NT][KS];
#pragma unroll
    for (int n = 0; n < MF_NT; ++n) {
      const int j = min(j0 + n * 16 + col, L - 1);
      const uint16_t *kp = kbase + (int64_t)j * s.kv_st;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kf[n][ks] = *(const bf16x8 *)(kp + ks * 32);
    }
    // ---- logits: acc[n][mt] = Q_mt . K_n^T -------------------------------------------------
    f32x4 acc[MF_NT][MT];
#pragma unroll
    for (int n = 0; n < MF_NT; ++n)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[n][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 araw = qfrag[(mt * KS + ks) * 64 + lane];
        const bf16x8 a = *(const bf16x8 *)&araw;
#pragma unroll
        for (int n = 0; n < MF_NT; ++n)
          acc[n][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, kf[n][ks], acc[n][mt], 0, 0, 0);
      }

    if (PASS == 1) {
      // base-2 logits, masked where the key is beyond the sequence or not visible to the row
      const bool tail = j0 + STEP > n_review;          // wave-uniform
      bool need = false;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float vmax = -INFINITY;
#pragma unroll
          for (int n = 0; n < MF_NT; ++n) {
            float v = acc[n][mt][e] * s.c1;
            if (tail) {   // rare: only the tiles that touch the observation block
              const int j = j0 + n * 16 + col;
              const int r = mt * 16 + quad * 4 + e;
              const int last_vis = r < s.M ? n_review + (r % s.w_obs) : -1;
              if (j > last_vis || j >= cend) v = -INFINITY;
            }
            acc[n][mt][e] = v;
            vmax = fmaxf(vmax, v);
          }
          need |= vmax > mref[mt][e] + MF_RESCALE;
        }
      if (__any(need)) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float vmax = mref[mt][e];
#pragma unroll
            for (int n = 0; n < MF_NT; ++n) vmax = fmaxf(vmax, acc[n][mt][e]);
            if (vmax > mref[mt][e]) {
              zsum[mt][e] *= fast_exp2(mref[mt][e] - vmax);   // mref = -inf gives 0
              mref[mt][e] = vmax;
            }
          }
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int n = 0; n < MF_NT; ++n)
            if (mref[mt][e] != -INFINITY) zsum[mt][e] += fast_exp2(acc[n][mt][e] - mref[mt][e]);
    } else {
      float tsum[MF_NT];
#pragma unroll
      for (int n = 0; n < MF_NT; ++n) {
        float a = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int e = 0; e < 4; ++e) a += fast_exp2(fmaf(acc[n][mt][e], s.c1, -lse_r[mt][e]));
        a += __shfl_xor(a, 16);
        a += __shfl_xor(a, 32);
        tsum[n] = a;
      }
      // quad n writes tile n: 16 consecutive floats per tile
#pragma unroll
      for (int n = 0; n < MF_NT; ++n) {
        const int j = j0 + n * 16 + col;
        if (quad == n && j < cend) trow[j] = tsum[n];
      }
    }
  }

  if (PASS == 1) {
    // merge the 16 key columns of each row (lanes with equal quad), then the 4 waves
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float m = mref[mt][e], z = zsum[mt][e];
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
          const float m2 = __shfl_xor(m, off), z2 = __shfl_xor(z, off);
          merge_stats(m, z, m2, z2);
        }
        if (col == 0) wave_part[wave][mt * 16 + quad * 4 + e] = make_float2(m, z);
      }
    __syncthreads();
    for (int r = threadIdx.x; r < pl.m_pad; r += MF_THREADS) {   // m_pad <= MT*16
      float m = wave_part[0][r].x, z = wave_part[0][r].y;
      for (int w = 1; w < MF_WAVES; ++w) merge_stats(m, z, wave_part[w][r].x, wave_part[w][r].y);
      partials[(row * pl.m_pad + r) * pl.n_chunks1 + blockIdx.x] = make_float2(m, z);
    }
  }
}

// =========================================================================================
// launch
// =========================================================================================
template <int D, int MT>
static hipError_t launch_mfma(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const GroupPtrs &gp,
                              int32_t n_groups, float2 *partials, float *t_out, hipStream_t stream,
                              hipEvent_t mid) {
  dim3 block(MF_THREADS);
  dim3 g1(pl.n_chunks1, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL((score_mfma_kernel<D, MT, 1>), g1, block, 0, stream, s, bp, gp, pl, partials, t_out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
  if (s.t_stride <= 0) return hipSuccess;
  dim3 g2(pl.n_chunks2, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL((score_mfma_kernel<D, MT, 2>), g2, block, 0, stream, s, bp, gp, pl, partials, t_out);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_generic(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const GroupPtrs &gp,
                                 int32_t n_groups, float2 *partials, float *t_out, hipStream_t stream,
                                 hipEvent_t mid) {
  int R = 1;
  while (R < pl.m_pad) R <<= 1;
  dim3 block(GEN_THREADS);
  dim3 g1(pl.n_chunks1, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL((stats_generic_kernel<T, D>), g1, block, 0, stream, s, bp, gp, pl, partials, R);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
  if (s.t_stride <= 0) return hipSuccess;
  const size_t lds = ((size_t)s.M * D + s.M) * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    e = hipFuncSetAttribute((const void *)score_generic_kernel<T, D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (WKV_MAX_OBS_ROWS * D + WKV_MAX_OBS_ROWS) * (int)sizeof(float));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 g2(pl.n_chunks2, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL((score_generic_kernel<T, D>), g2, block, lds, stream, s, bp, gp, pl, partials, t_out);
  return hipGetLastError();
}

hipError_t launch_score(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const GroupPtrs &gp,
                        int32_t n_groups, float2 *partials, float *t_out, hipStream_t stream, hipEvent_t mid) {
  if (pl.mfma) {
    const int mt = pl.m_pad / 16;
#define WKV_MFMA_CASE(DD, MM) \
  if (s.d == DD && mt <= MM) return launch_mfma<DD, MM>(s, bp, pl, gp, n_groups, partials, t_out, stream, mid);
    WKV_MFMA_CASE(128, 1) WKV_MFMA_CASE(128, 2) WKV_MFMA_CASE(128, 4) WKV_MFMA_CASE(128, 8)
    WKV_MFMA_CASE(64, 1) WKV_MFMA_CASE(64, 2) WKV_MFMA_CASE(64, 4) WKV_MFMA_CASE(64, 8)
#undef WKV_MFMA_CASE
    return hipErrorInvalidValue;
  }
  if (s.dtype == WKV_BF16) {
    if (s.d == 128) return launch_generic<uint16_t, 128>(s, bp, pl, gp, n_groups, partials, t_out, stream, mid);
    return launch_generic<uint16_t, 64>(s, bp, pl, gp, n_groups, partials, t_out, stream, mid);
  }
  if (s.d == 128) return launch_generic<float, 128>(s, bp, pl, gp, n_groups, partials, t_out, stream, mid);
  return launch_generic<float, 64>(s, bp, pl, gp, n_groups, partials, t_out, stream, mid);
}

}  // namespace wkv
