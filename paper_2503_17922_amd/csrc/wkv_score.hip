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
//   fold            one tiny launch turns the partials of every row into lse2_i = m_i + log2(z_i).
//   pass 2 (score)  each workgroup recomputes its logits and writes t_j = sum_i 2^(v_ij - lse2_i).
//
// A caller whose prefill attention kept the normalisers of the observation rows hands them
// over; pass 1 and the fold are then skipped and the keys are read once.
//
// Two kernel families implement the passes:
//   * MFMA (bf16 or fp16 inputs): v_mfma_f32_16x16x32_bf16 / _f16 with the keys as the A operand,
//     loaded straight from global memory into registers in operand layout, so K never passes
//     through LDS and the four waves of a workgroup never synchronise in the loop; the
//     query rows are the B operand, read as pre-arranged fragments from LDS.
//   * generic (fp32 inputs): plain fp32 FMAs, thread-per-row for the stats,
//     thread-per-key for the scores, the other operand broadcast from LDS.
#include "wkv_device.h"
#include "wkv_pool.h"

namespace wkv {

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const void *p, int64_t i) { return ((const float *)p)[i]; }
};

// =========================================================================================
// fold: per-chunk (m, z) partials of pass 1 -> one lse2 per row, once per (group, sequence, KV head)
// =========================================================================================
constexpr int FOLD_THREADS = 256;

__global__ __launch_bounds__(FOLD_THREADS) void fold_kernel(Shape s, ScorePlan pl, const float2 *__restrict__ partials,
                                                            float *__restrict__ lse, const uint32_t *__restrict__ only_if) {
  __shared__ float2 part_s[FOLD_THREADS];
  if (only_if && *only_if == 0u) return;
  const int64_t row = (int64_t)blockIdx.y * s.B * s.Hkv + blockIdx.x;
  // TPR threads share a row; rows are handled in passes of FOLD_THREADS / TPR
  const int TPR = pl.m_pad >= 128 ? 2 : (pl.m_pad >= 64 ? 4 : 8);
  const int rows_per_pass = FOLD_THREADS / TPR;
  for (int r0 = 0; r0 < pl.m_pad; r0 += rows_per_pass) {
    const int r = r0 + threadIdx.x % rows_per_pass, part_id = threadIdx.x / rows_per_pass;
    float m = -INFINITY, z = 0.0f;
    if (r < s.M)
      fold_partials_strided(partials + (row * pl.m_pad + r) * pl.n_chunks1, pl.n_chunks1, part_id, TPR, m, z);
    __syncthreads();
    part_s[threadIdx.x] = make_float2(m, z);
    __syncthreads();
    if (part_id == 0 && r < pl.m_pad) {
      for (int i = 1; i < TPR; ++i) merge_stats(m, z, part_s[i * rows_per_pass + threadIdx.x].x, part_s[i * rows_per_pass + threadIdx.x].y);
      lse[row * pl.m_pad + r] = r < s.M ? m + fast_log2(z) : INFINITY;   // padded rows: 2^-inf = 0
    }
  }
}

// The base-2 log-sum-exp of softmax row r of (group g, sequence b, KV head h): converted from the
// caller's natural-log normalisers [B, Hq, w_obs] when they were handed over (the rows of a KV
// head are contiguous there), else what the fold left in the workspace.  Padded rows get +inf
// (2^-inf = 0: they contribute nothing).
__device__ __forceinline__ float row_lse2(const Shape &s, const ScorePlan &pl, const GroupPtrs &gp,
                                          const float *__restrict__ lse_ws, int g, int b, int h, int64_t row, int r) {
  if (r >= s.M) return INFINITY;
  const float *given = gp.lse[g];
  if (given) return given[((int64_t)b * s.Hq + (int64_t)h * s.G) * s.w_obs + r] * 1.4426950408889634f;
  return lse_ws[row * pl.m_pad + r];
}

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
                                                                    const float *__restrict__ lse_g,
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
  for (int r = threadIdx.x; r < s.M; r += GEN_THREADS) lse[r] = row_lse2(s, pl, gp, lse_g, g, b, h, row, r);
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
// Orientation: D[key, query row] = sum_c K[key, c] * Q[row, c].  The keys are the A operand (16
// keys x 32 channels per instruction, loaded straight from global memory: lane l holds key
// l%16, the 16-byte piece l/16 of a 64-byte run, so the four lanes of a key read 64 contiguous
// bytes), the stacked query rows are the B operand (fragments pre-arranged in LDS, one
// conflict-free ds_read_b128 each).  In the 16x16 result a lane holds 4 consecutive keys of
// ONE query row per row tile, so a lane needs only MT row constants (reference / lse2), the
// row statistics of pass 1 are in-lane accumulations merged once per chunk, and the column
// sums of pass 2 are in-lane adds over the row tiles plus one 16-lane DPP reduction.
// PASS 1: stats.  PASS 2: scores.
//
// Up to 128 rows (HV = 1) a workgroup is 4 waves that take different key tiles of an iteration
// and all MT row tiles each; three workgroups share a CU.  With 129..256 rows (HV = 2: eight
// query heads per KV head at 32 observation queries) a workgroup is 8 waves: waves 0-3 work on
// row tiles 0..MT-1 and waves 4-7 on row tiles MT..2MT-1 of the same key tiles (the second
// read of a key tile hits the CU's vector cache), the 64 KB of query fragments allow one
// workgroup per CU, and pass 2 adds the column sums of the two halves in its epilogue.
template <int D, int MT, int HV, int PASS, bool F16>
__global__ __launch_bounds__(MF_THREADS * HV, HV == 1 ? 3 : 2) void score_mfma_kernel(Shape s, BatchParams bp, GroupPtrs gp,
                                                                   ScorePlan pl, float2 *__restrict__ partials,
                                                                   const float *__restrict__ lse_g,
                                                                   float *__restrict__ t_out,
                                                                   float *__restrict__ s_pool,
                                                                   const uint32_t *__restrict__ only_if) {
  constexpr int KS = D / 32;
  constexpr int STEP = 16 * MF_KT;                    // keys per wave iteration
  constexpr int NT = MF_THREADS * HV;                 // threads of the workgroup
  // Launched behind the single-read kernel as its fall-back: nothing to do unless that kernel
  // raised the word (uniform over the grid).
  if (only_if && *only_if == 0u) return;
  constexpr int MTT = MT * HV;                        // row tiles of the workgroup
  constexpr int TS_LEN = MAX_CHUNK2 + 256;            // token scores of a chunk + the scrap area
  __shared__ uint4 qfrag[MTT * KS * 64];
  __shared__ float2 wave_part[PASS == 1 ? MF_WAVES * HV : 1][MT * 16];
  // Pass 2 collects the chunk's token scores here and writes them out once at the end: global
  // stores inside the loop would share the vector-memory counter with the key prefetch and make
  // every wait for keys also wait for store acknowledgements.
  __shared__ __attribute__((aligned(16))) float t_s[PASS == 2 ? HV * TS_LEN : 1];
  __shared__ float lse_s[PASS == 2 ? MTT * 16 : 1];

  // Pass 2 walks the work items in the opposite order of pass 1: the keys pass 1 read last
  // are the ones most likely still held by the memory-side cache.
  const int bx = PASS == 1 ? blockIdx.x : gridDim.x - 1 - blockIdx.x;
  const int bh = PASS == 1 ? blockIdx.y : gridDim.y - 1 - blockIdx.y;
  const int g = PASS == 1 ? blockIdx.z : gridDim.z - 1 - blockIdx.z;
  const int h = bh % s.Hkv;
  const int b = PASS == 1 ? bp.by_length[bh / s.Hkv] : bh / s.Hkv;      // statistics: short sequences first
  const int L = bp.seq[b].L;
  const int n_review = L - s.w_obs;
  const int64_t row = ((int64_t)g * s.B + b) * s.Hkv + h;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int half = wave / MF_WAVES, kw = wave % MF_WAVES;   // row half, key tile slot of this wave
  const int col = lane & 15, quad = lane >> 4;

  const int chunk = PASS == 1 ? pl.chunk1 : pl.chunk2;
  const int c0 = bx * chunk;
  const int limit = PASS == 1 ? L : n_review;         // keys that matter to this pass
  float *trow = PASS == 2 ? t_out + row * s.t_stride : nullptr;

  if (PASS == 2) {
    const int cend_fill = min(c0 + chunk, s.t_stride);
    if (c0 >= n_review) {
      if (!s_pool)
        for (int j = c0 + threadIdx.x; j < cend_fill; j += NT) trow[j] = 0.0f;
      return;
    }
  }
  if (PASS == 1 && c0 >= L) {                         // a chunk past the end of a short sequence
    for (int r = threadIdx.x; r < pl.m_pad; r += NT)
      partials[(row * pl.m_pad + r) * pl.n_chunks1 + bx] = make_float2(-INFINITY, 0.0f);
    return;
  }
  // Loads that depend on nothing staged below go out first, so that their latencies overlap: the
  // query fragments of this workgroup and the first key tile of every wave.
  QStage<D, MTT, NT> qstage;
  qstage.load(s, gp.q[g], b, h);
  const int cend = min(c0 + chunk, limit);
  const uint16_t *kbase = (const uint16_t *)gp.k[g] + (int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh + quad * 8;
  int j0 = c0 + kw * STEP;
  KFrags<KS> ka, kb;
  load_k<KS>(ka, kbase, s.kv_st, j0, col, max(cend, 1));

  if (PASS == 2) {
    // The base-2 log-sum-exp of the MT*16 rows, into LDS.  With few chunks per row the workgroup
    // folds the (m, z) partials of pass 1 itself (TPR adjacent lanes share a row; the query
    // and key loads issued above are in flight meanwhile); otherwise a fold launch or the caller provided them.
    constexpr int TPR = NT / (MTT * 16);
    const int r = threadIdx.x / TPR, part = threadIdx.x % TPR;
    if (pl.fold_in_pass2) {
      float m = -INFINITY, z = 0.0f;
      if (r < s.M) fold_partials_strided(partials + (row * pl.m_pad + r) * pl.n_chunks1, pl.n_chunks1, part, TPR, m, z);
#pragma unroll
      for (int off = 1; off < TPR; off <<= 1) {
        const float m2 = __shfl_xor(m, off), z2 = __shfl_xor(z, off);
        merge_stats(m, z, m2, z2);
      }
      if (part == 0) lse_s[r] = r < s.M ? m + fast_log2(z) : INFINITY;      // padded rows: 2^-inf = 0
    } else if (part == 0) {
      lse_s[r] = row_lse2(s, pl, gp, lse_g, g, b, h, row, r);
    }
  }
  qstage.store(qfrag);
  __syncthreads();

  // per-lane row constants: this lane's query row of its row tile mt is 16*(half*MT + mt) + col
  float lse_r[MT], mref[MT], zsum[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    lse_r[mt] = PASS == 2 ? lse_s[(half * MT + mt) * 16 + col] : 0.0f;
    mref[mt] = -INFINITY;
    zsum[mt] = 0.0f;
  }

  const float c1 = s.c1;

  // One wave iteration: prefetch the keys of the next iteration into `kn`, compute on `kf`.
  // The loop below calls it with the two buffers swapped in turn, so no register copies are
  // needed and the wait for a buffer sits a whole iteration after its loads were issued.
  auto iteration = [&](const KFrags<KS> &kf, KFrags<KS> &kn, const int j0) __attribute__((always_inline)) {
    // The query fragments are loop invariant; without this barrier the compiler hoists all of
    // them into registers (128 VGPRs) and spills.  They are meant to be re-read from LDS.
    asm volatile("" ::: "memory");
    // ---- prefetch the next iteration's keys while this one is computed --------------------
    // Unconditional: a prefetch behind a branch makes every wait for `kf` also wait for it.
    // Past the end of the chunk the row index clamps to the chunk's last key (a cache hit).
    load_k<KS>(kn, kbase, s.kv_st, j0 + MF_WAVES * STEP, col, cend);

    // ---- logits acc[n][mt][e] = k_{j0+16n+4*quad+e} . q_{16*mt+col}, and their exponentials --------
    // Written so that the MFMAs of row tile mt and the exponentials of row tile mt-1 alternate
    // in ONE basic block: the matrix pipe and the vector ALU then overlap inside a wave instead
    // of taking turns (the rare paths - mask, re-reference - come after the block).
    f32x4 acc[MF_KT][MT];
    float psum[MT];                                     // pass 1: sum of the tile's terms per row
    f32x4 tq[MF_KT];                                    // pass 2: column sums over this lane's rows
#pragma unroll
    for (int n = 0; n < MF_KT; ++n) tq[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt <= MT; ++mt) {
      if (mt < MT) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const uint4 qraw = qfrag[((half * MT + mt) * KS + ks) * 64 + lane];
          const bf16x8 qb = *(const bf16x8 *)&qraw;
#pragma unroll
          for (int n = 0; n < MF_KT; ++n)
            acc[n][mt] = mfma_16x16x32<F16>(kf.f[n][ks], qb, ks == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[n][mt]);
        }
      }
      if (mt > 0) {
        const int m1 = mt - 1;
        if (PASS == 1) {
          float a = 0.0f;
#pragma unroll
          for (int n = 0; n < MF_KT; ++n)
#pragma unroll
            for (int e = 0; e < 4; ++e) a += fast_exp2(fmaf(acc[n][m1][e], c1, -mref[m1]));
          psum[m1] = a;
        } else {
#pragma unroll
          for (int n = 0; n < MF_KT; ++n)
#pragma unroll
            for (int e = 0; e < 4; ++e) tq[n][e] += fast_exp2(fmaf(acc[n][m1][e], c1, -lse_r[m1]));
        }
      }
    }

    if (PASS == 1) {
      if (j0 + STEP > n_review) {
        // tiles that touch the observation block: causal mask (key j visible to observation
        // query io iff j <= n_review + io) and the end of the sequence; redo their sums
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int r = (half * MT + mt) * 16 + col;
          const int last_vis = r < s.M ? n_review + (r % s.w_obs) : -1;
          float a = 0.0f;
#pragma unroll
          for (int n = 0; n < MF_KT; ++n)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int j = j0 + n * 16 + quad * 4 + e;
              if (j > last_vis || j >= cend) acc[n][mt][e] = -INFINITY;
              a += fast_exp2(fmaf(acc[n][mt][e], c1, -mref[mt]));
            }
          psum[mt] = a;
        }
      }
      // A sum that is huge, infinite or NaN (first tile: mref = -inf) means a logit far above the
      // row's reference: re-reference the row and redo its part of the tile.
      bool redo = false;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) redo |= !(psum[mt] <= MF_BIG);
      if (__any(redo)) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (!(psum[mt] <= MF_BIG)) {
            float vmax = -INFINITY;
#pragma unroll
            for (int n = 0; n < MF_KT; ++n)
#pragma unroll
              for (int e = 0; e < 4; ++e) vmax = fmaxf(vmax, acc[n][mt][e]);
            const float nref = fmaxf(mref[mt], vmax * c1);
            float a = 0.0f;
            if (nref != -INFINITY) {
              zsum[mt] *= fast_exp2(mref[mt] - nref);      // mref = -inf: 2^-inf = 0 and zsum is 0
              mref[mt] = nref;
#pragma unroll
              for (int n = 0; n < MF_KT; ++n)
#pragma unroll
                for (int e = 0; e < 4; ++e) a += fast_exp2(fmaf(acc[n][mt][e], c1, -nref));
            }
            psum[mt] = a;
          }
        }
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) zsum[mt] += psum[mt];
    } else {
      // t_j: the lane's partial column sums, summed over the 16 lanes (rows 16*mt + 0..15)
      // Every lane stores (lanes other than the first of each 16 into a scrap area past the
      // chunk): a store under a lane predicate would put a branch into the middle of the block.
      float *ts = t_s + half * TS_LEN;
      float *dst = col == 0 ? ts + (j0 - c0) + quad * 4 : ts + MAX_CHUNK2 + lane * 4;
#pragma unroll
      for (int n = 0; n < MF_KT; ++n) {
#pragma unroll
        for (int e = 0; e < 4; ++e) tq[n][e] = row16_sum(tq[n][e]);
        *(f32x4 *)(dst + (col == 0 ? n * 16 : 0)) = tq[n];                // 4 consecutive keys per quad
      }
    }
  };

  while (j0 < cend) {
    iteration(ka, kb, j0);
    j0 += MF_WAVES * STEP;
    if (j0 >= cend) break;
    iteration(kb, ka, j0);
    j0 += MF_WAVES * STEP;
  }

  if (PASS == 2) {
    __syncthreads();
    if (HV == 2) {                                    // column sums of the second half of the rows
      for (int j = threadIdx.x; j < cend - c0; j += NT) t_s[j] += t_s[TS_LEN + j];
      __syncthreads();
    }
    if (s_pool) {
      // Eq. 3-4 on the chunk's token scores while they are in LDS: the chunk starts on a window
      // boundary and no window but the sequence's last (partial) one ends outside it
      const SeqParam sp = bp.seq[b];
      const int w0 = c0 / sp.win, w1 = (cend + sp.win - 1) / sp.win;
      float *srow = s_pool + row * s.nw_max;
      for (int w = w0 + threadIdx.x; w < w1; w += NT)
        srow[w] = pool_window(t_s - c0, w, sp.win, n_review, sp.p);
    } else {
      const int cend_fill = min(c0 + chunk, s.t_stride);
      for (int j = c0 + threadIdx.x; j < cend_fill; j += NT) trow[j] = j < cend ? t_s[j - c0] : 0.0f;
    }
  }
  if (PASS == 1) {
    // merge the 4 quads of each row (lanes col, col+16, col+32, col+48), then the 4 waves
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float m = mref[mt], z = zsum[mt];
#pragma unroll
      for (int off = 16; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m, off), z2 = __shfl_xor(z, off);
        merge_stats(m, z, m2, z2);
      }
      if (quad == 0) wave_part[wave][mt * 16 + col] = make_float2(m, z);
    }
    __syncthreads();
    for (int r = threadIdx.x; r < pl.m_pad; r += NT) {           // m_pad <= MTT*16
      const int w0 = r / (MT * 16) * MF_WAVES, rr = r % (MT * 16);   // the waves that hold row r
      float m = wave_part[w0][rr].x, z = wave_part[w0][rr].y;
      for (int w = 1; w < MF_WAVES; ++w) merge_stats(m, z, wave_part[w0 + w][rr].x, wave_part[w0 + w][rr].y);
      partials[(row * pl.m_pad + r) * pl.n_chunks1 + bx] = make_float2(m, z);
    }
  }
}

// =========================================================================================
// launch
// =========================================================================================
template <int D, int MT, int HV, bool F16>
static hipError_t launch_mfma(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const GroupPtrs &gp,
                              int32_t n_groups, bool have_lse, float2 *partials, float *lse, float *t_out,
                              float *s_pool, hipStream_t stream, hipEvent_t mid, const uint32_t *only_if) {
  dim3 block(MF_THREADS * HV);
  hipError_t e;
  if (have_lse) {                                      // no statistics pass: pass 2 reads the caller's normalisers
    if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
    if (s.t_stride <= 0) return hipSuccess;
  } else {
    dim3 g1(pl.n_chunks1, s.B * s.Hkv, n_groups);
    hipLaunchKernelGGL((score_mfma_kernel<D, MT, HV, 1, F16>), g1, block, 0, stream, s, bp, gp, pl, partials, lse, t_out, s_pool, only_if);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
    if (s.t_stride <= 0) return hipSuccess;
    if (!pl.fold_in_pass2) {
      hipLaunchKernelGGL(fold_kernel, dim3(s.B * s.Hkv, n_groups), dim3(FOLD_THREADS), 0, stream, s, pl, partials, lse, only_if);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  ScorePlan pl2 = pl;
  if (have_lse) pl2.fold_in_pass2 = false;
  dim3 g2(pl.n_chunks2, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL((score_mfma_kernel<D, MT, HV, 2, F16>), g2, block, 0, stream, s, bp, gp, pl2, partials, lse, t_out, s_pool, only_if);
  return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_generic(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const GroupPtrs &gp,
                                 int32_t n_groups, bool have_lse, float2 *partials, float *lse, float *t_out,
                                 hipStream_t stream, hipEvent_t mid) {
  int R = 1;
  while (R < pl.m_pad) R <<= 1;
  dim3 block(GEN_THREADS);
  hipError_t e;
  if (have_lse) {                                      // no statistics pass: pass 2 reads the caller's normalisers
    if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
    if (s.t_stride <= 0) return hipSuccess;
  } else {
    dim3 g1(pl.n_chunks1, s.B * s.Hkv, n_groups);
    hipLaunchKernelGGL((stats_generic_kernel<T, D>), g1, block, 0, stream, s, bp, gp, pl, partials, R);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
    if (s.t_stride <= 0) return hipSuccess;
    hipLaunchKernelGGL(fold_kernel, dim3(s.B * s.Hkv, n_groups), dim3(FOLD_THREADS), 0, stream, s, pl, partials, lse, (const uint32_t *)nullptr);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  const size_t lds = ((size_t)s.M * D + s.M) * sizeof(float);
  if (lds > 48 * 1024) {     // beyond the default dynamic-LDS limit: raise it (per device, any thread)
    e = hipFuncSetAttribute((const void *)score_generic_kernel<T, D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (WKV_MAX_OBS_ROWS * D + WKV_MAX_OBS_ROWS) * (int)sizeof(float));
    if (e != hipSuccess) return e;
  }
  dim3 g2(pl.n_chunks2, s.B * s.Hkv, n_groups);
  hipLaunchKernelGGL((score_generic_kernel<T, D>), g2, block, lds, stream, s, bp, gp, pl, lse, t_out);
  return hipGetLastError();
}

hipError_t launch_score(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const GroupPtrs &gp,
                        int32_t n_groups, bool have_lse, float2 *partials, float *lse, float *t_out, float *s_pool,
                        hipStream_t stream, hipEvent_t mid, const uint32_t *only_if) {
  if (pl.mfma) {
    const int mt = pl.m_pad / 16;
    const bool f16 = s.dtype == WKV_F16;
#define WKV_MFMA_CASE(DD, MM, HH)                                                                              \
  if (s.d == DD && mt <= MM * HH)                                                                              \
    return f16 ? launch_mfma<DD, MM, HH, true>(s, bp, pl, gp, n_groups, have_lse, partials, lse, t_out, s_pool, stream, mid, only_if) \
               : launch_mfma<DD, MM, HH, false>(s, bp, pl, gp, n_groups, have_lse, partials, lse, t_out, s_pool, stream, mid, only_if);
    WKV_MFMA_CASE(128, 1, 1) WKV_MFMA_CASE(128, 2, 1) WKV_MFMA_CASE(128, 4, 1) WKV_MFMA_CASE(128, 8, 1)
    WKV_MFMA_CASE(64, 1, 1) WKV_MFMA_CASE(64, 2, 1) WKV_MFMA_CASE(64, 4, 1) WKV_MFMA_CASE(64, 8, 1)
    WKV_MFMA_CASE(128, 8, 2) WKV_MFMA_CASE(64, 8, 2)      // 129..256 rows: two halves of 8 row tiles
#undef WKV_MFMA_CASE
    return hipErrorInvalidValue;
  }
  if (s.d == 128) return launch_generic<float, 128>(s, bp, pl, gp, n_groups, have_lse, partials, lse, t_out, stream, mid);
  return launch_generic<float, 64>(s, bp, pl, gp, n_groups, have_lse, partials, lse, t_out, stream, mid);
}

}  // namespace wkv
