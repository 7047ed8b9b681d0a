// Observation-window token scores (WindowKV Eq. 1-2) with ONE read of the keys.
//
// The normaliser of a softmax row needs every key of the prefix before any column sum can be
// finished, so the two-pass kernels stream the keys of the scored layer twice.  Here a slice
// of keys stays on chip between the statistics phase and the score phase instead:
//
//   * a persistent grid (as many workgroups as fit on the device at once) walks over the slices
//     of all (group, sequence, KV head) rows in row order; a slice is RK_SLICE consecutive keys
//     and lives in the registers of one workgroup, in MFMA operand layout, for both phases;
//   * phase 1: logits of the slice against the stacked query rows (MFMA), running maximum and
//     sum per row; the slice's (m, z) partials are written to the workspace and the workgroup
//     counts itself in at the row's arrival counter;
//   * the workgroup that arrives last folds all partials of the row into one base-2
//     log-sum-exp per softmax row (in slice order: the result does not depend on who arrived
//     when), publishes them and raises the row's ready word;
//   * phase 2: once the row is ready, the logits are recomputed from the resident keys and
//     t_j = sum_i 2^(v_ij - lse2_i) goes out (or, pooled, the window scores of Eq. 3-4).
//
// What workgroups exchange travels in device-scope relaxed atomics (stores, loads, one add per
// slice); a wait for the stores' acknowledgement orders them, no cache is written back or
// invalidated.  Phase 1 never waits, and a workgroup only waits for slices that belong to
// workgroups which have finished everything before them, so with the whole grid resident the
// earliest unfinished row always completes.  Every wait is bounded all the same: when it runs
// out the workgroup raises the `fail` word and carries on without waiting any more, every wave
// exits, and the two-pass kernels (enqueued right behind, returning at once otherwise)
// recompute everything.
#include <atomic>
#include <type_traits>

#include "wkv_device.h"
#include "wkv_pool.h"

namespace wkv {

static_assert(RK_SLICE == 2 * MF_WAVES * 16 * MF_KT, "a slice is two tile pairs per wave");

__device__ __forceinline__ void store_agent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(unsigned long long *p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_agent(const unsigned long long *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t load_agent(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All vector-memory operations of this wave issued so far have been acknowledged.
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

#ifdef WKV_RK_TIMING
// Debug build only: per-workgroup wall-clock (10 ns ticks) spent in each part of a slice.
__device__ unsigned long long rk_timing[1024][8];
#define RK_T(i) do { if (tid == 0) { const unsigned long long now_ = wall_clock64(); rk_timing[blockIdx.x][i] += now_ - tprev_; tprev_ = now_; } } while (0)
#else
#define RK_T(i) do { } while (0)
#endif

__global__ __launch_bounds__(256) void resident_clear_kernel(uint32_t *sync_words, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) sync_words[i] = 0u;
}

template <int D, int MT, bool F16>
__global__ __launch_bounds__(MF_THREADS, 3) void score_resident_kernel(Shape s, BatchParams bp, GroupPtrs gp, ResidentPlan rp,
                                                                      unsigned long long *__restrict__ partials,
                                                                      float *__restrict__ lse_g, uint32_t *__restrict__ sync,
                                                                      float *__restrict__ t_out, float *__restrict__ s_pool) {
  constexpr int KS = D / 32;
  constexpr int STEP = 16 * MF_KT;                    // keys per wave iteration
  constexpr int NT = MF_THREADS;
  constexpr int ROWS = MT * 16;
  __shared__ uint4 qfrag[MT * KS * 64];
  __shared__ float2 wave_part[MF_WAVES][ROWS];
  __shared__ __attribute__((aligned(16))) float t_s[RK_SLICE + 256];     // the slice's token scores + a scrap area
  __shared__ float lse_s[ROWS];
  __shared__ int last_s, ok_s;

  const float c1 = s.c1;
  uint32_t *fail = sync + RK_FAIL;
  bool gave_up = false;                                // uniform: once set, this workgroup waits no more

  for (int item = blockIdx.x; item < rp.n_items; item += gridDim.x) {
    // The thread's own indices are re-derived for every slice from a value the compiler cannot see
    // through: hoisted out of this loop, the dozens of per-thread constants that follow from them
    // (addresses, masks) would occupy registers for the whole kernel and push the tile loops into
    // spilling.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 15, quad = lane >> 4;
#ifdef WKV_RK_TIMING
    unsigned long long tprev_ = wall_clock64();
#endif
    // ---- which slice ----------------------------------------------------------------------
    // (slices are numbered group by group, inside a group sequence by sequence, then KV head, then position)
    const int g = item / rp.items_per_group;
    const int rem = item - g * rp.items_per_group;
    int b = 0, first = 0;
    for (;; ++b) {
      const int n = (bp.seq[b].L + RK_SLICE - 1) / RK_SLICE * s.Hkv;
      if (rem < first + n || b == s.B - 1) break;
      first += n;
    }
    const int L = bp.seq[b].L;
    const int n_review = L - s.w_obs;
    const int nsl = (L + RK_SLICE - 1) / RK_SLICE;
    const int within = rem - first;
    const int h = within / nsl, sl = within - h * nsl;
    const int64_t row = ((int64_t)g * s.B + b) * s.Hkv + h;
    const int c0 = sl * RK_SLICE;
    const int cend = min(c0 + RK_SLICE, L);            // keys of this slice (phase 1)
    const int cend2 = min(c0 + RK_SLICE, n_review);    // keys that get a score (phase 2)
    uint32_t *row_sync = sync + RK_GLOBAL_WORDS + RK_SYNC_WORDS * row;

    __syncthreads();                                   // the previous slice's readers of qfrag / t_s / lse_s are done
    QStage<D, MT, NT> qstage;
    qstage.load(s, gp.q[g], b, h, tid);
    const uint16_t *kbase = (const uint16_t *)gp.k[g] + (int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh + quad * 8;
    const int ja = c0 + wave * STEP, jb = ja + MF_WAVES * STEP;
    KFrags<KS> ka, kb;                                 // resident for both phases
    load_k<KS>(ka, kbase, s.kv_st, ja, col, cend);
    load_k<KS>(kb, kbase, s.kv_st, jb, col, cend);
    qstage.store(qfrag, tid);
    __syncthreads();
    RK_T(0);

    float mref[MT], zsum[MT], lse_r[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) { mref[mt] = -INFINITY; zsum[mt] = 0.0f; lse_r[mt] = 0.0f; }

    // One tile pair (2 x 16 keys) against all row tiles.  PASS 1 accumulates the row statistics,
    // PASS 2 writes the column sums into t_s.  The MFMAs of row tile mt and the exponentials of
    // row tile mt-1 alternate in one basic block, so that the matrix pipe and the vector ALU
    // overlap inside a wave (see the two-pass kernel, which has the same body).
    auto tile_pair = [&](auto pass_tag, const KFrags<KS> &kf, const int j0) __attribute__((always_inline)) {
      constexpr int PASS = decltype(pass_tag)::value;
      asm volatile("" ::: "memory");                   // keep the query fragments in LDS (see the two-pass kernel)
      f32x4 acc[MF_KT][MT];
      float psum[MT];
      f32x4 tq[MF_KT];
#pragma unroll
      for (int n = 0; n < MF_KT; ++n) tq[n] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int mt = 0; mt <= MT; ++mt) {
        if (mt < MT) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            const uint4 qraw = qfrag[(mt * KS + ks) * 64 + lane];
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
        if (j0 + STEP > n_review) {                    // causal mask of the observation block, end of the sequence
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const int r = mt * 16 + col;
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
        bool redo = false;                             // a huge, infinite or NaN sum: re-reference the row
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
                zsum[mt] *= fast_exp2(mref[mt] - nref);
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
        float *dst = col == 0 ? t_s + (j0 - c0) + quad * 4 : t_s + RK_SLICE + lane * 4;
#pragma unroll
        for (int n = 0; n < MF_KT; ++n) {
#pragma unroll
          for (int e = 0; e < 4; ++e) tq[n][e] = row16_sum(tq[n][e]);
          *(f32x4 *)(dst + (col == 0 ? n * 16 : 0)) = tq[n];
        }
      }
    };

    // ---- phase 1: the slice's row statistics ---------------------------------------------------
    if (ja < cend) tile_pair(std::integral_constant<int, 1>{}, ka, ja);
    if (jb < cend) tile_pair(std::integral_constant<int, 1>{}, kb, jb);
    RK_T(1);
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
    if (tid < rp.m_pad) {
      const int r = tid;
      float m = wave_part[0][r].x, z = wave_part[0][r].y;
      for (int w = 1; w < MF_WAVES; ++w) merge_stats(m, z, wave_part[w][r].x, wave_part[w][r].y);
      const unsigned long long bits = ((unsigned long long)__float_as_uint(z) << 32) | __float_as_uint(m);
      store_agent(partials + ((row * rp.nsl_max + sl) * rp.m_pad + r), bits);
    }
    wait_vmem();                                       // the partials are out before the arrival is counted
    __syncthreads();
    if (tid == 0)
      last_s = __hip_atomic_fetch_add(row_sync + RK_ARRIVED, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)(nsl - 1);
    __syncthreads();
    const bool last = last_s != 0;
    RK_T(2);
    if (!s_pool && sl == 0 && n_review <= 0) {          // no review context at all: the row of token scores is all padding
      float *trow = t_out + row * s.t_stride;
      for (int j = tid; j < s.t_stride; j += NT) trow[j] = 0.0f;
    }
    if (c0 >= n_review && !last) continue;             // a slice inside the observation block has nothing to score

    if (last) {
      // ---- fold the row: TPR = 2 threads per softmax row, slices part, part + 2, ... in order -------
      const int r = tid >> 1, part = tid & 1;
      float m = -INFINITY, z = 0.0f;
      if (r < rp.m_pad) {
        const unsigned long long *p = partials + (row * rp.nsl_max * rp.m_pad + r);
        for (int s0 = part; s0 < nsl; s0 += 32) {      // 16 loads in flight
          unsigned long long v[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int ss = s0 + 2 * i;
            v[i] = ss < nsl ? load_agent(p + (int64_t)ss * rp.m_pad) : 0xff800000ull;    // (m = -inf, z = 0)
          }
#pragma unroll
          for (int i = 0; i < 16; ++i) merge_stats(m, z, __uint_as_float((uint32_t)v[i]), __uint_as_float((uint32_t)(v[i] >> 32)));
        }
      }
      const float m2 = __shfl_xor(m, 1), z2 = __shfl_xor(z, 1);
      merge_stats(m, z, m2, z2);                       // even slices with odd slices
      if (part == 0 && r < rp.m_pad) {
        const float l2 = r < s.M ? m + fast_log2(z) : INFINITY;      // padded rows: 2^-inf = 0
        lse_s[r] = l2;
        store_agent(lse_g + row * rp.m_pad + r, l2);
      }
      wait_vmem();
      __syncthreads();
      if (tid == 0) __hip_atomic_store(row_sync + RK_READY, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      RK_T(3);
      if (c0 >= n_review) continue;
    } else {
      // ---- wait (bounded) for the row's normalisers -------------------------------------------------
      if (tid == 0) {
        int ok = 1;
        if (!gave_up) {
          int spins = 0;
          while (load_agent(row_sync + RK_READY) == 0u) {
            if (++spins > rp.spin_limit || load_agent(fail) != 0u) {
              __hip_atomic_store(fail, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              ok = 0;
              break;
            }
            __builtin_amdgcn_s_sleep(8);
          }
        } else {
          ok = 0;
        }
        ok_s = ok;
      }
      __syncthreads();
      if (ok_s == 0) gave_up = true;                 // results of this launch are void; never wait again
      if (tid < rp.m_pad) lse_s[tid] = gave_up ? INFINITY : load_agent(lse_g + row * rp.m_pad + tid);
      __syncthreads();
      RK_T(4);
    }

    // ---- phase 2: scores from the resident keys ----------------------------------------------------------
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) lse_r[mt] = lse_s[mt * 16 + col];
    if (ja < cend2) tile_pair(std::integral_constant<int, 2>{}, ka, ja);
    if (jb < cend2) tile_pair(std::integral_constant<int, 2>{}, kb, jb);
    __syncthreads();
    RK_T(5);
    if (s_pool) {
      // Eq. 3-4 on the slice's token scores while they are in LDS: the slice starts on a window
      // boundary and no window but the sequence's last (partial) one ends outside it
      const SeqParam sp = bp.seq[b];
      const int w0 = c0 / sp.win, w1 = (cend2 + sp.win - 1) / sp.win;
      float *srow = s_pool + row * s.nw_max;
      for (int w = w0 + tid; w < w1; w += NT) srow[w] = pool_window(t_s - c0, w, sp.win, n_review, sp.p);
    } else {
      float *trow = t_out + row * s.t_stride;
      const int cfill = c0 + RK_SLICE >= n_review ? s.t_stride : c0 + RK_SLICE;   // the row's padding is zeroed by its last scoring slice
      for (int j = c0 + tid; j < cfill; j += NT) trow[j] = j < cend2 ? t_s[j - c0] : 0.0f;
    }
    RK_T(6);
  }
}

#ifdef WKV_RK_TIMING
extern "C" int wkv_debug_rk_timing(unsigned long long *host_out /* [1024][8] */, int clear) {
  hipError_t e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipMemcpyFromSymbol(host_out, HIP_SYMBOL(rk_timing), sizeof(rk_timing));
  static const unsigned long long zeros[1024][8] = {};
  if (e == hipSuccess && clear) e = hipMemcpyToSymbol(HIP_SYMBOL(rk_timing), zeros, sizeof(zeros));
  return (int)e;
}
#endif

template <int D, int MT, bool F16>
static hipError_t launch_resident_t(const Shape &s, const BatchParams &bp, const ResidentPlan &rp, const GroupPtrs &gp,
                                    unsigned long long *partials, float *lse, uint32_t *sync, float *t_out, float *s_pool,
                                    hipStream_t stream) {
  // as many workgroups as the device holds at once (asked once; the answer depends on the kernel only)
  static std::atomic<int> resident_wgs{0};
  int n_wg = resident_wgs.load(std::memory_order_relaxed);
  if (n_wg == 0) {
    int dev = 0, cus = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, score_resident_kernel<D, MT, F16>, MF_THREADS, 0);
    if (e != hipSuccess) return e;
    n_wg = cus * (per_cu < 3 ? per_cu : 3);
    if (n_wg <= 0) return hipErrorLaunchFailure;
    resident_wgs.store(n_wg, std::memory_order_relaxed);
  }
  if (n_wg > rp.n_items) n_wg = rp.n_items;
  hipLaunchKernelGGL((score_resident_kernel<D, MT, F16>), dim3(n_wg), dim3(MF_THREADS), 0, stream, s, bp, gp, rp, partials,
                     lse, sync, t_out, s_pool);
  return hipGetLastError();
}

hipError_t launch_resident(const Shape &s, const BatchParams &bp, const ResidentPlan &rp, const GroupPtrs &gp,
                           int32_t n_groups, unsigned long long *partials, float *lse, uint32_t *sync, float *t_out,
                           float *s_pool, hipStream_t stream) {
  const int n_words = (int)(RK_SYNC_WORDS * (int64_t)n_groups * s.B * s.Hkv + RK_GLOBAL_WORDS);
  hipLaunchKernelGGL(resident_clear_kernel, dim3((n_words + 255) / 256), dim3(256), 0, stream, sync, n_words);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (s.t_stride <= 0) return hipSuccess;
  const int mt = rp.m_pad / 16;
  const bool f16 = s.dtype == WKV_F16;
#define WKV_RK_CASE(DD, MM)                                                                                        \
  if (s.d == DD && mt <= MM)                                                                                       \
    return f16 ? launch_resident_t<DD, MM, true>(s, bp, rp, gp, partials, lse, sync, t_out, s_pool, stream)        \
               : launch_resident_t<DD, MM, false>(s, bp, rp, gp, partials, lse, sync, t_out, s_pool, stream);
  WKV_RK_CASE(128, 1) WKV_RK_CASE(128, 2) WKV_RK_CASE(128, 4) WKV_RK_CASE(128, 8)
  WKV_RK_CASE(64, 1) WKV_RK_CASE(64, 2) WKV_RK_CASE(64, 4) WKV_RK_CASE(64, 8)
#undef WKV_RK_CASE
  return hipErrorInvalidValue;
}

}  // namespace wkv
