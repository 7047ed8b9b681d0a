// Single-pass token scores (WindowKV Eq. 1-2): the keys of the scored layer are read from HBM
// exactly once.
//
// The softmax normaliser of a row needs every key of the prefix, so a workgroup cannot finish
// its column sums alone.  Instead of reading the keys twice, each workgroup keeps the raw
// logits of its 256-key chunk in registers (they are the MFMA accumulators: 128 VGPRs per
// lane) and the workgroups of one (group, sequence, KV head) exchange two small vectors through
// device-scope atomics:
//
//   phase 1  S = K_chunk . Q^T (MFMA), causal mask, per-row maximum of the chunk
//            -> atomicMax into the problem's row maxima; arrive on counter 1; wait for all chunks
//   phase 2  P = 2^(c1*(S - rowmax)) in place, per-row sums of the chunk
//            -> fixed-point atomicAdd (2^-40 units, so the result does not depend on arrival
//               order) into the problem's row sums; arrive on counter 2; wait
//   phase 3  t_j = sum_i P_ij / Z_i, written to the token-score array
//
// Waiting is safe because work is handed out by a ticket counter in problem-major order: a
// workgroup only ever waits for tickets of its own problem, every smaller ticket has already
// been taken by a workgroup that is running or finished, and the host only uses this kernel
// when one problem's chunks fit into half of the workgroup slots that can be resident at once,
// so a free slot always exists for the problem's next ticket.  The spin is bounded anyway: if it
// runs out, the workgroup raises the error word of the sync block and carries on, so every
// wave exits.
//
// Two workgroups per CU (256 VGPRs each): while one waits at a counter the other streams keys.
#include "wkv_device.h"

namespace wkv {

constexpr int FU_TP = FUSED_CHUNK / (MF_WAVES * 16 * MF_KT);   // tile pairs per wave (2)
constexpr int FU_SPIN_LIMIT = 1 << 20;
constexpr float FU_FIX = 1099511627776.0f;                     // 2^40
static_assert(FU_TP * MF_WAVES * 16 * MF_KT == FUSED_CHUNK, "chunk must be whole tile pairs");

__global__ void sync_init_kernel(uint32_t *sync, size_t n_words) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x)
    sync[i] = 0u;
}

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float order_unkey(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Thread 0 waits (bounded) until *cnt reaches target; the workgroup then continues together.
__device__ __forceinline__ void wait_for(uint32_t *cnt, uint32_t target, uint32_t *err) {
  if (threadIdx.x == 0) {
    int spins = 0;
    while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(4);
      if (++spins > FU_SPIN_LIMIT) {
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
  }
  __syncthreads();
}

template <int D, int MT>
__global__ __launch_bounds__(MF_THREADS, 2) void score_fused_kernel(Shape s, BatchParams bp, GroupPtrs gp,
                                                                    FusedPlan fp, uint32_t *__restrict__ sync,
                                                                    float *__restrict__ t_out) {
  constexpr int KS = D / 32;
  constexpr int ROWS = MT * 16;
  __shared__ uint4 qfrag[MT * KS * 64];
  __shared__ float red_s[MF_WAVES][ROWS];
  __shared__ float row_s[ROWS];
  __shared__ float t_s[FUSED_CHUNK];
  __shared__ int ticket_s;

  // ---- take a ticket: (group, sequence, KV head, chunk) in problem-major order ----------------
  if (threadIdx.x == 0) ticket_s = (int)atomicAdd(sync + SYNC_TICKET, 1u);
  __syncthreads();
  const int ticket = ticket_s;
  const int g = ticket / fp.tickets_per_group;
  int rem = ticket - g * fp.tickets_per_group;
  int b = 0;
  while (b + 1 < s.B && rem >= fp.first[b + 1]) ++b;
  rem -= fp.first[b];
  const int nch = fp.nch[b];
  const int h = rem / nch, chunk = rem - h * nch;

  const int L = bp.seq[b].L, n_review = L - s.w_obs;
  const int64_t row = ((int64_t)g * s.B + b) * s.Hkv + h;
  uint32_t *ps = sync + SYNC_HEADER_WORDS + row * SYNC_PROBLEM_WORDS;
  uint32_t *rowmax = ps + SYNC_ROWMAX;
  unsigned long long *zfix = (unsigned long long *)(ps + SYNC_ZFIX);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;
  const int c0 = chunk * FUSED_CHUNK;
  const int cend = min(c0 + FUSED_CHUNK, L);
  const float c1 = s.c1;

  stage_q_fragments<D, MT>(s, gp.q[g], b, h, qfrag);

  // ---- phase 1: logits of the chunk, kept in registers -------------------------------------------
  const uint16_t *kbase = (const uint16_t *)gp.k[g] + (int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh + quad * 8;
  KFrags<KS> kf[FU_TP];
#pragma unroll
  for (int tp = 0; tp < FU_TP; ++tp)
    load_k<KS>(kf[tp], kbase, s.kv_st, c0 + (tp * MF_WAVES + wave) * (16 * MF_KT), col, cend);
  __syncthreads();                                   // query fragments staged

  f32x4 S[FU_TP][MF_KT][MT];
  float rmax[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) rmax[mt] = -INFINITY;
#pragma unroll
  for (int tp = 0; tp < FU_TP; ++tp) {
    const int j0 = c0 + (tp * MF_WAVES + wave) * (16 * MF_KT);
#pragma unroll
    for (int n = 0; n < MF_KT; ++n)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) S[tp][n][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 qraw = qfrag[(mt * KS + ks) * 64 + lane];
        const bf16x8 qb = *(const bf16x8 *)&qraw;
#pragma unroll
        for (int n = 0; n < MF_KT; ++n)
          S[tp][n][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tp].f[n][ks], qb, S[tp][n][mt], 0, 0, 0);
      }
    if (j0 + 16 * MF_KT > n_review) {
      // causal mask of the observation block (key j visible to observation query io iff
      // j <= n_review + io) and the end of the sequence
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int r = mt * 16 + col;
        const int last_vis = r < s.M ? n_review + (r % s.w_obs) : -1;
#pragma unroll
        for (int n = 0; n < MF_KT; ++n)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int j = j0 + n * 16 + quad * 4 + e;
            if (j > last_vis || j >= cend) S[tp][n][mt][e] = -INFINITY;
          }
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int n = 0; n < MF_KT; ++n)
        rmax[mt] = fmaxf(rmax[mt], fmaxf(fmaxf(S[tp][n][mt][0], S[tp][n][mt][1]), fmaxf(S[tp][n][mt][2], S[tp][n][mt][3])));
  }
  // row maxima of the chunk: 4 quads of a wave, then 4 waves
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float m = rmax[mt];
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    if (quad == 0) red_s[wave][mt * 16 + col] = m;
  }
  __syncthreads();
  if (threadIdx.x < ROWS) {
    const int r = threadIdx.x;
    const float m = fmaxf(fmaxf(red_s[0][r], red_s[1][r]), fmaxf(red_s[2][r], red_s[3][r]));
    if (m != -INFINITY) atomicMax(rowmax + r, order_key(m));
  }
  // Everything the workgroups exchange travels in device-scope atomics, so no cache has to be
  // written back or invalidated (a device-scope fence would do both to the whole L2 of the XCD).
  // What is needed is order: every lane waits for its own atomics to be acknowledged before the
  // barrier (the barrier alone does not wait for vector-memory operations), and only then does
  // thread 0 announce the arrival.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(ps + SYNC_CNT1, 1u);
  wait_for(ps + SYNC_CNT1, (uint32_t)nch, sync + SYNC_ERROR);

  // ---- phase 2: P = 2^(c1 * (S - rowmax)), row sums ------------------------------------------------
  if (threadIdx.x < ROWS)
    row_s[threadIdx.x] = c1 * order_unkey(__hip_atomic_load(rowmax + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  __syncthreads();
  float zs[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const float mg = row_s[mt * 16 + col];
    float z = 0.0f;
#pragma unroll
    for (int tp = 0; tp < FU_TP; ++tp)
#pragma unroll
      for (int n = 0; n < MF_KT; ++n)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = fast_exp2(fmaf(S[tp][n][mt][e], c1, -mg));
          S[tp][n][mt][e] = p;
          z += p;
        }
    z += __shfl_xor(z, 16);
    z += __shfl_xor(z, 32);
    zs[mt] = z;
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    if (quad == 0) red_s[wave][mt * 16 + col] = zs[mt];
  __syncthreads();
  if (threadIdx.x < ROWS) {
    const int r = threadIdx.x;
    const float z = (red_s[0][r] + red_s[1][r]) + (red_s[2][r] + red_s[3][r]);   // <= 256: exact scaling below
    atomicAdd(zfix + r, (unsigned long long)(z * FU_FIX));
  }
  __builtin_amdgcn_s_waitcnt(0);                     // as above: acknowledged before the arrival
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(ps + SYNC_CNT2, 1u);
  wait_for(ps + SYNC_CNT2, (uint32_t)nch, sync + SYNC_ERROR);

  // ---- phase 3: t_j = sum_i P_ij / Z_i ---------------------------------------------------------------
  if (threadIdx.x < ROWS) {
    const int r = threadIdx.x;
    const unsigned long long zf = __hip_atomic_load(zfix + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const float Z = (float)((double)zf * (1.0 / 1099511627776.0));
    row_s[r] = (r < s.M && Z > 0.0f) ? 1.0f / Z : 0.0f;     // padded rows contribute nothing
  }
  __syncthreads();
  float inv[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) inv[mt] = row_s[mt * 16 + col];
#pragma unroll
  for (int tp = 0; tp < FU_TP; ++tp)
#pragma unroll
    for (int n = 0; n < MF_KT; ++n) {
      f32x4 tq;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a = fmaf(S[tp][n][mt][e], inv[mt], a);
        tq[e] = row16_sum(a);
      }
      if (col == 0) *(f32x4 *)(t_s + (tp * MF_WAVES + wave) * (16 * MF_KT) + n * 16 + quad * 4) = tq;
    }
  __syncthreads();
  float *trow = t_out + row * s.t_stride;
  const int tend = min(c0 + FUSED_CHUNK, n_review);
  for (int j = c0 + threadIdx.x; j < tend; j += MF_THREADS) trow[j] = t_s[j - c0];
  if (chunk == nch - 1)        // the last chunk also clears the row beyond the review context
    for (int j = n_review + threadIdx.x; j < s.t_stride; j += MF_THREADS) trow[j] = 0.0f;
}

template <int D, int MT>
static hipError_t launch_fused_t(const Shape &s, const BatchParams &bp, const FusedPlan &fp, const GroupPtrs &gp,
                                 uint32_t *sync, size_t sync_words, float *t_out, hipStream_t stream,
                                 hipEvent_t mid, bool *used) {
  // resident workgroup slots of this kernel on this device (queried once per instantiation)
  static int slots = -1;
  if (slots < 0) {
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess)
      e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)score_fused_kernel<D, MT>, MF_THREADS, 0);
    if (e != hipSuccess) return e;
    slots = per_cu * prop.multiProcessorCount;
  }
  int nch_max = 0;
  for (int b = 0; b < s.B; ++b) nch_max = fp.nch[b] > nch_max ? fp.nch[b] : nch_max;
  if (nch_max * 2 > slots) { *used = false; return hipSuccess; }   // caller falls back to two passes
  *used = true;
  const int zero_blocks = (int)((sync_words + 255) / 256 < 64 ? (sync_words + 255) / 256 : 64);
  hipLaunchKernelGGL(sync_init_kernel, dim3(zero_blocks), dim3(256), 0, stream, sync, sync_words);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (mid && (e = hipEventRecord(mid, stream)) != hipSuccess) return e;
  hipLaunchKernelGGL((score_fused_kernel<D, MT>), dim3(fp.total_tickets), dim3(MF_THREADS), 0, stream, s, bp, gp, fp,
                     sync, t_out);
  return hipGetLastError();
}

hipError_t launch_score_fused(const Shape &s, const BatchParams &bp, const ScorePlan &pl, const FusedPlan &fp,
                              const GroupPtrs &gp, uint32_t *sync, size_t sync_words, float *t_out,
                              hipStream_t stream, hipEvent_t mid, bool *used) {
  const int mt = pl.m_pad / 16;
#define WKV_FUSED_CASE(DD, MM) \
  if (s.d == DD && mt <= MM) return launch_fused_t<DD, MM>(s, bp, fp, gp, sync, sync_words, t_out, stream, mid, used);
  WKV_FUSED_CASE(128, 1) WKV_FUSED_CASE(128, 2) WKV_FUSED_CASE(128, 4) WKV_FUSED_CASE(128, 8)
  WKV_FUSED_CASE(64, 1) WKV_FUSED_CASE(64, 2) WKV_FUSED_CASE(64, 4) WKV_FUSED_CASE(64, 8)
#undef WKV_FUSED_CASE
  *used = false;
  return hipSuccess;
}

}  // namespace wkv
