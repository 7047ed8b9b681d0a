// One decode step over the compact cache: the new token's K/V row is appended and its query
// heads attend to every retained row (softmax(q.K^T * scale).V, nothing masked).
//
// With one query row per head this is a matrix-vector product per KV head: every K and V row
// is read once and used for G = Hq/Hkv dot products, so the step is bound by the HBM stream of
// the two caches; what matters is that the arithmetic per row stays well below the memory rate.
//
//   partial kernel  grid (splits, B*Hkv): a workgroup walks one key range of one KV head.
//                   fp32 inputs: everything on the vector ALU, as follows.  16-bit inputs: the
//                   scores come from the matrix pipe (decode_partial_mfma_kernel below), the
//                   value side keeps this layout.  A
//                   16-byte piece of a row per lane, so D*esize/16 lanes cover a row and a wave
//                   load instruction reads 64/that many consecutive rows (fully coalesced).  Each
//                   lane group keeps its own online-softmax state (running max, sum, output
//                   piece) per query head, so nothing crosses lanes inside the loop except the
//                   dot-product reduction within a row's lanes; lane groups, then waves, merge
//                   once at the end and the workgroup writes (m, l, o) to the workspace.
//   combine kernel  grid (B*Hkv): merges the splits, normalises, writes fp32 output, bumps the
//                   row count.
#include <atomic>
#include <mutex>

#include "wkv_device.h"

namespace wkv {

// Scratch memory of wkv_decode_step_static: part of the device image, one copy per GPU at that
// GPU's own address.  In host code the name is only a handle for hipGetSymbolAddress; the device
// address found there (per device, once) is what the kernels get.
static __device__ __align__(256) unsigned char scratch[WKV_DECODE_STATIC_SCRATCH_BYTES];

constexpr int DEC_THREADS = 256;
constexpr int DEC_WAVES = DEC_THREADS / 64;
constexpr int DEC_U = 4;            // row tiles per wave batch (loads in flight: 2 * DEC_U per lane)

struct half_t { uint16_t bits; };             // element tag of IEEE half tensors (uint16_t stands for bfloat16)

template <typename T> struct Piece;           // the 16-byte piece of a row held by one lane
template <> struct Piece<half_t> {
  static constexpr int E = 8;
  static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[8]) {
    const f16x8 h = __builtin_bit_cast(f16x8, r);
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
  }
};
template <> struct Piece<uint16_t> {
  static constexpr int E = 8;
  static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[8]) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <> struct Piece<float> {
  static constexpr int E = 4;
  static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[4]) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
};

// Sum over the LPK (8, 16 or 32) adjacent lanes that hold one row; every lane gets the total.
template <int LPK>
__device__ __forceinline__ float row_lanes_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, false)); // row_half_mirror
  if (LPK >= 16)
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, false)); // row_mirror
  if (LPK >= 32) x += __shfl_xor(x, 16);
  return x;
}

// Merge the online-softmax state (m2, l2, o2) into (m, l, o); all in base 2.
template <int E>
__device__ __forceinline__ void merge_state(float &m, float &l, float (&o)[E], float m2, float l2, const float (&o2)[E]) {
  const float mn = fmaxf(m, m2);
  if (mn == -INFINITY) return;                      // both empty
  const float a = fast_exp2(m - mn), b = fast_exp2(m2 - mn);
  l = l * a + l2 * b;
#pragma unroll
  for (int c = 0; c < E; ++c) o[c] = o[c] * a + o2[c] * b;
  m = mn;
}

// Partial result of one (row of the grid, split): per query head g, D output channels then m, l.
__device__ __forceinline__ int64_t part_offset(const DecodeShape &s, int bh, int split, int g) {
  return (((int64_t)bh * s.n_splits + split) * s.G + g) * (s.d + 2);
}

// Merge the per-wave states in LDS ([wave][head][D outputs, m, l]) and store the workgroup's
// partial result: one thread per (head, channel); the statistics are recomputed per thread.
template <int D, int G>
__device__ __forceinline__ void merge_waves_and_store(const DecodeShape &s, float (&wave_state)[DEC_WAVES][G][D + 2],
                                                      int bh, int split, float *__restrict__ part) {
  __syncthreads();
  for (int i = threadIdx.x; i < G * D; i += DEC_THREADS) {
    const int g = i / D, c = i % D;
    float mm = wave_state[0][g][D];
#pragma unroll
    for (int w = 1; w < DEC_WAVES; ++w) mm = fmaxf(mm, wave_state[w][g][D]);
    float ll = 0.0f, oo = 0.0f;
    if (mm != -INFINITY) {
#pragma unroll
      for (int w = 0; w < DEC_WAVES; ++w) {
        const float a = fast_exp2(wave_state[w][g][D] - mm);
        ll += wave_state[w][g][D + 1] * a;
        oo += wave_state[w][g][c] * a;
      }
    }
    float *dst = part + part_offset(s, bh, split, g);
    dst[c] = oo;
    if (c == 0) { dst[D] = mm; dst[D + 1] = ll; }
  }
}

template <typename T, int D, int G>
__global__ __launch_bounds__(DEC_THREADS) void decode_partial_kernel(DecodeShape s, const T *__restrict__ q_new,
                                                                     const T *__restrict__ k_new,
                                                                     const T *__restrict__ v_new, T *k_cache, T *v_cache,
                                                                     const int32_t *__restrict__ n_valid,
                                                                     float *__restrict__ part) {
  constexpr int E = Piece<T>::E;
  constexpr int LPK = D / E;                 // lanes per row
  constexpr int KPT = 64 / LPK;              // rows per wave load instruction
  __shared__ float wave_state[DEC_WAVES][G][D + 2];

  const int bh = blockIdx.y, b = bh / s.Hkv, h = bh % s.Hkv, split = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int slot = lane / LPK, piece = lane % LPK;
  const int n = n_valid[bh];
  const bool usable = n >= 0 && n < s.capacity;       // room for the new row
  const int n_total = usable ? n + 1 : 0;             // rows attended to, the new one last

  T *kc = k_cache + (int64_t)b * s.sb + (int64_t)h * s.sh;
  T *vc = v_cache + (int64_t)b * s.sb + (int64_t)h * s.sh;
  const T *kn = k_new + ((int64_t)b * s.Hkv + h) * D;
  const T *vn = v_new + ((int64_t)b * s.Hkv + h) * D;

  // append: the first workgroup of the row copies the new K/V row into the caches.  Nobody
  // reads it from there in this launch (the new row is always taken from k_new / v_new).
  if (split == 0 && usable && threadIdx.x < 2 * LPK) {
    const int pc = threadIdx.x % LPK;
    if (threadIdx.x < LPK) *(uint4 *)(kc + (int64_t)n * s.st + pc * E) = *(const uint4 *)(kn + pc * E);
    else *(uint4 *)(vc + (int64_t)n * s.st + pc * E) = *(const uint4 *)(vn + pc * E);
  }

  // this lane's piece of the G query rows, pre-multiplied by scale * log2(e)
  float qv[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float f[E];
    Piece<T>::unpack(*(const uint4 *)(q_new + ((int64_t)b * s.Hq + (int64_t)h * G + g) * D + piece * E), f);
#pragma unroll
    for (int c = 0; c < E; ++c) qv[g][c] = f[c] * s.c1;
  }

  float m[G], l[G], o[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY; l[g] = 0.0f;
#pragma unroll
    for (int c = 0; c < E; ++c) o[g][c] = 0.0f;
  }

  const int c0 = split * s.chunk, cend = min(c0 + s.chunk, n_total);
  // rows of this wave: tiles of KPT rows, tile index wave, wave + DEC_WAVES, ...; DEC_U tiles per batch
  auto row_ptr = [&](const T *cache, const T *fresh, int j) -> const uint4 * {
    // rows below n live in the cache; row n (and anything clamped past the end) is the new one
    return (const uint4 *)(j < n ? cache + (int64_t)j * s.st + piece * E : fresh + piece * E);
  };
  uint4 kr[DEC_U], vr[DEC_U];
  auto load_batch = [&](int t0) {
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) {
      const int j = c0 + (t0 + u * DEC_WAVES) * KPT + slot;
      kr[u] = *row_ptr(kc, kn, j);
      vr[u] = *row_ptr(vc, vn, j);
    }
  };
  int t0 = wave;
  if (c0 < cend) load_batch(t0);
  for (; c0 + t0 * KPT < cend; t0 += DEC_U * DEC_WAVES) {
    uint4 kcur[DEC_U], vcur[DEC_U];
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) { kcur[u] = kr[u]; vcur[u] = vr[u]; }
    load_batch(t0 + DEC_U * DEC_WAVES);          // next batch (addresses clamp to the new row past the end)

    float sc[DEC_U][G];
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) {
      float kf[E];
      Piece<T>::unpack(kcur[u], kf);
      const int j = c0 + (t0 + u * DEC_WAVES) * KPT + slot;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = 0.0f;
#pragma unroll
        for (int c = 0; c < E; ++c) a = fmaf(qv[g][c], kf[c], a);
        a = row_lanes_sum<LPK>(a);
        sc[u][g] = j < cend ? a : -INFINITY;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float bm = sc[0][g];
#pragma unroll
      for (int u = 1; u < DEC_U; ++u) bm = fmaxf(bm, sc[u][g]);
      const float mn = fmaxf(m[g], bm);
      if (mn != -INFINITY) {
        const float corr = fast_exp2(m[g] - mn);    // m = -inf: 0
        m[g] = mn;
        l[g] *= corr;
#pragma unroll
        for (int c = 0; c < E; ++c) o[g][c] *= corr;
      }
    }
#pragma unroll
    for (int u = 0; u < DEC_U; ++u) {
      float vf[E];
      Piece<T>::unpack(vcur[u], vf);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = m[g] == -INFINITY ? 0.0f : fast_exp2(sc[u][g] - m[g]);
        l[g] += p;
#pragma unroll
        for (int c = 0; c < E; ++c) o[g][c] = fmaf(p, vf[c], o[g][c]);
      }
    }
  }

  // merge the KPT lane groups of the wave (lanes with equal piece)
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int off = LPK; off < 64; off <<= 1) {
      float o2[E];
      const float m2 = __shfl_xor(m[g], off), l2 = __shfl_xor(l[g], off);
#pragma unroll
      for (int c = 0; c < E; ++c) o2[c] = __shfl_xor(o[g][c], off);
      merge_state<E>(m[g], l[g], o[g], m2, l2, o2);
    }
    if (slot == 0) {
#pragma unroll
      for (int c = 0; c < E; ++c) wave_state[wave][g][piece * E + c] = o[g][c];
      if (piece == 0) { wave_state[wave][g][D] = m[g]; wave_state[wave][g][D + 1] = l[g]; }
    }
  }
  merge_waves_and_store<D, G>(s, wave_state, bh, split, part);
}

// ---- bf16 / fp16: scores on the matrix pipe --------------------------------------------------
// The G query rows (padded to 16) are the B operand of v_mfma_f32_16x16x32_bf16 (_f16) and 16 cache rows
// the A operand, loaded in operand layout as in the score kernels, so a block of 16 rows costs
// D/32 MFMAs instead of 16 * G dot-product reductions, and each lane takes the exponent of 4
// scores instead of G per row.  The probabilities go through a small per-wave LDS tile to the
// value side, which keeps the row-piece layout above (V is contracted over rows, the wrong way
// round for an MFMA operand).  Every lane of a wave uses the same running maximum per head, so
// the lane groups' outputs simply add up at the end.
template <int D, int G, bool F16>
__global__ __launch_bounds__(DEC_THREADS) void decode_partial_mfma_kernel(
    DecodeShape s, const uint16_t *__restrict__ q_new, const uint16_t *__restrict__ k_new,
    const uint16_t *__restrict__ v_new, uint16_t *k_cache, uint16_t *v_cache, const int32_t *__restrict__ n_valid,
    float *__restrict__ part) {
  constexpr int E = 8;
  constexpr int LPK = D / E;                 // lanes per row (value side)
  constexpr int KPT = 64 / LPK;              // rows per wave load instruction (value side)
  constexpr int VT = 16 / KPT;               // value loads per block of 16 rows
  constexpr int KS = D / 32;                 // MFMA steps over the channels
  constexpr int GP = G <= 4 ? 4 : 8;         // heads padded to whole float4s in LDS
  __shared__ float wave_state[DEC_WAVES][G][D + 2];
  __shared__ __attribute__((aligned(16))) float p_s[DEC_WAVES][16][GP];     // probabilities of the wave's block, [row][head]
  __shared__ __attribute__((aligned(16))) float corr_s[DEC_WAVES][GP];      // rescale factor of the outputs, per head

  const int bh = blockIdx.y, b = bh / s.Hkv, h = bh % s.Hkv, split = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, quad = lane >> 4;            // score side: head, 4 rows
  const int slot = lane / LPK, piece = lane % LPK;        // value side: row of the tile, 16-byte piece
  const int n = n_valid[bh];
  const bool usable = n >= 0 && n < s.capacity;
  const int n_total = usable ? n + 1 : 0;

  uint16_t *kc = k_cache + (int64_t)b * s.sb + (int64_t)h * s.sh;
  uint16_t *vc = v_cache + (int64_t)b * s.sb + (int64_t)h * s.sh;
  const uint16_t *kn = k_new + ((int64_t)b * s.Hkv + h) * D;
  const uint16_t *vn = v_new + ((int64_t)b * s.Hkv + h) * D;

  if (split == 0 && usable && threadIdx.x < 2 * LPK) {     // append (see the kernel above)
    const int pc = threadIdx.x % LPK;
    if (threadIdx.x < LPK) *(uint4 *)(kc + (int64_t)n * s.st + pc * E) = *(const uint4 *)(kn + pc * E);
    else *(uint4 *)(vc + (int64_t)n * s.st + pc * E) = *(const uint4 *)(vn + pc * E);
  }

  // query rows as B fragments: lane (head col, quad) holds channels 32*ks + 8*quad .. +7; heads >= G are zero
  bf16x8 qb[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (col < G) v = *(const uint4 *)(q_new + ((int64_t)b * s.Hq + (int64_t)h * G + col) * D + ks * 32 + quad * 8);
    qb[ks] = *(const bf16x8 *)&v;
  }

  float m = -INFINITY, l = 0.0f;             // of head `col` (lanes with col < G), l over this lane's rows only
  float o[G][E];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int c = 0; c < E; ++c) o[g][c] = 0.0f;

  const int c0 = split * s.chunk, cend = min(c0 + s.chunk, n_total);
  auto k_ptr = [&](int j, int ks) -> const uint4 * {      // rows below n live in the cache, the rest is the new row
    return (const uint4 *)((j < n ? kc + (int64_t)j * s.st : kn) + ks * 32 + quad * 8);
  };
  auto v_ptr = [&](int j) -> const uint4 * {
    return (const uint4 *)((j < n ? vc + (int64_t)j * s.st : vn) + piece * E);
  };
  uint4 kr[KS], vr[VT];
  auto load_block = [&](int blk) {
    const int r0 = c0 + blk * 16;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kr[ks] = *k_ptr(r0 + col, ks);
#pragma unroll
    for (int t = 0; t < VT; ++t) vr[t] = *v_ptr(r0 + t * KPT + slot);
  };
  int blk = wave;
  if (c0 < cend) load_block(blk);
  for (; c0 + blk * 16 < cend; blk += DEC_WAVES) {
    uint4 kcur[KS], vcur[VT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kcur[ks] = kr[ks];
#pragma unroll
    for (int t = 0; t < VT; ++t) vcur[t] = vr[t];
    load_block(blk + DEC_WAVES);               // next block (addresses clamp to the new row past the end)

    // scores of 16 rows x 16 (padded) heads
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      acc = mfma_16x16x32<F16>(*(const bf16x8 *)&kcur[ks], qb[ks], acc);
    const int r0 = c0 + blk * 16;
    float sc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) sc[e] = r0 + quad * 4 + e < cend ? acc[e] * s.c1 : -INFINITY;
    float bm = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    bm = fmaxf(bm, __shfl_xor(bm, 16));
    bm = fmaxf(bm, __shfl_xor(bm, 32));          // the same in the 4 lanes of a head
    const float mn = fmaxf(m, bm);
    float corr = 1.0f, pr[4] = {0.f, 0.f, 0.f, 0.f};
    if (mn != -INFINITY) {
      corr = fast_exp2(m - mn);                  // m = -inf: 0
      m = mn;
      float ps = 0.0f;
#pragma unroll
      for (int e = 0; e < 4; ++e) { pr[e] = fast_exp2(sc[e] - mn); ps += pr[e]; }
      l = l * corr + ps;
    }
    if (col < G) {
#pragma unroll
      for (int e = 0; e < 4; ++e) p_s[wave][quad * 4 + e][col] = pr[e];
      if (quad == 0) corr_s[wave][col] = corr;
    }
    // the wave's own LDS writes above are read back below: LDS serves a wave's requests in order
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();

    float cr[GP];
#pragma unroll
    for (int i = 0; i < GP; i += 4) *(float4 *)&cr[i] = *(const float4 *)&corr_s[wave][i];
    bool rescale = false;
#pragma unroll
    for (int g = 0; g < G; ++g) rescale |= cr[g] != 1.0f;
    if (__any(rescale)) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < E; ++c) o[g][c] *= cr[g];
    }
#pragma unroll
    for (int t = 0; t < VT; ++t) {
      float pg[GP], vf[E];
#pragma unroll
      for (int i = 0; i < GP; i += 4) *(float4 *)&pg[i] = *(const float4 *)&p_s[wave][t * KPT + slot][i];
      if constexpr (F16) Piece<half_t>::unpack(vcur[t], vf); else Piece<uint16_t>::unpack(vcur[t], vf);
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int c = 0; c < E; ++c) o[g][c] = fmaf(pg[g], vf[c], o[g][c]);
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
  }

  // the wave's totals: outputs over the lane groups (lanes with equal piece), l over the 4 lanes of a head
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int c = 0; c < E; ++c) {
      float x = o[g][c];
#pragma unroll
      for (int off = LPK; off < 64; off <<= 1) x += __shfl_xor(x, off);
      o[g][c] = x;
    }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (slot == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int c = 0; c < E; ++c) wave_state[wave][g][piece * E + c] = o[g][c];
  }
  if (lane < G) { wave_state[wave][lane][D] = m; wave_state[wave][lane][D + 1] = l; }    // lane = head (quad 0)
  merge_waves_and_store<D, G>(s, wave_state, bh, split, part);
}

constexpr int DEC_MAX_SPLITS = 64;

__global__ __launch_bounds__(DEC_THREADS) void decode_combine_kernel(DecodeShape s, const float *__restrict__ part,
                                                                     int32_t *n_valid, float *__restrict__ out) {
  // weight of every (head, split) in the merged result: 2^(m_split - m) / l, or 0
  __shared__ float wgt[8][DEC_MAX_SPLITS];
  __shared__ float m_s[8][DEC_MAX_SPLITS], l_s[8][DEC_MAX_SPLITS];
  const int bh = blockIdx.x, b = bh / s.Hkv, h = bh % s.Hkv;
  const int D = s.d;
  for (int i = threadIdx.x; i < s.G * s.n_splits; i += DEC_THREADS) {      // all (m, l) pairs at once
    const int g = i / s.n_splits, sp = i % s.n_splits;
    const float *p = part + part_offset(s, bh, sp, g);
    m_s[g][sp] = p[D];
    l_s[g][sp] = p[D + 1];
  }
  __syncthreads();
  if (threadIdx.x < s.G) {
    const int g = threadIdx.x;
    float mm = -INFINITY, ll = 0.0f;
    for (int sp = 0; sp < s.n_splits; ++sp) mm = fmaxf(mm, m_s[g][sp]);
    for (int sp = 0; sp < s.n_splits; ++sp) {
      const float a = mm == -INFINITY ? 0.0f : fast_exp2(m_s[g][sp] - mm);
      wgt[g][sp] = a;
      ll += l_s[g][sp] * a;
    }
    // no row could be attended to (the cache is full or its count is invalid): NaN marks it
    const float inv = ll > 0.0f ? 1.0f / ll : __uint_as_float(0x7fc00000u);
    for (int sp = 0; sp < s.n_splits; ++sp) wgt[g][sp] *= inv;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < s.G * D; i += DEC_THREADS) {
    const int g = i / D, c = i % D;
    const float *p = part + part_offset(s, bh, 0, g) + c;
    const int64_t stride = (int64_t)s.G * (D + 2);                         // between the splits of one head
    float oo = 0.0f;
    int sp = 0;
    for (; sp + 4 <= s.n_splits; sp += 4) {                                 // four independent loads in flight
      const float a0 = p[sp * stride], a1 = p[(sp + 1) * stride], a2 = p[(sp + 2) * stride], a3 = p[(sp + 3) * stride];
      oo += a0 * wgt[g][sp] + a1 * wgt[g][sp + 1] + a2 * wgt[g][sp + 2] + a3 * wgt[g][sp + 3];
    }
    for (; sp < s.n_splits; ++sp) oo += p[sp * stride] * wgt[g][sp];
    out[((int64_t)b * s.Hq + (int64_t)h * s.G + g) * D + c] = oo;
  }
  if (threadIdx.x == 0) {
    const int n = n_valid[bh];
    if (n >= 0 && n < s.capacity && !s.keep_count) n_valid[bh] = n + 1;
  }
}

template <typename T, int D, int G>
static void launch_partial_g(const DecodeShape &s, dim3 grid, const void *q, const void *kn, const void *vn, void *kc,
                             void *vc, const int32_t *n_valid, float *part, hipStream_t stream) {
  if constexpr (sizeof(T) == 2)     // bf16 / fp16: scores on the matrix pipe
    hipLaunchKernelGGL((decode_partial_mfma_kernel<D, G, sizeof(T) == 2 && !__is_same(T, uint16_t)>), grid, dim3(DEC_THREADS), 0, stream, s, (const uint16_t *)q,
                       (const uint16_t *)kn, (const uint16_t *)vn, (uint16_t *)kc, (uint16_t *)vc, n_valid, part);
  else
    hipLaunchKernelGGL((decode_partial_kernel<T, D, G>), grid, dim3(DEC_THREADS), 0, stream, s, (const T *)q,
                       (const T *)kn, (const T *)vn, (T *)kc, (T *)vc, n_valid, part);
}

template <typename T, int D>
static hipError_t launch_partial(const DecodeShape &s, const void *q, const void *kn, const void *vn, void *kc,
                                 void *vc, const int32_t *n_valid, float *part, hipStream_t stream) {
  dim3 grid(s.n_splits, s.B * s.Hkv);
#define WKV_DEC_CASE(GG) \
  case GG: launch_partial_g<T, D, GG>(s, grid, q, kn, vn, kc, vc, n_valid, part, stream); break;
  switch (s.G) {
    WKV_DEC_CASE(1) WKV_DEC_CASE(2) WKV_DEC_CASE(3) WKV_DEC_CASE(4) WKV_DEC_CASE(5) WKV_DEC_CASE(6)
    WKV_DEC_CASE(7) WKV_DEC_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef WKV_DEC_CASE
  return hipGetLastError();
}

hipError_t launch_decode(const DecodeShape &s, const void *q_new, const void *k_new, const void *v_new, void *k_cache,
                         void *v_cache, int32_t *n_valid, float *out, float *part, hipStream_t stream) {
  hipError_t e;
  if (s.dtype == WKV_BF16)
    e = s.d == 128 ? launch_partial<uint16_t, 128>(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, part, stream)
                   : launch_partial<uint16_t, 64>(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, part, stream);
  else if (s.dtype == WKV_F16)
    e = s.d == 128 ? launch_partial<half_t, 128>(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, part, stream)
                   : launch_partial<half_t, 64>(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, part, stream);
  else
    e = s.d == 128 ? launch_partial<float, 128>(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, part, stream)
                   : launch_partial<float, 64>(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, part, stream);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_combine_kernel, dim3(s.B * s.Hkv), dim3(DEC_THREADS), 0, stream, s, part, n_valid, out);
  return hipGetLastError();
}

constexpr int MAX_DEVICES = 64;
static std::atomic<void *> scratch_ptr[MAX_DEVICES];
static std::mutex scratch_mutex;

hipError_t launch_decode_static(const DecodeShape &s, const void *q_new, const void *k_new, const void *v_new,
                                void *k_cache, void *v_cache, int32_t *n_valid, float *out, hipStream_t stream) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  void *p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {                                 // first call on this device (which is the current one)
    std::lock_guard<std::mutex> lock(scratch_mutex);
    p = scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!p) return hipErrorInvalidSymbol;
      scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  // every partial result a combine reads is written by the partial kernel of the same call:
  // nothing in the array has to be cleared
  return launch_decode(s, q_new, k_new, v_new, k_cache, v_cache, n_valid, out, (float *)p, stream);
}

}  // namespace wkv
