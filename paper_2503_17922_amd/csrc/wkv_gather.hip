// Shared-index row gather (WindowKV Section 2.2.2): every layer of a group keeps the K and V
// rows at the group's retained positions.  A pure copy, bound by HBM bandwidth.
//
// Mapping: a row of head_dim elements is 256 or 512 bytes; `LPR` lanes (16 B each) cover one
// row, so one 256-thread workgroup moves 256/LPR rows per load instruction and keeps UNROLL
// such instructions in flight per lane.  grid.x walks row blocks of the compact cache,
// grid.y the (sequence, KV head) pairs, grid.z the (layer, K|V) tensors, so neighbouring
// workgroups (which land on different XCDs) stream neighbouring 16-32 KB pieces of the same
// tensor.  Selected rows come in runs of `win` consecutive tokens, i.e. 2-32 KB contiguous
// reads; writes are fully contiguous.
#include "wkv_internal.h"

namespace wkv {

constexpr int GATHER_THREADS = 256;
constexpr int GATHER_UNROLL = 2;   // measured on MI355X: 2 rows in flight per lane beat 1, 3, 4, 8 and 16
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int LPR>  // lanes per row
__global__ __launch_bounds__(GATHER_THREADS) void gather_kernel(
    Shape s, LayerPtrs lp, int32_t gamma, const int32_t *__restrict__ tok_idx,
    const int32_t *__restrict__ n_keep, int64_t row_bytes_in, int64_t row_bytes_out, int64_t esize) {
  constexpr int ROWS_PER_PASS = GATHER_THREADS / LPR;
  const int bh = blockIdx.y;                 // b * Hkv + h
  const int b = bh / s.Hkv, h = bh % s.Hkv;
  const int layer = blockIdx.z >> 1;
  const bool is_v = blockIdx.z & 1;
  const int group = layer / gamma;
  const char *src = (const char *)(is_v ? lp.v_in[layer] : lp.k_in[layer]) +
                    ((int64_t)b * s.kv_sb + (int64_t)h * s.kv_sh) * esize;
  char *dst = (char *)(is_v ? lp.v_out[layer] : lp.k_out[layer]) +
              ((int64_t)b * s.o_sb + (int64_t)h * s.o_sh) * esize;
  const int64_t irow = (int64_t)group * s.B * s.Hkv + bh;
  const int32_t *idx = tok_idx + irow * s.nkeep_max;
  const int nk = min(n_keep[irow], s.nkeep_max);
  const int n_write = s.fill_padding ? s.nkeep_max : nk;   // rows past n_keep: zero-filled or left alone
  const int max_tok = s.t_stride + s.w_obs;      // token capacity of the full cache
  const int lane_in_row = threadIdx.x % LPR;
  const int row_in_pass = threadIdx.x / LPR;
  const int row0 = blockIdx.x * (ROWS_PER_PASS * GATHER_UNROLL) + row_in_pass;
  if (blockIdx.x * (ROWS_PER_PASS * GATHER_UNROLL) >= n_write) return;

  u32x4 v[GATHER_UNROLL];
  int r[GATHER_UNROLL];
#pragma unroll
  for (int u = 0; u < GATHER_UNROLL; ++u) {
    r[u] = row0 + u * ROWS_PER_PASS;
    v[u] = u32x4{0u, 0u, 0u, 0u};
    if (r[u] < nk) {
      const int tok = idx[r[u]];
      if (tok >= 0 && tok < max_tok)               // indices are caller data: never read out of bounds
        v[u] = __builtin_nontemporal_load((const u32x4 *)(src + (int64_t)tok * row_bytes_in) + lane_in_row);
    }
  }
#pragma unroll
  for (int u = 0; u < GATHER_UNROLL; ++u) {
    if (r[u] < n_write)
      __builtin_nontemporal_store(v[u], (u32x4 *)(dst + (int64_t)r[u] * row_bytes_out) + lane_in_row);
  }
}

hipError_t launch_gather(const Shape &s, const LayerPtrs &lp, int32_t n_layers, int32_t gamma,
                         const int32_t *tok_idx, const int32_t *n_keep, hipStream_t stream) {
  if (s.nkeep_max <= 0) return hipSuccess;
  const int64_t esize = elem_bytes(s.dtype);
  const int lpr = (int)(s.d * esize / 16);   // 8 (bf16 d=64), 16, 16, or 32 (f32 d=128)
  const int rows_per_block = GATHER_THREADS / lpr * GATHER_UNROLL;
  dim3 grid((s.nkeep_max + rows_per_block - 1) / rows_per_block, s.B * s.Hkv, n_layers * 2);
  dim3 block(GATHER_THREADS);
  const int64_t rbi = s.kv_st * esize, rbo = s.o_st * esize;
  switch (lpr) {
    case 8:  hipLaunchKernelGGL(gather_kernel<8>, grid, block, 0, stream, s, lp, gamma, tok_idx, n_keep, rbi, rbo, esize); break;
    case 16: hipLaunchKernelGGL(gather_kernel<16>, grid, block, 0, stream, s, lp, gamma, tok_idx, n_keep, rbi, rbo, esize); break;
    case 32: hipLaunchKernelGGL(gather_kernel<32>, grid, block, 0, stream, s, lp, gamma, tok_idx, n_keep, rbi, rbo, esize); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace wkv
