/* The header as strict C99 and the library from a plain C program: host-only entry points. */
#include <stdio.h>
#include <string.h>
#include "wkv.h"
int main(void) {
  int32_t L[1] = {4096}, win[1] = {8}, p[1] = {8}, k[1] = {64};
  wkv_problem pr; memset(&pr, 0, sizeof pr);
  pr.batch = 1; pr.n_q_heads = 32; pr.n_kv_heads = 8; pr.head_dim = 128; pr.w_obs = 32; pr.max_seq_len = 4096;
  pr.dtype = WKV_BF16; pr.seq_len = L; pr.win = win; pr.top_p = p; pr.k_windows = k;
  pr.q_stride_b = 32 * 32 * 128; pr.q_stride_h = 32 * 128; pr.q_stride_t = 128;
  pr.kv_stride_b = 8LL * 4096 * 128; pr.kv_stride_h = 4096 * 128; pr.kv_stride_t = 128;
  pr.out_stride_b = 8LL * 544 * 128; pr.out_stride_h = 544 * 128; pr.out_stride_t = 128;
  wkv_dims d;
  wkv_status st = wkv_get_dims(&pr, &d);
  printf("%d %d %d %d %d %zu %s\n", (int)st, d.obs_rows, d.nw_max, d.k_max, d.nkeep_max, wkv_workspace_bytes(&pr, 1), wkv_status_string(st));
  return st == WKV_OK ? 0 : 1;
}
