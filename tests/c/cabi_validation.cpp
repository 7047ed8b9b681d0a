// Drives every entry point of the C ABI through its host-side validation with valid and invalid
// arguments.  Linked against the host half of the library and the launcher stand-ins, built with
// AddressSanitizer + UndefinedBehaviorSanitizer: any out-of-bounds access, overflow or misuse in the
// validation, size and planning code aborts the program.  Device pointers are fake (never
// dereferenced: the stubs launch nothing).
#include <cstdio>
#include <cstring>
#include <vector>

#include "wkv.h"

extern "C" int wkv_stub_launches;
static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, wkv_last_error()); ++failures; } } while (0)

struct Prob {
  std::vector<int32_t> L, win, p, k;
  wkv_problem pr;
  Prob(int batch, int L0, int hq, int hkv, int d, int w_obs, int w, int tp, int kk, int dtype) : L(batch), win(batch, w), p(batch, tp), k(batch, kk) {
    std::memset(&pr, 0, sizeof pr);
    int lmax = 0;
    for (int b = 0; b < batch; ++b) { L[b] = L0 - 17 * b; if (L[b] > lmax) lmax = L[b]; }
    pr.batch = batch; pr.n_q_heads = hq; pr.n_kv_heads = hkv; pr.head_dim = d; pr.w_obs = w_obs; pr.max_seq_len = lmax;
    pr.dtype = dtype; pr.seq_len = L.data(); pr.win = win.data(); pr.top_p = p.data(); pr.k_windows = k.data();
    pr.q_stride_b = (int64_t)hq * w_obs * d; pr.q_stride_h = (int64_t)w_obs * d; pr.q_stride_t = d;
    pr.kv_stride_b = (int64_t)hkv * lmax * d; pr.kv_stride_h = (int64_t)lmax * d; pr.kv_stride_t = d;
    const int64_t nk = (int64_t)kk * w + w_obs;
    pr.out_stride_b = hkv * nk * d; pr.out_stride_h = nk * d; pr.out_stride_t = d;
  }
};

int main() {
  void *dev = (void *)0x7f0000001000ull;      // "device" memory: aligned, never touched
  // ---- dims, workspace sizes and layouts over a sweep of shapes (the planning code runs for each) -------
  const int dtypes[3] = {WKV_F32, WKV_BF16, WKV_F16};
  for (int dt = 0; dt < 3; ++dt)
    for (int batch : {1, 3, 64})
      for (int L0 : {2400, 4096, 32768, 262176})
        for (int hq : {8, 32, 64})
          for (int w : {1, 8, 24, 128}) {
            if ((int64_t)(L0 - 32) / w > WKV_MAX_WINDOWS) continue;
            Prob P(batch, L0, hq, 8, 128, 32, w, (w + 1) / 2, 3, dtypes[dt]);
            wkv_dims d;
            const wkv_status st = wkv_get_dims(&P.pr, &d);
            EXPECT(st == WKV_OK);
            if (st != WKV_OK) continue;
            EXPECT(d.obs_rows == hq / 8 * 32 && d.t_stride == L0 - 32 && d.nkeep_max == 3 * w + 32);
            for (int ng : {1, 8, 64}) {
              const size_t ws = wkv_workspace_bytes(&P.pr, ng);
              wkv_workspace_layout lay;
              EXPECT(ws > 0 && ws % 256 == 0);
              EXPECT(wkv_get_workspace_layout(&P.pr, ng, &lay) == WKV_OK);
              EXPECT(lay.t_offset < lay.s_offset && lay.s_offset < ws && lay.t_written + lay.s_written == 1);
            }
          }
  // ---- every entry point: valid arguments reach the (stub) launchers, invalid ones launch nothing -----------
  Prob P(2, 4096, 32, 8, 128, 32, 8, 8, 64, WKV_BF16);
  const size_t ws1 = wkv_workspace_bytes(&P.pr, 1), ws2 = wkv_workspace_bytes(&P.pr, 2);
  const void *kl[4] = {dev, dev, dev, dev}; void *ol[4] = {dev, dev, dev, dev};
  const void *qg[2] = {dev, dev}; const float *lg[2] = {(const float *)dev, (const float *)dev};
  int32_t *idev = (int32_t *)dev; float *fdev = (float *)dev;
  int before = wkv_stub_launches;
  EXPECT(wkv_score(&P.pr, dev, dev, nullptr, fdev, dev, ws1, nullptr) == WKV_OK);
  EXPECT(wkv_window_pool(&P.pr, fdev, fdev, nullptr) == WKV_OK);
  EXPECT(wkv_topk_windows(&P.pr, fdev, idev, idev, idev, nullptr) == WKV_OK);
  EXPECT(wkv_gather_group(&P.pr, 4, kl, kl, idev, idev, ol, ol, nullptr) == WKV_OK);
  EXPECT(wkv_compress_group(&P.pr, 4, dev, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws1, nullptr) == WKV_OK);
  EXPECT(wkv_compress_groups(&P.pr, 2, 2, qg, lg, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws2, nullptr) == WKV_OK);
  int32_t kg[4] = {64, 10, 0, 64};
  EXPECT(wkv_compress_groups(&P.pr, 2, 2, qg, nullptr, kg, kl, kl, ol, ol, idev, idev, idev, dev, ws2, nullptr) == WKV_OK);
  EXPECT(wkv_index_jaccard(&P.pr, 4, idev, idev, fdev, nullptr) == WKV_OK);
  EXPECT(wkv_stub_launches > before);
  before = wkv_stub_launches;
  EXPECT(wkv_score(&P.pr, nullptr, dev, nullptr, fdev, dev, ws1, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_score(&P.pr, (char *)dev + 2, dev, nullptr, fdev, dev, ws1, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_score(&P.pr, dev, dev, nullptr, fdev, nullptr, ws1, nullptr) == WKV_ERR_WORKSPACE);
  EXPECT(wkv_score(&P.pr, dev, dev, nullptr, fdev, (char *)dev + 64, ws1, nullptr) == WKV_ERR_WORKSPACE);
  EXPECT(wkv_score(&P.pr, dev, dev, nullptr, fdev, dev, ws1 - 1, nullptr) == WKV_ERR_WORKSPACE);
  EXPECT(wkv_score(nullptr, dev, dev, nullptr, fdev, dev, ws1, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_window_pool(&P.pr, nullptr, fdev, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_topk_windows(&P.pr, fdev, idev, nullptr, idev, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_gather_group(&P.pr, 0, kl, kl, idev, idev, ol, ol, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_gather_group(&P.pr, WKV_MAX_LAYERS + 1, kl, kl, idev, idev, ol, ol, nullptr) == WKV_ERR_INVALID_ARG);
  const void *kl_bad[4] = {dev, nullptr, dev, dev};
  EXPECT(wkv_gather_group(&P.pr, 4, kl_bad, kl, idev, idev, ol, ol, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_compress_group(&P.pr, 0, dev, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws1, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_compress_group(&P.pr, 4, nullptr, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws1, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_compress_groups(&P.pr, 0, 2, qg, nullptr, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws2, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_compress_groups(&P.pr, 2, 64, qg, nullptr, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws2, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_compress_groups(&P.pr, 2, 2, qg, nullptr, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws1, nullptr) == WKV_ERR_WORKSPACE);
  const float *lg_bad[2] = {(const float *)dev, nullptr};
  EXPECT(wkv_compress_groups(&P.pr, 2, 2, qg, lg_bad, nullptr, kl, kl, ol, ol, idev, idev, idev, dev, ws2, nullptr) == WKV_ERR_INVALID_ARG);
  int32_t kg_bad[4] = {64, 65, 0, 64};
  EXPECT(wkv_compress_groups(&P.pr, 2, 2, qg, nullptr, kg_bad, kl, kl, ol, ol, idev, idev, idev, dev, ws2, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_index_jaccard(&P.pr, 0, idev, idev, fdev, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_get_workspace_layout(&P.pr, 1, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_get_dims(&P.pr, nullptr) == WKV_ERR_INVALID_ARG);
  EXPECT(wkv_workspace_bytes(&P.pr, 0) == 0);
  EXPECT(std::strlen(wkv_last_error()) > 0);
  EXPECT(wkv_stub_launches == before);
  // ---- decode -------------------------------------------------------------------------------------------------
  wkv_decode_shape ds; std::memset(&ds, 0, sizeof ds);
  ds.batch = 64; ds.n_q_heads = 32; ds.n_kv_heads = 8; ds.head_dim = 128; ds.dtype = WKV_BF16; ds.capacity = 4200;
  ds.cache_stride_b = 8LL * 4200 * 128; ds.cache_stride_h = 4200 * 128; ds.cache_stride_t = 128;
  const size_t dws = wkv_decode_workspace_bytes(&ds);
  EXPECT(dws > 0);
  EXPECT(wkv_decode_step(&ds, dev, dev, dev, dev, dev, idev, fdev, dev, dws, nullptr) == WKV_OK);
  ds.flags = WKV_DECODE_KEEP_COUNT;
  EXPECT(wkv_decode_step(&ds, dev, dev, dev, dev, dev, idev, fdev, dev, dws, nullptr) == WKV_OK);
  ds.flags = 2;
  EXPECT(wkv_decode_step(&ds, dev, dev, dev, dev, dev, idev, fdev, dev, dws, nullptr) == WKV_ERR_INVALID_ARG);
  ds.flags = 0;
  EXPECT(wkv_decode_step(&ds, dev, dev, dev, dev, dev, idev, fdev, dev, dws - 1, nullptr) == WKV_ERR_WORKSPACE);
  EXPECT(wkv_decode_step(&ds, dev, dev, dev, dev, dev, nullptr, fdev, dev, dws, nullptr) == WKV_ERR_INVALID_ARG);
  before = wkv_stub_launches;
  EXPECT(wkv_decode_step_static(&ds, dev, dev, dev, dev, dev, idev, fdev, nullptr) == WKV_OK);
  EXPECT(wkv_stub_launches == before + 1);
  EXPECT(wkv_decode_step_static(&ds, dev, dev, nullptr, dev, dev, idev, fdev, nullptr) == WKV_ERR_INVALID_ARG);
  ds.batch = 4000;                    // 32000 rows of partial results: beyond the static scratch array
  EXPECT(wkv_decode_workspace_bytes(&ds) > WKV_DECODE_STATIC_SCRATCH_BYTES);
  EXPECT(wkv_decode_step_static(&ds, dev, dev, dev, dev, dev, idev, fdev, nullptr) == WKV_ERR_WORKSPACE);
  EXPECT(wkv_stub_launches == before + 1);
  ds.batch = 64;
  ds.n_q_heads = 72;
  EXPECT(wkv_decode_workspace_bytes(&ds) == 0);
  // ---- budgets (Eq. 5-7) ----------------------------------------------------------------------------------------
  double bud[8];
  EXPECT(wkv_group_budgets(32768.0, 8, 14.0, bud) == WKV_OK);
  double sum = 0; for (double x : bud) sum += x;
  EXPECT(sum > 32767.99 && sum < 32768.01);
  EXPECT(wkv_group_budgets(1.0, 0, 14.0, bud) == WKV_ERR_INVALID_ARG);
  EXPECT(std::strcmp(wkv_status_string(WKV_ERR_HIP), "HIP error") == 0);
  std::printf("%s (%d checks failed)\n", failures ? "FAILED" : "ok", failures);
  return failures ? 1 : 0;
}
