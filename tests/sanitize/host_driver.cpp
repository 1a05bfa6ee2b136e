// Calls every host-only entry point of the library (layout, budget rule, row pointers, plan sections, latency table,
// tuning, batching) on valid, degenerate and invalid problems.  tests/test_sanitizers.py builds it together with the
// library's host code under -fsanitize=address,undefined (host side only) and expects exit status 0.
#include <stdint.h>
#include <stdio.h>

#include <vector>

#include "sparsebal.h"

#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { printf("line %d: %s failed (%s)\n", __LINE__, #cond, sb_last_error()); return 1; } \
  } while (0)

int main() {
  const std::vector<int32_t> lens = {700, 64, 0, 5000, 12000, 1, 2300, 131072};
  std::vector<int32_t> cu(lens.size() + 1, 0);
  for (size_t s = 0; s < lens.size(); ++s) cu[s + 1] = cu[s] + lens[s];
  const int S = (int)lens.size();
  for (int B : {64, 128, 256})
    for (int mode : {SB_SELECT_PER_QHEAD, SB_SELECT_PER_KVGROUP}) {
      std::vector<float> rho = {0.3f, 1.0f, 0.5f, 0.1f, 0.05f, 0.0f, 0.9f, 0.05f};
      std::vector<int32_t> topk(S);
      EXPECT(sb_keep_ratio_to_topk(cu.data(), S, B, rho.data(), topk.data()) == SB_OK);
      sb_problem p{};
      p.total_tokens = cu[S]; p.num_seqs = S; p.num_q_heads = 8; p.num_kv_heads = 2; p.head_dim = 128; p.block_size = B;
      p.dtype = SB_BF16; p.select_mode = mode; p.cu_seqlens_host = cu.data(); p.topk_host = topk.data();
      sb_layout lay{};
      EXPECT(sb_get_layout(&p, &lay) == SB_OK);
      EXPECT(lay.sel_nnz > 0 && lay.plan_bytes > 0 && lay.bwd_ws_bytes > 0);
      std::vector<int32_t> rowptr(lay.sel_rows + 1);
      EXPECT(sb_sel_rowptr_host(&p, rowptr.data()) == SB_OK);
      EXPECT(rowptr[lay.sel_rows] == lay.sel_nnz);
      int64_t sec[SB_PLAN_NUM_SECTIONS];
      EXPECT(sb_plan_sections(&p, sec) == SB_OK);
      EXPECT(sec[SB_PLAN_SPLIT_COLS] < lay.plan_bytes && sec[SB_PLAN_SPLIT_WEIGHT] >= 512);
      // tuning on a synthetic coverage curve: C_s(k) = k / n_s
      std::vector<float> cov(lay.num_qblocks);
      int64_t o = 0;
      for (int s = 0; s < S; ++s) {
        const int n = (lens[s] + B - 1) / B;
        for (int k = 1; k <= n; ++k) cov[o + k - 1] = (float)k / (float)n;
        o += n;
      }
      const float xs[3] = {1024.f, 16384.f, 131072.f}, ks[3] = {1.f, 32.f, 128.f};
      const float lat[9] = {0.1f, 0.3f, 0.9f, 0.5f, 2.6f, 7.5f, 3.f, 20.f, 70.f};
      sb_perf_table tab{3, 3, xs, ks, lat};
      std::vector<int32_t> kf(S), ka(S);
      double ta = 0;
      for (int anchor : {SB_ANCHOR_MIN, SB_ANCHOR_MEAN, SB_ANCHOR_MAX})
        EXPECT(sb_dst_tune(&p, cov.data(), &tab, anchor, 0.1, kf.data(), ka.data(), &ta) == SB_OK);
      double v = 0;
      EXPECT(sb_perf_predict(&tab, 5000.0, 17.0, &v) == SB_OK && v > 0);
      int32_t kb = 0;
      EXPECT(sb_perf_align(&tab, 5000.0, v, 300, &kb) == SB_OK && kb >= 17);
      // batching
      const float edges[4] = {0.f, 2048.f, 16384.f, 1e9f};
      float ema[3] = {0, 0, 0};
      uint8_t seen[3] = {0, 0, 0};
      EXPECT(sb_spar_update(ema, seen, edges, 3, 0.9, lens.data(), kf.data(), S) == SB_OK);
      std::vector<double> kp(S), w(S);
      for (int s = 0; s < S; ++s) EXPECT(sb_spar_predict(ema, seen, edges, 3, lens[s], 8.0, &kp[s]) == SB_OK);
      std::vector<int32_t> dp(S), mb(S), bin(S);
      EXPECT(sb_sab_batches(&tab, lens.data(), kp.data(), S, 2, 1, 2, w.data(), dp.data(), mb.data()) == SB_OK);
      EXPECT(sb_balanced_partition(w.data(), S, 3, bin.data()) == SB_OK);
    }
  // degenerate and invalid problems
  {
    const int32_t cu0[2] = {0, 0}, k1[1] = {1}, kbad[1] = {0}, cubad[2] = {0, 5};
    sb_problem p{};
    p.num_seqs = 1; p.num_q_heads = 4; p.num_kv_heads = 2; p.head_dim = 64; p.block_size = 64;
    p.cu_seqlens_host = cu0; p.topk_host = k1;
    sb_layout lay{};
    EXPECT(sb_get_layout(&p, &lay) == SB_OK && lay.sel_nnz == 0);
    p.topk_host = kbad; p.cu_seqlens_host = cubad; p.total_tokens = 5;
    EXPECT(sb_get_layout(&p, &lay) == SB_ERR_INVALID_ARG);
    p.topk_host = k1; p.head_dim = 96;
    EXPECT(sb_get_layout(&p, &lay) == SB_ERR_UNSUPPORTED);
    p.head_dim = 64; p.num_q_heads = 5;
    EXPECT(sb_get_layout(&p, &lay) == SB_ERR_INVALID_ARG);
    EXPECT(sb_get_layout(nullptr, &lay) == SB_ERR_INVALID_ARG);
    // the entry point without a workspace rejects a problem whose tables exceed its built-in scratch before it
    // touches the device
    std::vector<int32_t> cubig(300001), kbig(300000, 1);
    for (int i = 0; i <= 300000; ++i) cubig[i] = i;
    sb_problem q{};
    q.total_tokens = 300000; q.num_seqs = 300000; q.num_q_heads = 2; q.num_kv_heads = 1; q.head_dim = 64; q.block_size = 64;
    q.cu_seqlens_host = cubig.data(); q.topk_host = kbig.data();
    int32_t dummy[4];
    EXPECT(sb_select_topk_static(&q, (const float*)dummy, dummy, dummy, nullptr) == SB_ERR_WORKSPACE_TOO_SMALL);
  }
  printf("host driver OK (%s)\n", sb_version());
  return 0;
}
