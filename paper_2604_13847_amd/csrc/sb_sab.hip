// Sparsity-aware batching (paper section 4.3, Algorithm 2), host only: the sparsity predictor Spar
// (per length bin, a moving average of the budgets the tuning step produced), the latency weights
// W[i] = Perf.predict(L[i], Spar.predict(L[i])) and the two-level balanced partition over DP ranks
// and micro-batches.  `bin_packing` is the longest-processing-time-first greedy: samples in order of
// decreasing weight (ties: lower index), each to the bin with the smallest load (ties: lower bin).
#include <algorithm>
#include <numeric>

#include "sb_internal.h"

namespace sb {

static int length_bin(const float* edges, int nb, double L) {
  int b = 0;
  while (b + 1 < nb && (double)edges[b + 1] <= L) ++b;  // edges[b] <= L < edges[b+1], clamped to the first / last bin
  return b;
}

static void lpt(const double* w, const int32_t* ids, int n, int nbins, int32_t* bin_of) {
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return w[ids ? ids[a] : a] > w[ids ? ids[b] : b]; });
  std::vector<double> load(nbins, 0.0);
  for (int o : order) {
    int best = 0;
    for (int b = 1; b < nbins; ++b)
      if (load[b] < load[best]) best = b;
    const int i = ids ? ids[o] : o;
    bin_of[i] = best;
    load[best] += w[i];
  }
}

}  // namespace sb

using namespace sb;

extern "C" {

int sb_spar_update(float* ema, uint8_t* seen, const float* bin_edges, int32_t num_bins, double decay, const int32_t* lengths,
                   const int32_t* k_final, int32_t n) {
  if (num_bins < 1 || !ema || !seen || !bin_edges || n < 0 || (n > 0 && (!lengths || !k_final)) || !(decay >= 0.0 && decay <= 1.0)) {
    set_error("bad arguments");
    return SB_ERR_INVALID_ARG;
  }
  for (int i = 0; i < n; ++i) {
    const int b = length_bin(bin_edges, num_bins, (double)lengths[i]);
    // the running value is kept in float; one step is computed in double and rounded once
    ema[b] = seen[b] ? (float)(decay * (double)ema[b] + (1.0 - decay) * (double)k_final[i]) : (float)k_final[i];
    seen[b] = 1;
  }
  return SB_OK;
}

int sb_spar_predict(const float* ema, const uint8_t* seen, const float* bin_edges, int32_t num_bins, int32_t length, double k_base,
                    double* k_out) {
  if (num_bins < 1 || !ema || !seen || !bin_edges || !k_out) { set_error("bad arguments"); return SB_ERR_INVALID_ARG; }
  const int b = length_bin(bin_edges, num_bins, (double)length);
  *k_out = seen[b] ? (double)ema[b] : k_base;
  return SB_OK;
}

int sb_balanced_partition(const double* weights, int32_t n, int32_t num_bins, int32_t* bin_of_out) {
  if (n < 0 || num_bins < 1 || (n > 0 && (!weights || !bin_of_out))) { set_error("bad arguments"); return SB_ERR_INVALID_ARG; }
  lpt(weights, nullptr, n, num_bins, bin_of_out);
  return SB_OK;
}

int sb_sab_batches(const sb_perf_table* perf, const int32_t* lengths, const double* k_pred, int32_t n, int32_t dp_size, int32_t dp_rank,
                   int32_t num_microbatches, double* weights_out, int32_t* dp_bin_out, int32_t* mb_bin_out) {
  if (n < 0 || dp_size < 1 || dp_rank < 0 || dp_rank >= dp_size || num_microbatches < 1 ||
      (n > 0 && (!lengths || !k_pred || !dp_bin_out || !mb_bin_out))) {
    set_error("bad arguments");
    return SB_ERR_INVALID_ARG;
  }
  std::vector<double> w(n);
  for (int i = 0; i < n; ++i) {
    int rc = sb_perf_predict(perf, (double)lengths[i], k_pred[i], &w[i]);
    if (rc != SB_OK) return rc;
    if (weights_out) weights_out[i] = w[i];
  }
  lpt(w.data(), nullptr, n, dp_size, dp_bin_out);
  std::vector<int32_t> mine;
  for (int i = 0; i < n; ++i) {
    mb_bin_out[i] = -1;
    if (dp_bin_out[i] == dp_rank) mine.push_back(i);
  }
  lpt(w.data(), mine.data(), (int)mine.size(), num_microbatches, mb_bin_out);
  return SB_OK;
}

}  // extern "C"
