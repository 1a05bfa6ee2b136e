// Budget controller around the attention path (paper section 4.1 and 4.2):
//   sb_score_coverage   coverage curves C_s(k) of the routing scores (Eq. 4) on the GPU
//   sb_perf_predict / sb_perf_align   the profiled latency table (Eq. 8-10), host
//   sb_dst_tune         Algorithm 1 (anchor, Perf.align, coverage threshold p, Eq. 3/5/7), host
//
// Coverage.  For one query block i and one selection head the candidates are the earlier blocks
// j < i; their scores are normalised by a softmax and sorted in descending order; a budget k keeps
// the diagonal block and the k-1 best candidates, so the row covers pref_i[min(k-1, i)], the sum of
// its min(k-1, i) largest shares (pref_i[i] = 1).  C_s(k) is the mean over the sequence's rows.
// Two kernels, both deterministic (fixed summation order, no atomics):
//   coverage_rows_kernel    one workgroup per query block (s, i) and group of selection heads: for every head in turn,
//                           softmax + bitonic sort + prefix sum in LDS, summed over heads into
//                           Pacc[s][i][m-1] = sum_hs pref_{hs,i}[m], m = 1..i
//   coverage_partial_kernel / coverage_reduce_kernel   one thread per (s, k): column sums of Pacc over slabs of 32 query
//                           blocks, then C_s(k) = (Hs*k + sum_{i>=k} Pacc[s][i][k-2]) / (Hs*n) (the k rows i < k are fully covered)
#include <math.h>

#include <mutex>

#include "sb_internal.h"

namespace sb {

__device__ inline float block_reduce_256(float v, float* tmp, bool is_max) {
  const int tid = threadIdx.x;
  for (int off = 32; off > 0; off >>= 1) {
    const float o = __shfl_xor(v, off, 64);
    v = is_max ? fmaxf(v, o) : v + o;
  }
  __syncthreads();
  if ((tid & 63) == 0) tmp[tid >> 6] = v;
  __syncthreads();
  float r = tmp[0];
  for (int w = 1; w < 4; ++w) r = is_max ? fmaxf(r, tmp[w]) : r + tmp[w];
  return r;  // the same value, combined in the same order, in every thread
}

__global__ __launch_bounds__(256) void coverage_rows_kernel(const float* __restrict__ scores, const int32_t* __restrict__ qb_off,
                                                            const int64_t* __restrict__ sc_off, const int32_t* __restrict__ qb_seq,
                                                            int Hs, int64_t slab, float* __restrict__ pacc) {
  extern __shared__ float smem[];  // keys[N], acc[N], tmp[260]
  const int tid = threadIdx.x;
  const int qb = blockIdx.x;
  const int s = qb_seq[qb];
  const int i = qb - qb_off[s];
  const int n = qb_off[s + 1] - qb_off[s];
  if (i == 0) return;  // no candidates: the row is fully covered at every budget
  int N = 1;
  while (N < i) N <<= 1;
  float* keys = smem;
  float* acc = smem + N;
  float* tmp = smem + 2 * N;
  for (int j = tid; j < i; j += 256) acc[j] = 0.f;
  const int chunk = (N + 255) / 256;  // contiguous elements per thread in the prefix sum
  const int hpg = (Hs + (int)gridDim.y - 1) / (int)gridDim.y;  // selection heads per group
  const int hs0 = blockIdx.y * hpg, hs1 = min(Hs, hs0 + hpg);
  for (int hs = hs0; hs < hs1; ++hs) {
    const float* row = scores + (int64_t)Hs * sc_off[s] + ((int64_t)hs * n + i) * n;
    float mx = -INFINITY;
    for (int j = tid; j < N; j += 256) {
      const float x = j < i ? row[j] : -INFINITY;
      keys[j] = x;
      mx = fmaxf(mx, x);
    }
    mx = block_reduce_256(mx, tmp, true);
    // Bitonic sort, descending.  Pair p of a stage with compare distance j2 is (lo, lo + j2), lo = (p / j2) * 2 j2 + p % j2.
    // The pairs are dealt to the four wavefronts in contiguous quarters: as long as j2 < N / 4 both elements of every
    // pair of wavefront w lie in its own quarter of the keys, and so did the pairs that last wrote them, so the stage
    // needs no workgroup barrier (the LDS operations of one wavefront complete in issue order); only the stages with
    // j2 >= N / 4 (three of 66 for 2048 keys) exchange data between wavefronts.
    {
      const int wave = tid >> 6, lane = tid & 63;
      const int ppw = N >> 3;  // pairs per wavefront (N >= 8 here: smaller rows take the plain loop)
      bool shared_prev = true;  // the keys were written by all threads above
      for (int k2 = 2; k2 <= N; k2 <<= 1) {
        for (int j2 = k2 >> 1; j2 > 0; j2 >>= 1) {
          const bool shared = N < 512 || j2 >= (N >> 2);
          if (shared || shared_prev) __syncthreads(); else asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          shared_prev = shared;
          if (N < 512) {
            for (int t = tid; t < (N >> 1); t += 256) {
              const int lo = ((t & ~(j2 - 1)) << 1) | (t & (j2 - 1)), hi = lo + j2;  // j2 is a power of two
              const bool desc = (lo & k2) == 0;
              const float a = keys[lo], b = keys[hi];
              if (desc ? a < b : a > b) { keys[lo] = b; keys[hi] = a; }
            }
          } else {
            for (int t = wave * ppw + lane; t < (wave + 1) * ppw; t += 64) {
              const int lo = ((t & ~(j2 - 1)) << 1) | (t & (j2 - 1)), hi = lo + j2;  // j2 is a power of two
              const bool desc = (lo & k2) == 0;
              const float a = keys[lo], b = keys[hi];
              if (desc ? a < b : a > b) { keys[lo] = b; keys[hi] = a; }
            }
          }
        }
      }
    }
    __syncthreads();
    // shares in sorted order, their total, and the running sum
    float part = 0.f;
    const int c0 = tid * chunk, c1 = min(c0 + chunk, N);
    for (int j = c0; j < c1; ++j) {
      const float e = j < i ? __expf(keys[j] - mx) : 0.f;
      keys[j] = e;
      part += e;
    }
    // exclusive prefix of the 256 partial sums: shuffle scan inside each wavefront, then the four wavefront totals
    float incl = part;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const float up = __shfl_up(incl, off, 64);
      if ((tid & 63) >= off) incl += up;
    }
    __syncthreads();
    if ((tid & 63) == 63) tmp[tid >> 6] = incl;
    __syncthreads();
    float before = incl - part, total = 0.f;
    for (int w = 0; w < 4; ++w) {
      if (w < (tid >> 6)) before += tmp[w];
      total += tmp[w];
    }
    const float inv = 1.0f / total;
    float run = before;
    for (int j = c0; j < c1; ++j) {
      run += keys[j];
      if (j < i) acc[j] += j == i - 1 ? 1.0f : run * inv;
    }
    __syncthreads();
  }
  float* out = pacc + (int64_t)blockIdx.y * slab + sc_off[s] + (int64_t)i * n;
  for (int j = tid; j < i; j += 256) out[j] = acc[j];
}

// partial column sums over slabs of kCovSlab query blocks: part[y][qb] = sum over head groups and rows i of slab y, i >= k
constexpr int kCovSlab = 32;
__global__ __launch_bounds__(256) void coverage_partial_kernel(const float* __restrict__ pacc, const int32_t* __restrict__ qb_off,
                                                               const int64_t* __restrict__ sc_off, const int32_t* __restrict__ qb_seq,
                                                               int64_t NQB, int groups, int64_t slab, float* __restrict__ part) {
  const int64_t qb = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (qb >= NQB) return;
  const int s = qb_seq[qb];
  const int n = qb_off[s + 1] - qb_off[s];
  const int k = (int)(qb - qb_off[s]) + 1;
  const int i0 = max(k, (int)blockIdx.y * kCovSlab), i1 = min(n, ((int)blockIdx.y + 1) * kCovSlab);
  float sum = 0.f;
  if (k >= 2) {
    for (int gidx = 0; gidx < groups; ++gidx) {
      const float* col = pacc + (int64_t)gidx * slab + sc_off[s] + (k - 2);
      for (int i = i0; i < i1; ++i) sum += col[(int64_t)i * n];
    }
  }
  part[(int64_t)blockIdx.y * NQB + qb] = sum;
}

__global__ __launch_bounds__(256) void coverage_reduce_kernel(const float* __restrict__ part, const int32_t* __restrict__ qb_off,
                                                              const int32_t* __restrict__ qb_seq, int64_t NQB, int Hs,
                                                              float* __restrict__ cov) {
  const int64_t qb = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (qb >= NQB) return;
  const int s = qb_seq[qb];
  const int n = qb_off[s + 1] - qb_off[s];
  const int k = (int)(qb - qb_off[s]) + 1;
  double sum = (double)Hs * k;  // the k rows i < k are fully covered
  for (int y = k / kCovSlab; y * kCovSlab < n; ++y) sum += (double)part[(int64_t)y * NQB + qb];
  cov[qb] = (float)(sum / ((double)Hs * n));
}

// selection heads are processed in up to kCovGroups groups by separate workgroups (one slab of partial sums each)
constexpr int kCovGroups = 4;
static int coverage_groups(const Geo& g) { return g.Hs < kCovGroups ? g.Hs : kCovGroups; }
static size_t coverage_slab(const Geo& g) { return align_up(sizeof(float) * (size_t)(g.scores_unit + 1)) / sizeof(float); }
static int coverage_row_slabs(const Geo& g) { return (g.n_max + kCovSlab - 1) / kCovSlab; }
size_t coverage_ws_bytes(const Geo& g) {
  return align_up(table_offsets(g).bytes) + sizeof(float) * coverage_slab(g) * (size_t)coverage_groups(g) +
         align_up(sizeof(float) * (size_t)(coverage_row_slabs(g) * g.NQB + 1));
}

// ---- latency table (host, double arithmetic)
static void bracket(const float* grid, int n, double v, int* a, double* w) {
  if (n == 1 || v <= (double)grid[0]) { *a = 0; *w = 0.0; return; }
  if (v >= (double)grid[n - 1]) { *a = n - 2; *w = 1.0; return; }
  int lo = 0;
  while (lo + 1 < n && (double)grid[lo + 1] <= v) ++lo;  // last bucket edge <= v
  *a = lo;
  *w = (v - (double)grid[lo]) / ((double)grid[lo + 1] - (double)grid[lo]);
}

static int check_table(const sb_perf_table* t) {
  if (!t || t->num_lengths < 1 || t->num_budgets < 1 || !t->lengths || !t->budgets || !t->latency) {
    set_error("bad latency table");
    return SB_ERR_INVALID_ARG;
  }
  for (int a = 1; a < t->num_lengths; ++a)
    if (!(t->lengths[a] > t->lengths[a - 1])) { set_error("latency table: lengths must increase"); return SB_ERR_INVALID_ARG; }
  for (int b = 1; b < t->num_budgets; ++b)
    if (!(t->budgets[b] > t->budgets[b - 1])) { set_error("latency table: budgets must increase"); return SB_ERR_INVALID_ARG; }
  return SB_OK;
}

static double predict(const sb_perf_table* t, double x, double k) {
  int a, b;
  double wa, wb;
  bracket(t->lengths, t->num_lengths, x, &a, &wa);
  bracket(t->budgets, t->num_budgets, k, &b, &wb);
  const int a2 = a + 1 < t->num_lengths ? a + 1 : t->num_lengths - 1, b2 = b + 1 < t->num_budgets ? b + 1 : t->num_budgets - 1;
  const int nk = t->num_budgets;
  const double lo = (1.0 - wb) * (double)t->latency[a * nk + b] + wb * (double)t->latency[a * nk + b2];
  const double hi = (1.0 - wb) * (double)t->latency[a2 * nk + b] + wb * (double)t->latency[a2 * nk + b2];
  return (1.0 - wa) * lo + wa * hi;
}

static int align(const sb_perf_table* t, double x, double target, int kmax) {
  int best = 1;
  for (int k = 1; k <= kmax; ++k)
    if (predict(t, x, (double)k) <= target) best = k;
  return best;
}

}  // namespace sb

using namespace sb;

extern "C" {

int sb_score_coverage(const sb_problem* p, const float* scores, float* coverage_out, void* ws, void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) return SB_OK;
  if (!scores || !coverage_out || !ws) { set_error("null scores, coverage_out or ws"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  rc = launch_geom(g, p, ws, st);
  if (rc != SB_OK) return rc;
  Tables t = make_tables(g, p, ws);
  float* pacc = (float*)((char*)ws + align_up(table_offsets(g).bytes));
  int N = 1;
  while (N < g.n_max) N <<= 1;
  const size_t smem = sizeof(float) * (size_t)(2 * N + 264);
  if (smem > 48 * 1024) {  // raise the kernel's dynamic LDS limit; once per device, whichever thread comes first
    static std::mutex mu;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    SB_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d out of range", dev); return SB_ERR_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(mu);
    if (!attr_set[dev]) {
      SB_CHECK_HIP(hipFuncSetAttribute((const void*)coverage_rows_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(sizeof(float) * (2 * SB_MAX_BLOCKS_PER_SEQ + 264))));
      attr_set[dev] = true;
    }
  }
  KernelTimer kt(K_COVERAGE, st);
  const int groups = coverage_groups(g);
  const int64_t slab = (int64_t)coverage_slab(g);
  hipLaunchKernelGGL(coverage_rows_kernel, dim3((unsigned)g.NQB, (unsigned)groups), dim3(256), smem, st, scores, t.qb_off, t.sc_off,
                     t.qb_seq, g.Hs, slab, pacc);
  SB_LAUNCH_CHECK("coverage_rows_kernel");
  float* part = pacc + slab * groups;
  hipLaunchKernelGGL(coverage_partial_kernel, dim3((unsigned)((g.NQB + 255) / 256), (unsigned)coverage_row_slabs(g)), dim3(256), 0, st, pacc,
                     t.qb_off, t.sc_off, t.qb_seq, g.NQB, groups, slab, part);
  SB_LAUNCH_CHECK("coverage_partial_kernel");
  hipLaunchKernelGGL(coverage_reduce_kernel, dim3((unsigned)((g.NQB + 255) / 256)), dim3(256), 0, st, part, t.qb_off, t.qb_seq, g.NQB, g.Hs,
                     coverage_out);
  SB_LAUNCH_CHECK("coverage_reduce_kernel");
  return SB_OK;
}

int sb_perf_predict(const sb_perf_table* t, double length, double budget, double* latency_out) {
  int rc = check_table(t);
  if (rc != SB_OK) return rc;
  if (!latency_out) { set_error("null latency_out"); return SB_ERR_INVALID_ARG; }
  *latency_out = predict(t, length, budget);
  return SB_OK;
}

int sb_perf_align(const sb_perf_table* t, double length, double target_latency, int32_t max_budget, int32_t* budget_out) {
  int rc = check_table(t);
  if (rc != SB_OK) return rc;
  if (!budget_out || max_budget < 1) { set_error("bad budget_out or max_budget"); return SB_ERR_INVALID_ARG; }
  *budget_out = align(t, length, target_latency, max_budget);
  return SB_OK;
}

int sb_dst_tune(const sb_problem* p, const float* coverage_host, const sb_perf_table* perf, int anchor, double threshold_p,
                int32_t* topk_final_out, int32_t* topk_anchor_out, double* t_anchor_out) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if ((rc = check_table(perf)) != SB_OK) return rc;
  if (anchor != SB_ANCHOR_MIN && anchor != SB_ANCHOR_MEAN && anchor != SB_ANCHOR_MAX) { set_error("bad anchor %d", anchor); return SB_ERR_INVALID_ARG; }
  if (g.S > 0 && (!coverage_host || !topk_final_out)) { set_error("null coverage_host or topk_final_out"); return SB_ERR_INVALID_ARG; }
  std::vector<int> n(g.S), kb(g.S);
  std::vector<double> T;
  for (int s = 0; s < g.S; ++s) {
    const int64_t L = (int64_t)p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
    n[s] = (int)((L + g.B - 1) / g.B);
    const int cap = n[s] > 1 ? n[s] : 1;
    kb[s] = p->topk_host[s] < cap ? p->topk_host[s] : cap;
    if (n[s] > 0) T.push_back(predict(perf, (double)L, (double)kb[s]));
  }
  double Ta = 0.0;
  if (!T.empty()) {
    if (anchor == SB_ANCHOR_MEAN) {
      double sum = 0.0;
      for (double v : T) sum += v;
      Ta = sum / (double)T.size();
    } else {
      Ta = T[0];
      for (double v : T) Ta = anchor == SB_ANCHOR_MIN ? (v < Ta ? v : Ta) : (v > Ta ? v : Ta);
    }
  }
  if (t_anchor_out) *t_anchor_out = Ta;
  int64_t off = 0;
  for (int s = 0; s < g.S; ++s) {
    int kf = kb[s], ka = kb[s];
    if (n[s] > 0) {
      const int64_t L = (int64_t)p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
      const float* C = coverage_host + off;
      ka = align(perf, (double)L, Ta, n[s]);
      kf = ka;
      if ((double)C[kb[s] - 1] - (double)C[ka - 1] > threshold_p) {
        for (int k = 1; k <= n[s]; ++k)
          if ((double)C[kb[s] - 1] - (double)C[k - 1] <= threshold_p) { kf = k; break; }
      }
    }
    topk_final_out[s] = kf;
    if (topk_anchor_out) topk_anchor_out[s] = ka;
    off += n[s];
  }
  return SB_OK;
}

}  // extern "C"
