// Budget controller around the attention path (paper section 4.1 and 4.2):
//   sb_score_coverage   coverage curves C_s(k) of the routing scores (Eq. 4) on the GPU
//   sb_perf_predict / sb_perf_align   the profiled latency table (Eq. 8-10), host
//   sb_dst_tune         Algorithm 1 (anchor, Perf.align, coverage threshold p, Eq. 3/5/7), host
//
// Coverage.  For one query block i and one selection head the candidates are the earlier blocks
// j < i; their scores are normalised by a softmax and sorted in descending order; a budget k keeps
// the diagonal block and the k-1 best candidates, so the row covers pref_i[min(k-1, i)], the sum of
// its min(k-1, i) largest shares (pref_i[i] = 1).  C_s(k) is the mean over the sequence's rows.
// All kernels are deterministic (fixed summation order, no atomics):
//   coverage_rows_regs_kernel   rows of at most 2048 candidates: one wavefront per (row, selection head) sorts the row in
//                           registers (bitonic network, cross-lane permutes only at distances of a lane's share and
//                           above), then softmax and prefix sums; summed over the heads of a group into
//                           Pacc[s][i][m-1] = sum_hs pref_{hs,i}[m], m = 1..i
//   coverage_rows_kernel    longer rows: one workgroup per query block and group of selection heads, for every head in
//                           turn softmax + bitonic sort + prefix sum in LDS, into the same Pacc
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

// P compare-exchanges of one bitonic stage per lane (pairs t, t + 64, ...): the pairs of a stage are disjoint, so all
// operands are read before anything is written back and the LDS latencies of the P pairs overlap.
template <int P>
__device__ inline void bitonic_pairs(float* keys, int t0, int j2, int k2) {
  int lo[P];
  float a[P], b[P];
#pragma unroll
  for (int u = 0; u < P; ++u) {
    const int t = t0 + 64 * u;
    lo[u] = ((t & ~(j2 - 1)) << 1) | (t & (j2 - 1));  // j2 is a power of two
    a[u] = keys[lo[u]];
    b[u] = keys[lo[u] + j2];
  }
#pragma unroll
  for (int u = 0; u < P; ++u) {  // branch-free: both elements are written back, swapped or not
    const bool lt = a[u] < b[u], gt = a[u] > b[u];
    const bool swap = (lo[u] & k2) == 0 ? lt : gt;
    keys[lo[u]] = swap ? b[u] : a[u];
    keys[lo[u] + j2] = swap ? a[u] : b[u];
  }
}

__global__ __launch_bounds__(256) void coverage_rows_kernel(const float* __restrict__ scores, const int32_t* __restrict__ qb_off,
                                                            const int64_t* __restrict__ sc_off, const int32_t* __restrict__ qb_seq,
                                                            int Hs, int64_t slab, int min_row, float* __restrict__ pacc) {
  extern __shared__ float smem[];  // keys[N], acc[N], tmp[260]
  const int tid = threadIdx.x;
  const int qb = blockIdx.x;
  const int s = qb_seq[qb];
  const int i = qb - qb_off[s];
  const int n = qb_off[s + 1] - qb_off[s];
  if (i == 0 || i < min_row) return;  // no candidates: the row is fully covered at every budget; short rows: the other kernel's
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
            if (tid < (N >> 1)) bitonic_pairs<1>(keys, tid, j2, k2);  // at most 128 pairs
          } else if (ppw == 64) {
            bitonic_pairs<1>(keys, wave * ppw + lane, j2, k2);
          } else if (ppw == 128) {
            bitonic_pairs<2>(keys, wave * ppw + lane, j2, k2);
          } else {  // a multiple of 256 pairs per wavefront
            for (int t = wave * ppw + lane; t < (wave + 1) * ppw; t += 256) bitonic_pairs<4>(keys, t, j2, k2);
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

// The same rows for sequences of at most kCovRegMax blocks, sorted in registers: one wavefront per (row, selection
// head), 64 E = N keys (N the row length rounded up to a power of two, at least 64), E per lane.  Key number lane * E + r
// of the bitonic network lives in register r of the lane, so the compare-exchanges at distances below E stay inside a lane
// (two instructions per pair, no memory) and only those at distances E and above cross lanes (one permute each); a
// wavefront alone needs no barrier.  A block of the network that sorts ascending is handled by negating its lanes' keys,
// so that every compare-exchange puts the larger key first.  The four wavefronts of a workgroup take the heads of the
// group in turn, keep their sums in registers and add them in wavefront order at the end: fixed summation order again.
// Scores must be numbers (a NaN is dropped by the max/min of a compare-exchange); sb_block_scores writes none for finite
// inputs.
constexpr int kCovRegMax = 2048;

template <int E>
__device__ __forceinline__ void coverage_row_regs(const float* __restrict__ row, int i, int lane, float (&acc)[E]) {
  float x[E];
#pragma unroll
  for (int r = 0; r < E; ++r) x[r] = r * 64 + lane < i ? row[r * 64 + lane] : -INFINITY;  // any initial placement will do
  // phases k2 = 2 .. E/2: inside a lane, directions known at compile time (bit k2 of r)
#pragma unroll
  for (int k2 = 2; k2 < E; k2 <<= 1) {
#pragma unroll
    for (int j2 = k2 >> 1; j2 > 0; j2 >>= 1) {
#pragma unroll
      for (int r = 0; r < E; ++r) {
        if ((r & j2) == 0) {
          const float hi = fmaxf(x[r], x[r | j2]), lo = fminf(x[r], x[r | j2]);
          const bool desc = (r & k2) == 0;
          x[r] = desc ? hi : lo;
          x[r | j2] = desc ? lo : hi;
        }
      }
      __builtin_amdgcn_sched_barrier(0);  // (left alone, the scheduler interleaves the stages and triples the register count)
    }
  }
  // phases k2 = E .. 64 E: the direction is bit k2 / E of the lane; ascending lanes work on negated keys
  bool negated = false;
#pragma unroll 1
  for (int t = (E > 1 ? 0 : 1); t <= 6; ++t) {
    const bool want = ((lane >> t) & 1) != 0 && t < 6;  // (the last phase, k2 = N, is descending everywhere)
    const uint32_t flip = want != negated ? 0x80000000u : 0u;
    negated = want;
#pragma unroll
    for (int r = 0; r < E; ++r) x[r] = __uint_as_float(__float_as_uint(x[r]) ^ flip);
    for (int d = (1 << t) >> 1; d > 0; d >>= 1) {  // distances d * E: lane l against lane l ^ d
      const int partner = (lane ^ d) << 2;
      const bool first = (lane & d) == 0;
      constexpr int C = E < 8 ? E : 8;  // registers exchanged at a time (keeps the values in flight few)
#pragma unroll
      for (int r0 = 0; r0 < E; r0 += C) {
        float y[C];
#pragma unroll
        for (int r = 0; r < C; ++r) y[r] = __int_as_float(__builtin_amdgcn_ds_bpermute(partner, __float_as_int(x[r0 + r])));
#pragma unroll
        for (int r = 0; r < C; ++r) {
          const float hi = fmaxf(x[r0 + r], y[r]), lo = fminf(x[r0 + r], y[r]);
          x[r0 + r] = first ? hi : lo;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int j2 = E >> 1; j2 > 0; j2 >>= 1) {
#pragma unroll
      for (int r = 0; r < E; ++r) {
        if ((r & j2) == 0) {
          const float hi = fmaxf(x[r], x[r | j2]), lo = fminf(x[r], x[r | j2]);
          x[r] = hi;
          x[r | j2] = lo;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // shares in sorted order (key 0 is the row maximum), their running sum, the coverage of every prefix
  const float mx = __shfl(x[0], 0, 64);
  float run = 0.f;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    x[r] = lane * E + r < i ? __expf(x[r] - mx) : 0.f;
    run += x[r];
  }
  float incl = run;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const float up = __shfl_up(incl, off, 64);
    if (lane >= off) incl += up;
  }
  const float inv = 1.0f / __shfl(incl, 63, 64);
  run = incl - run;  // the shares of the lanes before this one
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int p = lane * E + r;
    run += x[r];
    if (p < i) acc[r] += p == i - 1 ? 1.0f : run * inv;
  }
}

template <int E>
__device__ __forceinline__ void coverage_rows_regs_body(const float* __restrict__ scores_s, int n, int i, int hs0, int hs1, float* part,
                                               float* __restrict__ out) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  float acc[E];
#pragma unroll
  for (int r = 0; r < E; ++r) acc[r] = 0.f;
  for (int hs = hs0 + wave; hs < hs1; hs += 4) coverage_row_regs<E>(scores_s + ((int64_t)hs * n + i) * n, i, lane, acc);
#pragma unroll
  for (int r = 0; r < E; ++r) part[wave * kCovRegMax + lane * E + r] = acc[r];
  __syncthreads();
  for (int p = tid; p < i; p += 256)
    out[p] = ((part[p] + part[kCovRegMax + p]) + part[2 * kCovRegMax + p]) + part[3 * kCovRegMax + p];
}

__global__ __launch_bounds__(256) void coverage_rows_regs_kernel(const float* __restrict__ scores, const int32_t* __restrict__ qb_off,
                                                                 const int64_t* __restrict__ sc_off, const int32_t* __restrict__ qb_seq,
                                                                 int Hs, int64_t slab, float* __restrict__ pacc) {
  __shared__ float part[4 * kCovRegMax];
  const int qb = blockIdx.x;
  const int s = qb_seq[qb];
  const int i = qb - qb_off[s];
  const int n = qb_off[s + 1] - qb_off[s];
  if (i == 0 || i > kCovRegMax) return;  // no candidates; longer rows are left to coverage_rows_kernel
  const int hpg = (Hs + (int)gridDim.y - 1) / (int)gridDim.y;  // selection heads per group
  const int hs0 = blockIdx.y * hpg, hs1 = min(Hs, hs0 + hpg);
  const float* scores_s = scores + (int64_t)Hs * sc_off[s];
  float* out = pacc + (int64_t)blockIdx.y * slab + sc_off[s] + (int64_t)i * n;
  if (i <= 64) coverage_rows_regs_body<1>(scores_s, n, i, hs0, hs1, part, out);
  else if (i <= 128) coverage_rows_regs_body<2>(scores_s, n, i, hs0, hs1, part, out);
  else if (i <= 256) coverage_rows_regs_body<4>(scores_s, n, i, hs0, hs1, part, out);
  else if (i <= 512) coverage_rows_regs_body<8>(scores_s, n, i, hs0, hs1, part, out);
  else if (i <= 1024) coverage_rows_regs_body<16>(scores_s, n, i, hs0, hs1, part, out);
  else coverage_rows_regs_body<32>(scores_s, n, i, hs0, hs1, part, out);
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
  hipLaunchKernelGGL(coverage_rows_regs_kernel, dim3((unsigned)g.NQB, (unsigned)groups), dim3(256), 0, st, scores, t.qb_off, t.sc_off,
                     t.qb_seq, g.Hs, slab, pacc);
  SB_LAUNCH_CHECK("coverage_rows_regs_kernel");
  if (g.n_max > kCovRegMax + 1) {  // rows with more than kCovRegMax candidates
    hipLaunchKernelGGL(coverage_rows_kernel, dim3((unsigned)g.NQB, (unsigned)groups), dim3(256), smem, st, scores, t.qb_off, t.sc_off,
                       t.qb_seq, g.Hs, slab, kCovRegMax + 1, pacc);
    SB_LAUNCH_CHECK("coverage_rows_kernel");
  }
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
