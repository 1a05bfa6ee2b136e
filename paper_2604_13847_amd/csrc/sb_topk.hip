// Top-K block selection (paper section 2.2): per row (sequence, selection head, query block i)
// keep the diagonal block plus the best c-1 past blocks under the total order
// (score descending, block index ascending; -0 == +0; NaN below everything).
// One workgroup per row: order-preserving 32-bit keys in LDS, a 4-pass radix select for the
// threshold key, then an index-ordered compaction, so the result is a pure function of the scores.
#include "sb_internal.h"

namespace sb {

__device__ inline uint32_t order_key(float x) {
  if (x != x) return 0u;              // NaN: lowest
  if (x == 0.0f) x = 0.0f;            // -0 and +0 share one key
  uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// exclusive prefix sum over the 256 threads of a workgroup; `tmp` holds 8 ints; returns the total in *total
__device__ inline int block_excl_scan_256(int v, int* tmp, int* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int t = __shfl_up(incl, off, 64);
    if (lane >= off) incl += t;
  }
  __syncthreads();  // tmp may still be read from a previous call
  if (lane == 63) tmp[w] = incl;
  __syncthreads();
  int base = 0;
  for (int a = 0; a < w; ++a) base += tmp[a];
  *total = tmp[0] + tmp[1] + tmp[2] + tmp[3];
  return base + incl - v;
}

__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ scores, const int32_t* __restrict__ qb_off,
                                                   const int64_t* __restrict__ sc_off, const int32_t* __restrict__ row_base,
                                                   const int32_t* __restrict__ kclamp, const int32_t* __restrict__ qb_seq,
                                                   int64_t NQB, int Hs, int64_t nnz_unit, int32_t* __restrict__ rowptr,
                                                   int32_t* __restrict__ idx) {
  extern __shared__ uint32_t keys[];  // n_max entries
  __shared__ int hist[256];
  __shared__ int tmp[8];
  __shared__ int sh_bin, sh_above;
  const int tid = threadIdx.x;
  const int qb = blockIdx.x, hs = blockIdx.y;
  const int s = qb_seq[qb];
  const int i = qb - qb_off[s];
  const int n = qb_off[s + 1] - qb_off[s];
  const int k = kclamp[s];
  const int c = min(k, i + 1);
  // closed-form row start: head offset + sequence offset + rows before i in this sequence
  const int m0 = min(i, k);  // rows i' < i with i'+1 <= k contribute i'+1, the rest contribute k
  const int64_t before = (int64_t)m0 * (m0 + 1) / 2 + (int64_t)(i - m0) * k;
  const int64_t start = (int64_t)hs * nnz_unit + row_base[s] + before;
  if (tid == 0) {
    rowptr[(int64_t)hs * NQB + qb] = (int32_t)start;
    if (hs == Hs - 1 && qb == NQB - 1) rowptr[(int64_t)Hs * NQB] = (int32_t)(start + c);
  }
  int32_t* out = idx + start;
  const int need = c - 1, m = i;  // choose `need` of the m past blocks
  if (need == m) {                // everything is kept (also covers need == 0 with i == 0)
    for (int j = tid; j <= i; j += 256) out[j] = j;
    return;
  }
  if (need == 0) {
    if (tid == 0) out[0] = i;
    return;
  }
  const float* row = scores + (int64_t)Hs * sc_off[s] + ((int64_t)hs * n + i) * n;
  for (int j = tid; j < m; j += 256) keys[j] = order_key(row[j]);
  // radix select: the need-th largest key
  uint32_t prefix = 0, mask = 0;
  int remaining = need;
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < m; j += 256) {
      uint32_t kk = keys[j];
      if ((kk & mask) == prefix) atomicAdd(&hist[(kk >> shift) & 255u], 1);
    }
    __syncthreads();
    // thread t looks at bin 255-t: `above` = number of matching keys in higher bins
    int mine = hist[255 - tid], total;
    int above = block_excl_scan_256(mine, tmp, &total);
    if (above < remaining && remaining <= above + mine) { sh_bin = 255 - tid; sh_above = above; }
    __syncthreads();
    prefix |= (uint32_t)sh_bin << shift;
    mask |= 255u << shift;
    remaining -= sh_above;
    __syncthreads();
  }
  // keys > prefix are all kept; of the keys == prefix the `remaining` lowest indices are kept
  const uint32_t thr = prefix;
  const int seg = (m + 255) / 256;
  const int j0 = min(tid * seg, m), j1 = min(j0 + seg, m);
  int eq = 0;
  for (int j = j0; j < j1; ++j) eq += keys[j] == thr;
  int total;
  int eq_before = block_excl_scan_256(eq, tmp, &total);
  int kept = 0;
  {
    int e = eq_before;
    for (int j = j0; j < j1; ++j) {
      uint32_t kk = keys[j];
      kept += (kk > thr) || (kk == thr && e < remaining);
      e += kk == thr;
    }
  }
  int pos = block_excl_scan_256(kept, tmp, &total);
  {
    int e = eq_before;
    for (int j = j0; j < j1; ++j) {
      uint32_t kk = keys[j];
      if ((kk > thr) || (kk == thr && e < remaining)) out[pos++] = j;
      e += kk == thr;
    }
  }
  if (tid == 0) out[need] = i;
}

}  // namespace sb

using namespace sb;

extern "C" int sb_select_topk(const sb_problem* p, const float* scores, int32_t* sel_rowptr_out, int32_t* sel_idx_out,
                              void* ws, void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (!sel_rowptr_out) { set_error("null sel_rowptr_out"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) {
    return fill_zero(sel_rowptr_out, sizeof(int32_t), st);
  }
  if (!scores || !sel_idx_out || !ws) { set_error("null scores, sel_idx_out or ws"); return SB_ERR_INVALID_ARG; }
  rc = launch_geom(g, p, ws, st);
  if (rc != SB_OK) return rc;
  Tables t = make_tables(g, p, ws);
  dim3 grid((unsigned)g.NQB, (unsigned)g.Hs);
  size_t smem = sizeof(uint32_t) * (size_t)(g.n_max + 1);
  if (smem > 48 * 1024) {
    static bool attr_set = false;
    if (!attr_set) {
      SB_CHECK_HIP(hipFuncSetAttribute((const void*)topk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(sizeof(uint32_t) * (SB_MAX_BLOCKS_PER_SEQ + 1))));
      attr_set = true;
    }
  }
  KernelTimer kt(K_TOPK, st);
  hipLaunchKernelGGL(topk_kernel, grid, dim3(256), smem, st, scores, t.qb_off, t.sc_off, t.row_base, t.kclamp, t.qb_seq,
                     g.NQB, g.Hs, g.nnz_unit, sel_rowptr_out, sel_idx_out);
  SB_LAUNCH_CHECK("topk_kernel");
  return SB_OK;
}
