// Work plan: longest-first ordering of the query-major items, the key-major transpose of the
// selection as a bitmap, and heaviest-first ordering of the key-major columns (per KV head).
//
// Query-major items.  Item (s,hs,i) costs c = min(k_s, i+1) selected tiles.  Because the cost is a
// closed form of (k_s, n_s, i), the rank of an item in the order (cost descending, then sequence,
// then query block, then head with the KV head fastest) is a closed form too: every thread
// computes its own rank with one pass over the S sequences, without sorting or atomics.  Adjacent
// ranks differ in the KV head first, so with workgroups dealt round-robin to the 8 XCDs each XCD's
// L2 keeps seeing the same KV heads.
//
// Key-major transpose.  Bit i of word (s,hs,j,i/32) says query block i kept key block j; the bitmap
// is a pure function of the selection, so the backward pass walks a column's query blocks in a
// fixed order and accumulates deterministically.
#include "sb_internal.h"

namespace sb {

__global__ __launch_bounds__(256) void plan_fwd_kernel(const int32_t* __restrict__ qb_off, const int32_t* __restrict__ kclamp,
                                                       const int32_t* __restrict__ qb_seq, const int32_t* __restrict__ cu,
                                                       const int32_t* __restrict__ rowptr, int S, int64_t NQB, int Hs,
                                                       int Hkv, int G, int mode, int32_t* __restrict__ work_fwd,
                                                       WorkItem* __restrict__ items) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;  // row id = hs*NQB + qb
  if (row >= (int64_t)Hs * NQB) return;
  const int hs = (int)(row / NQB);
  const int qb = (int)(row - (int64_t)hs * NQB);
  const int s = qb_seq[qb];
  const int i = qb - qb_off[s];
  const int ks = kclamp[s];
  const int c = min(ks, i + 1);
  int64_t pos = 0;
  for (int t = 0; t < S; ++t) {
    const int nt = qb_off[t + 1] - qb_off[t], kt = kclamp[t];
    if (nt == 0) continue;
    if (kt > c) pos += (int64_t)Hs * (nt - c);                          // items of t with larger cost
    if (t < s) pos += (int64_t)Hs * (kt == c ? nt - c + 1 : (kt > c ? 1 : 0));  // equal cost, earlier sequence
  }
  int hrank;  // order of the selection heads inside one query block: KV head fastest
  if (mode == SB_SELECT_PER_QHEAD) hrank = (hs % G) * Hkv + hs / G; else hrank = hs;
  pos += (c < ks) ? hrank : (int64_t)(i - (ks - 1)) * Hs + hrank;
  work_fwd[pos] = (int32_t)row;
  WorkItem it;
  it.row = (int32_t)row; it.seq0 = cu[s]; it.len = cu[s + 1] - cu[s]; it.i = i;
  it.e0 = rowptr[row]; it.ntiles = rowptr[row + 1] - it.e0; it.hs = hs; it.s = s;
  items[pos] = it;
}

// One workgroup per (selection head, sequence, 32 consecutive query blocks) builds word i/32 of
// every column of the sequence in LDS (LDS atomics) and then stores it: every bitmap word has one
// owner, so the bitmap needs neither clearing nor global atomics; the column weights get one global
// add per non-empty word instead of one per selected tile.
constexpr int kTrChunk = 8192;  // columns handled per pass (32 KiB of LDS)
__global__ __launch_bounds__(256) void plan_transpose_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ idx,
                                                             const int32_t* __restrict__ qb_off, const int64_t* __restrict__ bm_off,
                                                             int S, int64_t NQB, int Hs, int G, int mode,
                                                             uint32_t* __restrict__ bitmap, int32_t* __restrict__ colcost) {
  __shared__ uint32_t wcol[kTrChunk];
  __shared__ int sh_s, sh_w;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  if (tid == 0) {
    int x = blockIdx.x, s = 0;
    for (; s < S; ++s) {
      const int w = (qb_off[s + 1] - qb_off[s] + 31) >> 5;
      if (x < w) break;
      x -= w;
    }
    sh_s = s; sh_w = x;
  }
  __syncthreads();
  const int s = sh_s, wi = sh_w;
  if (s >= S) return;
  const int hs = blockIdx.y;
  const int n = qb_off[s + 1] - qb_off[s];
  const int w = (n + 31) >> 5;
  uint32_t* bm = bitmap + (int64_t)Hs * bm_off[s] + (int64_t)hs * n * w;
  const int g = mode == SB_SELECT_PER_QHEAD ? hs / G : hs;
  const int weight = mode == SB_SELECT_PER_QHEAD ? 1 : G;  // query-head tiles an entry stands for
  int32_t* cost = colcost + (int64_t)g * NQB + qb_off[s];
  const int64_t row0 = (int64_t)hs * NQB + qb_off[s] + 32 * wi;
  const int nrows = min(32, n - 32 * wi);
  for (int j0 = 0; j0 < n; j0 += kTrChunk) {
    const int nj = min(kTrChunk, n - j0);
    for (int j = tid; j < nj; j += 256) wcol[j] = 0u;
    __syncthreads();
    for (int r = wave; r < nrows; r += 4)
      for (int e = rowptr[row0 + r] + lane; e < rowptr[row0 + r + 1]; e += 64) {
        const int j = idx[e] - j0;
        if (j >= 0 && j < nj) atomicOr(&wcol[j], 1u << r);
      }
    __syncthreads();
    for (int j = tid; j < nj; j += 256) {
      const uint32_t x = wcol[j];
      bm[(int64_t)(j0 + j) * w + wi] = x;
      if (x) atomicAdd(&cost[j0 + j], weight * __popc(x));
    }
    __syncthreads();
  }
}

// Key-major items are ordered heaviest first separately for every KV head g, and the Hkv lists are
// interleaved (position = rank_in_g * Hkv + g).  Neighbouring workgroups of one KV head then walk
// neighbouring key blocks of one sequence and meet the same Q/dO tiles in the L2 of their XCD at
// about the same time, while the heaviest-first rule still holds inside each list.
// An item is a whole column, or, for a column heavier than `wmax` tiles, one of its parts: the column's
// bitmap words are walked from the last query block down (the order the backward kernel uses) and a part
// closes as soon as it has gathered wmax tiles (see ColItem).  A column kept by every query block of a
// long sequence (an attention sink) would otherwise be one workgroup's job for longer than the rest of
// the launch takes.
// One workgroup per KV head: a counting sort on the item weight in LDS (histogram, suffix sums,
// scatter); items of equal weight end up in no particular order.
struct ColumnWalk {
  const uint32_t* bm;  // first bitmap word of the column's first selection head
  int64_t head_stride; // words between the same column of consecutive selection heads
  int nsel, hpe, words, wj;
  __device__ inline int word_weight(int w) const {
    int t = 0;
    for (int sel = 0; sel < nsel; ++sel) t += __popc(bm[sel * head_stride + w]);
    return t * hpe;
  }
  // calls emit(lo, hi, weight) for every part, last query blocks first; returns the number of parts
  template <typename F>
  __device__ inline int parts(int wmax, F emit) const {
    int acc = 0, hi = words, np = 0;
    for (int w = words - 1; w >= wj; --w) {
      acc += word_weight(w);
      if (acc >= wmax && w > wj) { emit(w, hi, acc); hi = w; acc = 0; ++np; }
    }
    emit(wj, hi, acc);
    return np + 1;
  }
};

__global__ __launch_bounds__(1024) void plan_bwd_order_kernel(const int32_t* __restrict__ colcost, const uint32_t* __restrict__ bitmap,
                                                              const int32_t* __restrict__ qb_off, const int32_t* __restrict__ qb_seq,
                                                              const int64_t* __restrict__ bm_off, int64_t NQB, int Hkv, int Hs, int G,
                                                              int mode, int wmax, ColItem* __restrict__ items,
                                                              int32_t* __restrict__ counters, int32_t* __restrict__ split_cols) {
  __shared__ int bins[kBwdBins];
  __shared__ int sh[1024];
  const int tid = threadIdx.x;
  const int64_t g = blockIdx.x;
  const int32_t* cost = colcost + g * NQB;
  auto walk_of = [&](int64_t c) {
    ColumnWalk cw;
    const int s = qb_seq[c], j = (int)(c - qb_off[s]), n = qb_off[s + 1] - qb_off[s];
    cw.words = (n + 31) >> 5;
    cw.wj = j >> 5;
    cw.nsel = mode == SB_SELECT_PER_QHEAD ? G : 1;
    cw.hpe = mode == SB_SELECT_PER_QHEAD ? 1 : G;
    const int64_t hs0 = mode == SB_SELECT_PER_QHEAD ? g * G : g;
    cw.head_stride = (int64_t)n * cw.words;
    cw.bm = bitmap + (int64_t)Hs * bm_off[s] + (hs0 * n + j) * cw.words;
    return cw;
  };
  for (int b = tid; b < kBwdBins; b += 1024) bins[b] = 0;
  __syncthreads();
  for (int64_t c = tid; c < NQB; c += 1024) {
    if (cost[c] <= wmax) {
      atomicAdd(&bins[min(cost[c], kBwdBins - 1)], 1);
    } else {
      walk_of(c).parts(wmax, [&](int, int, int wt) { atomicAdd(&bins[min(wt, kBwdBins - 1)], 1); });
    }
  }
  __syncthreads();
  // bins[b] <- number of items with a bin > b; thread t owns bins (kBwdBins-1 - t*per) downwards
  constexpr int per = kBwdBins / 1024;
  int v[per], sum = 0;
#pragma unroll
  for (int a = 0; a < per; ++a) { v[a] = bins[kBwdBins - 1 - (tid * per + a)]; sum += v[a]; }
  sh[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {
    const int t = tid >= off ? sh[tid - off] : 0;
    __syncthreads();
    sh[tid] += t;
    __syncthreads();
  }
  int run = sh[tid] - sum;
#pragma unroll
  for (int a = 0; a < per; ++a) { bins[kBwdBins - 1 - (tid * per + a)] = run; run += v[a]; }
  __syncthreads();
  for (int64_t c = tid; c < NQB; c += 1024) {
    const int32_t col = (int32_t)(g * NQB + c);
    const ColumnWalk cw = walk_of(c);
    int np = 1;
    if (cost[c] > wmax) np = cw.parts(wmax, [](int, int, int) {});
    if (np == 1) {
      const int rank = atomicAdd(&bins[min(cost[c], kBwdBins - 1)], 1);
      items[(int64_t)rank * Hkv + g] = ColItem{col, cw.wj | (cw.words << 16), -1, cost[c]};
    } else {
      const int slot0 = atomicAdd(&counters[0], np);
      const int si = atomicAdd(&counters[1], 1);
      split_cols[3 * si] = col; split_cols[3 * si + 1] = slot0; split_cols[3 * si + 2] = np;
      int part = 0;
      cw.parts(wmax, [&](int lo, int hi, int wt) {
        const int rank = atomicAdd(&bins[min(wt, kBwdBins - 1)], 1);
        items[(int64_t)rank * Hkv + g] = ColItem{col, lo | (hi << 16), slot0 + part, wt};
        ++part;
      });
    }
  }
}

// ---- selection blocks larger than a tile (B = 64 r, r > 1) -------------------------------------
// The attention kernels work on 64-row tiles.  Query tile it of block I = it / r keeps, for every
// earlier block J its block kept, the r key tiles rJ .. rJ+r-1 (whole blocks in the past), and of
// its own block the tiles rI .. it (causality inside the diagonal block, at tile granularity; the
// token-level mask stays inside tile it).  One wavefront per tile row writes the tile-level CSR.
__global__ __launch_bounds__(256) void plan_expand_kernel(const int32_t* __restrict__ b_rowptr, const int32_t* __restrict__ b_idx,
                                                          const int32_t* __restrict__ cu, const int32_t* __restrict__ b_qb_off,
                                                          const int32_t* __restrict__ kclamp, const int32_t* __restrict__ t_qb_off,
                                                          const int32_t* __restrict__ t_qb_seq, int S, int64_t NQB, int64_t NT, int Hs,
                                                          int r, int64_t nnzT_unit, int32_t* __restrict__ t_rowptr,
                                                          int32_t* __restrict__ t_idx) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // hs * NT + global tile
  if (row >= (int64_t)Hs * NT) return;
  const int lane = threadIdx.x & 63;
  const int hs = (int)(row / NT);
  const int64_t qt = row - (int64_t)hs * NT;
  const int s = t_qb_seq[qt];
  const int it = (int)(qt - t_qb_off[s]);
  int64_t base = 0;  // entries of the earlier sequences (one selection head)
  for (int t = 0; t < s; ++t) base += tile_entries_before(t_qb_off[t + 1] - t_qb_off[t], kclamp[t], r);
  const int64_t k = kclamp[s];
  const int64_t e0 = (int64_t)hs * nnzT_unit + base + tile_entries_before(it, k, r);
  const int I = it / r, a = it % r;
  const int64_t brow = (int64_t)hs * NQB + b_qb_off[s] + I;
  const int be0 = b_rowptr[brow], past = b_rowptr[brow + 1] - be0 - 1;  // kept earlier blocks
  if (lane == 0) {
    t_rowptr[row] = (int32_t)e0;
    if (row == (int64_t)Hs * NT - 1) t_rowptr[row + 1] = (int32_t)(e0 + (int64_t)past * r + a + 1);
  }
  for (int x = lane; x < past * r; x += 64) t_idx[e0 + x] = b_idx[be0 + x / r] * r + x % r;
  for (int x = lane; x <= a; x += 64) t_idx[e0 + (int64_t)past * r + x] = I * r + x;
}

// Query-major items for r > 1.  The tile count of a row grows with the query tile until the budget
// saturates, so "later query tiles first" is close to longest-first, keeps the heads of one query
// tile adjacent (KV head fastest, see plan_fwd_kernel) and is a closed form again: the position of
// (s, it, hs) counts the rows of all sequences with a larger tile index, then the rows with the same
// tile index in earlier sequences.
__global__ __launch_bounds__(256) void plan_fwd_tiles_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ qb_off,
                                                             const int32_t* __restrict__ qb_seq, const int32_t* __restrict__ cu, int S,
                                                             int64_t NQB, int Hs, int Hkv, int G, int mode,
                                                             int32_t* __restrict__ work_fwd, WorkItem* __restrict__ items) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row >= (int64_t)Hs * NQB) return;
  const int hs = (int)(row / NQB);
  const int qb = (int)(row - (int64_t)hs * NQB);
  const int s = qb_seq[qb];
  const int it = qb - qb_off[s];
  int64_t pos = 0;
  for (int t = 0; t < S; ++t) {
    const int nt = qb_off[t + 1] - qb_off[t];
    if (nt > it + 1) pos += (int64_t)Hs * (nt - 1 - it);  // rows of t with a larger tile index
    if (t < s && nt > it) pos += Hs;                      // same tile index, earlier sequence
  }
  pos += mode == SB_SELECT_PER_QHEAD ? (hs % G) * Hkv + hs / G : hs;
  work_fwd[pos] = (int32_t)row;
  WorkItem w;
  w.row = (int32_t)row; w.seq0 = cu[s]; w.len = cu[s + 1] - cu[s]; w.i = it;
  w.e0 = rowptr[row]; w.ntiles = rowptr[row + 1] - w.e0; w.hs = hs; w.s = s;
  items[pos] = w;
}

}  // namespace sb

using namespace sb;

extern "C" int sb_plan_worklist(const sb_problem* p, const int32_t* sel_rowptr, const int32_t* sel_idx, void* plan_out,
                                void* stream) {
  Geo gb;
  int rc = make_geo(p, &gb);
  if (rc != SB_OK) return rc;
  if (gb.S == 0 || gb.T == 0 || gb.NQB == 0) return SB_OK;
  if (!sel_rowptr || !sel_idx || !plan_out) { set_error("null sel_rowptr, sel_idx or plan_out"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  const Geo g = tile_geo(gb);  // everything below is at the granularity of the 64-row tiles
  PlanOffsets po = plan_offsets(gb);
  char* base = (char*)plan_out;
  rc = launch_geom(g, p, base + po.tables, st);
  if (rc != SB_OK) return rc;
  Tables t = make_tables(g, p, base + po.tables);
  int32_t* work_fwd = (int32_t*)(base + po.work_fwd);
  int32_t* colcost = (int32_t*)(base + po.colcost);
  ColItem* bwd_items = (ColItem*)(base + po.bwd_items);
  int32_t* counters = (int32_t*)(base + po.counters);
  uint32_t* bitmap = (uint32_t*)(base + po.bitmap);
  const int64_t rows = (int64_t)g.Hs * g.NQB, ncol = (int64_t)g.Hkv * g.NQB;
  KernelTimer kt(K_PLAN, st);
  if ((rc = fill_zero(colcost, sizeof(int32_t) * (size_t)ncol, st)) != SB_OK) return rc;  // the only part of the plan that is accumulated into
  const int32_t* rowptr = sel_rowptr;
  const int32_t* idx = sel_idx;
  if (gb.r == 1) {
    hipLaunchKernelGGL(plan_fwd_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, t.qb_off, t.kclamp, t.qb_seq,
                       t.cu, sel_rowptr, g.S, g.NQB, g.Hs, g.Hkv, g.G, g.mode, work_fwd, (WorkItem*)(base + po.items));
    SB_LAUNCH_CHECK("plan_fwd_kernel");
  } else {
    rc = launch_geom(gb, p, base + po.blk_tables, st);
    if (rc != SB_OK) return rc;
    Tables tb = make_tables(gb, p, base + po.blk_tables);
    int32_t* t_rowptr = (int32_t*)(base + po.t_rowptr);
    int32_t* t_idx = (int32_t*)(base + po.t_idx);
    hipLaunchKernelGGL(plan_expand_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, sel_rowptr, sel_idx, t.cu, tb.qb_off,
                       tb.kclamp, t.qb_off, t.qb_seq, g.S, gb.NQB, g.NQB, g.Hs, gb.r, g.nnz_unit, t_rowptr, t_idx);
    SB_LAUNCH_CHECK("plan_expand_kernel");
    rowptr = t_rowptr;
    idx = t_idx;
    hipLaunchKernelGGL(plan_fwd_tiles_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st, rowptr, t.qb_off, t.qb_seq, t.cu, g.S,
                       g.NQB, g.Hs, g.Hkv, g.G, g.mode, work_fwd, (WorkItem*)(base + po.items));
    SB_LAUNCH_CHECK("plan_fwd_tiles_kernel");
  }
  int64_t words = 0;  // (sequence, 32 query blocks) pairs
  for (int s = 0; s < g.S; ++s) {
    const int64_t L = (int64_t)p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
    words += ((L + g.B - 1) / g.B + 31) / 32;
  }
  hipLaunchKernelGGL(plan_transpose_kernel, dim3((unsigned)words, (unsigned)g.Hs), dim3(256), 0, st, rowptr, idx, t.qb_off, t.bm_off,
                     g.S, g.NQB, g.Hs, g.G, g.mode, bitmap, colcost);
  SB_LAUNCH_CHECK("plan_transpose_kernel");
  // the item lists are padded to their largest possible length; unused entries say "no item"
  const size_t n_items = (size_t)g.Hkv * ((size_t)g.NQB + (size_t)split_extra_max(g));
  if ((rc = fill_words(bwd_items, sizeof(ColItem) * n_items, 0xffffffffu, st)) != SB_OK) return rc;
  if ((rc = fill_zero(counters, sizeof(int32_t) * 4, st)) != SB_OK) return rc;
  hipLaunchKernelGGL(plan_bwd_order_kernel, dim3((unsigned)g.Hkv), dim3(1024), 0, st, colcost, bitmap, t.qb_off, t.qb_seq, t.bm_off,
                     g.NQB, g.Hkv, g.Hs, g.G, g.mode, split_weight(g), bwd_items, counters, (int32_t*)(base + po.split_cols));
  SB_LAUNCH_CHECK("plan_bwd kernels");
  return SB_OK;
}
