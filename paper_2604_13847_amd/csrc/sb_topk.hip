// Top-K block selection (paper section 2.2): per row (sequence, selection head, query block i)
// keep the diagonal block plus the best c-1 past blocks under the total order
// (score descending, block index ascending; -0 == +0; NaN below everything).
// One wavefront per row: order-preserving 32-bit keys in LDS, a 4-pass radix select for the
// threshold key, then an index-ordered compaction, so the result is a pure function of the scores.
#include <mutex>

#include "sb_internal.h"
#include "sb_score_tile.h"

namespace sb {

// One wavefront per row (several rows per workgroup, no workgroup barrier anywhere): keys and a
// 256-bin histogram in the wavefront's own LDS region.
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ scores, const int32_t* __restrict__ qb_off,
                                                   const int64_t* __restrict__ sc_off, const int32_t* __restrict__ row_base,
                                                   const int32_t* __restrict__ kclamp, const int32_t* __restrict__ qb_seq,
                                                   int64_t NQB, int Hs, int64_t nnz_unit, int region_words,
                                                   int32_t* __restrict__ rowptr, int32_t* __restrict__ idx) {
  extern __shared__ uint32_t smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row_id = (int64_t)blockIdx.x * (blockDim.x >> 6) + wave;  // hs * NQB + query block
  if (row_id >= (int64_t)Hs * NQB) return;
  uint32_t* keys = smem + (size_t)wave * region_words;
  int* hist = (int*)(keys + region_words - 256);
  const int hs = (int)(row_id / NQB);
  const int qb = (int)(row_id - (int64_t)hs * NQB);
  const int s = qb_seq[qb];
  const int i = qb - qb_off[s];
  const int n = qb_off[s + 1] - qb_off[s];
  const int k = kclamp[s];
  const int c = min(k, i + 1);
  const int64_t start = (int64_t)hs * nnz_unit + row_base[s] + sel_rows_before(i, k);
  if (lane == 0) {
    rowptr[row_id] = (int32_t)start;
    if (row_id == (int64_t)Hs * NQB - 1) rowptr[(int64_t)Hs * NQB] = (int32_t)(start + c);
  }
  int32_t* out = idx + start;
  const int need = c - 1, m = i;  // choose `need` of the m past blocks
  if (need == m) {                // everything is kept (also covers need == 0 with i == 0)
    for (int j = lane; j <= i; j += 64) out[j] = j;
    return;
  }
  if (need == 0) {
    if (lane == 0) out[0] = i;
    return;
  }
  const float* row = scores + (int64_t)Hs * sc_off[s] + ((int64_t)hs * n + i) * n;
  for (int j0 = lane; j0 < m; j0 += 64 * 8) {  // eight independent loads in flight per lane: the row comes from HBM
    float x[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) x[u] = j0 + 64 * u < m ? row[j0 + 64 * u] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (j0 + 64 * u < m) keys[j0 + 64 * u] = order_key(x[u]);
  }
  wave_lds_fence();
  select_row(keys, hist, lane, m, need, i, out);
}

// Scores and selection in one kernel: the scores of a row never leave the compute unit.  One
// workgroup of 16 wavefronts owns R consecutive query blocks of the packed batch and one selection
// head.  For each sequence that these blocks touch, every wavefront computes 16 x 16 score tiles
// (the rows' pooled queries in registers, pooled keys straight from memory: they are small and stay
// in L2) and leaves the order keys of the past blocks in LDS, row by row; after a barrier wavefront
// w selects for row w exactly as topk_kernel does.  R (16, or fewer for very long sequences) is what
// fits in LDS: R rows of `stride` keys plus one histogram per wavefront.
constexpr int kFusedWaves = 16;

template <int D>
__global__ __launch_bounds__(64 * kFusedWaves) void score_select_kernel(
    const float* __restrict__ qbar, const float* __restrict__ kbar, const int32_t* __restrict__ qb_off,
    const int32_t* __restrict__ row_base, const int32_t* __restrict__ kclamp, const int32_t* __restrict__ qb_seq, int64_t NQB,
    int Hq, int Hkv, int Hs, int G, int mode, float scale, int64_t nnz_unit, int R, int stride, int32_t* __restrict__ rowptr,
    int32_t* __restrict__ idx) {
  extern __shared__ uint32_t smem[];
  uint32_t* keys = smem;                            // [R][stride]
  int* hist = (int*)(smem + (size_t)R * stride);    // [kFusedWaves][256]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, kq = lane >> 4;
  // Workgroup ids run over the selection heads first and workgroups go to the eight XCDs in turn: head index
  // (x % 8) * (Hs / 8) + x / 8 gives every XCD a contiguous range of heads, i.e. few KV heads, whose pooled keys
  // (n * D floats each) then stay in that XCD's L2.
  const int hx = blockIdx.x % Hs;
  const int64_t gy = blockIdx.x / Hs, ngroups = gridDim.x / Hs;
  const int hs = (Hs & 7) == 0 ? (hx & 7) * (Hs >> 3) + (hx >> 3) : hx;
  const int heads = mode == SB_SELECT_PER_QHEAD ? 1 : G;
  const int h0 = mode == SB_SELECT_PER_QHEAD ? hs : hs * G;
  const int g = h0 / G;
  // rows late in a sequence have the most past blocks: hand out the last groups of blocks first
  const int64_t b0 = (ngroups - 1 - gy) * R, b1 = min(NQB, b0 + R);
  for (int64_t ba = b0; ba < b1;) {
    const int s = qb_seq[ba];
    const int64_t qb0 = qb_off[s];
    const int n = qb_off[s + 1] - (int)qb0;
    const int ia = (int)(ba - qb0), ib = (int)min((int64_t)n, ia + (b1 - ba));  // rows [ia, ib) of sequence s
    const int nrows = ib - ia;
    const int k = kclamp[s];
    // a row needs its scores only if it keeps some but not all of its past blocks: 2 <= k <= i
    if (k >= 2 && ib - 1 >= k) {
      float a[D / 4];
#pragma unroll
      for (int t = 0; t < D / 4; ++t) a[t] = 0.f;
      const int ra = min(ia + l16, ib - 1);  // rows past the segment repeat its last row; their results are dropped
      for (int hh = 0; hh < heads; ++hh) add_quarter<D>(a, qbar + ((qb0 + ra) * Hq + h0 + hh) * D, kq);
      const int ncol = ib - 1;  // block j is in the past of some row of the segment iff j < ib - 1
      for (int ct = wave; ct * 16 < ncol; ct += kFusedWaves) {
        const int j = ct * 16 + l16;
        float b[D / 4];
        load_quarter<D>(b, kbar + ((qb0 + min(j, n - 1)) * Hkv + g) * D, kq);
        const f32x4s acc = score_tile16<D>(a, b);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r = 4 * kq + v;
          if (r < nrows && j < ia + r) keys[(size_t)r * stride + j] = order_key(scale * acc[v]);
        }
      }
    }
    __syncthreads();
    if (wave < nrows) {
      const int i = ia + wave;
      const int c = min(k, i + 1);
      const int64_t row_id = (int64_t)hs * NQB + ba + wave;
      const int64_t start = (int64_t)hs * nnz_unit + row_base[s] + sel_rows_before(i, k);
      if (lane == 0) {
        rowptr[row_id] = (int32_t)start;
        if (row_id == (int64_t)Hs * NQB - 1) rowptr[(int64_t)Hs * NQB] = (int32_t)(start + c);
      }
      int32_t* out = idx + start;
      const int need = c - 1, m = i;
      if (need == m) {
        for (int j = lane; j <= i; j += 64) out[j] = j;
      } else if (need == 0) {
        if (lane == 0) out[0] = i;
      } else {
        select_row(keys + (size_t)wave * stride, hist + 256 * wave, lane, m, need, i, out);
      }
    }
    __syncthreads();  // the keys are overwritten by the next segment
    ba += nrows;
  }
}

}  // namespace sb

using namespace sb;

// launches the selection on tables that are already in device memory
static int select_launch(const Geo& g, const Tables& t, const float* scores, int32_t* sel_rowptr_out, int32_t* sel_idx_out,
                         hipStream_t st) {
  // every wavefront owns a region of n_max keys (rounded up to 64) plus 256 histogram bins; as many rows per workgroup
  // (at most four) as fit in 64 KiB
  const int region_words = (int)((g.n_max + 63) / 64 * 64 + 256);
  int W = (int)(65536 / (sizeof(uint32_t) * (size_t)region_words));
  W = W < 1 ? 1 : (W > 4 ? 4 : W);
  const size_t smem = sizeof(uint32_t) * (size_t)region_words * W;
  if (smem > 48 * 1024) {  // raise the kernel's dynamic LDS limit; once per device, whichever thread comes first
    static std::mutex mu;
    static bool attr_set[kMaxDevices] = {};
    int dev = 0;
    SB_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d out of range", dev); return SB_ERR_UNSUPPORTED; }
    std::lock_guard<std::mutex> lock(mu);
    if (!attr_set[dev]) {
      SB_CHECK_HIP(hipFuncSetAttribute((const void*)topk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(sizeof(uint32_t) * (SB_MAX_BLOCKS_PER_SEQ + 256))));
      attr_set[dev] = true;
    }
  }
  const int64_t rows = (int64_t)g.Hs * g.NQB;
  dim3 grid((unsigned)((rows + W - 1) / W));
  KernelTimer kt(K_TOPK, st);
  hipLaunchKernelGGL(topk_kernel, grid, dim3(64 * W), smem, st, scores, t.qb_off, t.sc_off, t.row_base, t.kclamp, t.qb_seq,
                     g.NQB, g.Hs, g.nnz_unit, region_words, sel_rowptr_out, sel_idx_out);
  SB_LAUNCH_CHECK("topk_kernel");
  return SB_OK;
}

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
  return select_launch(g, make_tables(g, p, ws), scores, sel_rowptr_out, sel_idx_out, st);
}

// launches the kernel that scores and selects; qbar/kbar are the pooled arrays
static int score_select_launch(const Geo& g, const Tables& t, const float* qbar, const float* kbar, int32_t* sel_rowptr_out,
                               int32_t* sel_idx_out, hipStream_t st) {
  static std::mutex mu;
  static int lds_of_device[kMaxDevices] = {};  // LDS a workgroup may use, once the kernels' limit has been raised to it
  int dev = 0;
  SB_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d out of range", dev); return SB_ERR_UNSUPPORTED; }
  int cap = 0;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!lds_of_device[dev]) {
      int per_block = 0;
      SB_CHECK_HIP(hipDeviceGetAttribute(&per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
      SB_CHECK_HIP(hipFuncSetAttribute((const void*)score_select_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, per_block));
      SB_CHECK_HIP(hipFuncSetAttribute((const void*)score_select_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, per_block));
      lds_of_device[dev] = per_block;
    }
    cap = lds_of_device[dev];
  }
  // a row of keys is padded to a stride of 4 mod 16 words, so that the four query rows a store instruction touches
  // fall into different banks
  const int stride = (g.n_max + 63) / 64 * 64 + 4;
  const size_t hist_words = 256 * (size_t)kFusedWaves;
  int R = kFusedWaves;
  while (R > 1 && sizeof(uint32_t) * ((size_t)R * stride + hist_words) > (size_t)cap) R >>= 1;
  const size_t smem = sizeof(uint32_t) * ((size_t)R * stride + hist_words);
  if (smem > (size_t)cap) {
    set_error("a sequence of %d blocks does not fit the fused selection (%zu bytes of LDS, %d available): pass scores_out", g.n_max,
              smem, cap);
    return SB_ERR_UNSUPPORTED;
  }
  const int64_t groups = (g.NQB + R - 1) / R;
  if (groups * g.Hs > 0x7fffffffll) { set_error("too many rows for one launch of the fused selection: pass scores_out"); return SB_ERR_UNSUPPORTED; }
  dim3 grid((unsigned)(groups * g.Hs));
  KernelTimer kt(K_SCORE_SELECT, st);
  if (g.D == 128)
    hipLaunchKernelGGL(score_select_kernel<128>, grid, dim3(64 * kFusedWaves), smem, st, qbar, kbar, t.qb_off, t.row_base, t.kclamp,
                       t.qb_seq, g.NQB, g.Hq, g.Hkv, g.Hs, g.G, g.mode, g.score_scale, g.nnz_unit, R, stride, sel_rowptr_out,
                       sel_idx_out);
  else
    hipLaunchKernelGGL(score_select_kernel<64>, grid, dim3(64 * kFusedWaves), smem, st, qbar, kbar, t.qb_off, t.row_base, t.kclamp,
                       t.qb_seq, g.NQB, g.Hq, g.Hkv, g.Hs, g.G, g.mode, g.score_scale, g.nnz_unit, R, stride, sel_rowptr_out,
                       sel_idx_out);
  SB_LAUNCH_CHECK("score_select_kernel");
  return SB_OK;
}

extern "C" int sb_score_select(const sb_problem* p, const void* q, const void* k, float* kbar_out, float* scores_out,
                               int32_t* sel_rowptr_out, int32_t* sel_idx_out, void* ws, void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (!sel_rowptr_out) { set_error("null sel_rowptr_out"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) {
    return fill_zero(sel_rowptr_out, sizeof(int32_t), st);
  }
  if (!sel_idx_out) { set_error("null sel_idx_out"); return SB_ERR_INVALID_ARG; }
  if (scores_out) {  // the caller wants the score matrix: write it, then select from it
    rc = sb_block_scores(p, q, k, kbar_out, scores_out, ws, stream);  // leaves the geometry tables at the start of ws
    if (rc != SB_OK) return rc;
    return select_launch(g, make_tables(g, p, ws), scores_out, sel_rowptr_out, sel_idx_out, st);
  }
  if (!q || !k || !ws) { set_error("null q, k or ws"); return SB_ERR_INVALID_ARG; }
  rc = launch_geom(g, p, ws, st);
  if (rc != SB_OK) return rc;
  Tables t = make_tables(g, p, ws);
  float *qbar = nullptr, *kbar = nullptr;
  if ((rc = launch_pool(g, p, t, q, k, kbar_out, ws, st, &qbar, &kbar)) != SB_OK) return rc;
  return score_select_launch(g, t, qbar, kbar, sel_rowptr_out, sel_idx_out, st);
}

// ---------------------------------------------------------------------------------------------
// sb_select_topk for callers that cannot allocate: the geometry tables that `ws` holds in sb_select_topk live in a
// file-scope device array instead.  In host code the array's name is only a stand-in; its device address is looked up
// once per device (each GPU has its own copy at its own address) and that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[SB_STATIC_SELECT_WS_BYTES];

static int static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptr_of_device[kMaxDevices] = {};
  int dev = 0;
  SB_CHECK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d out of range", dev); return SB_ERR_UNSUPPORTED; }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* ptr = nullptr;
    SB_CHECK_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) { set_error("hipGetSymbolAddress returned a null pointer"); return SB_ERR_HIP; }
    ptr_of_device[dev] = ptr;
  }
  *out = ptr_of_device[dev];
  return SB_OK;
}

extern "C" int sb_select_topk_static(const sb_problem* p, const float* scores, int32_t* sel_rowptr_out, int32_t* sel_idx_out,
                                     void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (!sel_rowptr_out) { set_error("null sel_rowptr_out"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) return fill_zero(sel_rowptr_out, sizeof(int32_t), st);
  if (!scores || !sel_idx_out) { set_error("null scores or sel_idx_out"); return SB_ERR_INVALID_ARG; }
  const size_t need = align_up(table_offsets(g).bytes);
  if (need > (size_t)SB_STATIC_SELECT_WS_BYTES) {
    set_error("problem needs %zu bytes of geometry tables, the built-in scratch holds %d (use sb_select_topk)", need,
              (int)SB_STATIC_SELECT_WS_BYTES);
    return SB_ERR_WORKSPACE_TOO_SMALL;
  }
  void* ws = nullptr;
  if ((rc = static_scratch_ptr(&ws)) != SB_OK) return rc;
  // every table entry the selection reads is rewritten by the geometry kernel of this call: nothing has to start at zero
  rc = launch_geom(g, p, ws, st);
  if (rc != SB_OK) return rc;
  return select_launch(g, make_tables(g, p, ws), scores, sel_rowptr_out, sel_idx_out, st);
}
