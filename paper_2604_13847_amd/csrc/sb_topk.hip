// Top-K block selection (paper section 2.2): per row (sequence, selection head, query block i)
// keep the diagonal block plus the best c-1 past blocks under the total order
// (score descending, block index ascending; -0 == +0; NaN below everything).
// One wavefront per row: order-preserving 32-bit keys in LDS, a 4-pass radix select for the
// threshold key, then an index-ordered compaction, so the result is a pure function of the scores.
#include <mutex>

#include "sb_internal.h"

namespace sb {

__device__ inline uint32_t order_key(float x) {
  if (x != x) return 0u;              // NaN: lowest
  if (x == 0.0f) x = 0.0f;            // -0 and +0 share one key
  uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// LDS operations of one wavefront are carried out in issue order, so a wavefront that works alone
// on its own LDS region needs no barrier between phases: only the compiler has to keep the order.
__device__ inline void wave_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

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
  // closed-form row start: head offset + sequence offset + rows before i in this sequence
  const int m0 = min(i, k);  // rows i' < i with i'+1 <= k contribute i'+1, the rest contribute k
  const int64_t before = (int64_t)m0 * (m0 + 1) / 2 + (int64_t)(i - m0) * k;
  const int64_t start = (int64_t)hs * nnz_unit + row_base[s] + before;
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
  // radix select, 8 bits per pass: the need-th largest key
  uint32_t prefix = 0, mask = 0;
  int remaining = need;
  for (int shift = 24; shift >= 0; shift -= 8) {
#pragma unroll
    for (int a = 0; a < 4; ++a) hist[lane + 64 * a] = 0;
    wave_lds_fence();
    for (int j = lane; j < m; j += 64) {
      const uint32_t kk = keys[j];
      if ((kk & mask) == prefix) atomicAdd(&hist[(kk >> shift) & 255u], 1);
    }
    wave_lds_fence();
    // lane L owns bins 255-4L .. 252-4L (descending); `above` = matching keys in higher bins
    int v[4], sum = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) { v[a] = hist[255 - 4 * lane - a]; sum += v[a]; }
    int incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off, 64);
      if (lane >= off) incl += t;
    }
    int run = incl - sum, bin = -1, above = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      if (run < remaining && remaining <= run + v[a]) { bin = 255 - 4 * lane - a; above = run; }
      run += v[a];
    }
    const unsigned long long found = __builtin_amdgcn_ballot_w64(bin >= 0);  // exactly one lane
    const int src = __builtin_ctzll(found);
    bin = __shfl(bin, src, 64);
    above = __shfl(above, src, 64);
    prefix |= (uint32_t)bin << shift;
    mask |= 255u << shift;
    remaining -= above;
    wave_lds_fence();  // the histogram is cleared again at the top
  }
  // keys > prefix are all kept; of the keys == prefix the `remaining` lowest indices are kept; output in index order
  const uint32_t thr = prefix;
  const unsigned long long lt = (1ull << lane) - 1ull;
  int eq_seen = 0, pos = 0;
  for (int j0 = 0; j0 < m; j0 += 64) {
    const int j = j0 + lane;
    const bool valid = j < m;
    const uint32_t kk = valid ? keys[j] : 0u;
    const bool is_eq = valid && kk == thr;
    const unsigned long long beq = __builtin_amdgcn_ballot_w64(is_eq);
    const int eq_rank = eq_seen + __builtin_popcountll(beq & lt);
    const bool keep = valid && (kk > thr || (is_eq && eq_rank < remaining));
    const unsigned long long bk = __builtin_amdgcn_ballot_w64(keep);
    if (keep) out[pos + __builtin_popcountll(bk & lt)] = j;
    pos += __builtin_popcountll(bk);
    eq_seen += __builtin_popcountll(beq);
  }
  if (lane == 0) out[need] = i;
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
  rc = sb_block_scores(p, q, k, kbar_out, scores_out, ws, stream);  // leaves the geometry tables at the start of ws
  if (rc != SB_OK) return rc;
  return select_launch(g, make_tables(g, p, ws), scores_out, sel_rowptr_out, sel_idx_out, st);
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
