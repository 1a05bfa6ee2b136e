// Host-side logic of libsparsebal: validation, closed-form sizes, device geometry tables.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <atomic>
#include <mutex>

#include "sb_internal.h"

namespace sb {

static thread_local char g_err[512] = "";
std::atomic<int> g_instrument{0};

// Instrumentation state.  The flag and the event records are process-wide and guarded by one mutex, so calls from
// several threads do not corrupt them (their records simply interleave).  Events are recycled through a free list:
// after the first few steps a timed launch costs two hipEventRecord calls and no event creation.
struct EventPair { hipEvent_t a, b; };
static std::mutex g_ev_mu;
static std::vector<EventPair> g_events[K_NUM];
static std::vector<hipEvent_t> g_free_events;

static hipEvent_t take_event() {
  {
    std::lock_guard<std::mutex> lock(g_ev_mu);
    if (!g_free_events.empty()) {
      hipEvent_t e = g_free_events.back();
      g_free_events.pop_back();
      return e;
    }
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

KernelTimer::KernelTimer(int slot_, hipStream_t st_) : slot(slot_), st(st_) {
  if (!(g_instrument & 2)) return;
  hipEvent_t a = take_event();
  if (!a) return;
  (void)hipEventRecord(a, st);
  start = (void*)a;
}
KernelTimer::~KernelTimer() {
  if (!start) return;
  hipEvent_t b = take_event();
  std::lock_guard<std::mutex> lock(g_ev_mu);
  if (!b) { g_free_events.push_back((hipEvent_t)start); return; }
  (void)hipEventRecord(b, st);
  g_events[slot].push_back({(hipEvent_t)start, b});
}

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int make_geo(const sb_problem* p, Geo* g) {
  if (!p || !g) { set_error("null problem"); return SB_ERR_INVALID_ARG; }
  if (p->total_tokens < 0 || p->num_seqs < 0) { set_error("negative T or S"); return SB_ERR_INVALID_ARG; }
  if (p->num_q_heads < 1 || p->num_kv_heads < 1 || p->num_q_heads % p->num_kv_heads != 0) {
    set_error("num_q_heads (%d) must be a positive multiple of num_kv_heads (%d)", p->num_q_heads, p->num_kv_heads);
    return SB_ERR_INVALID_ARG;
  }
  if (p->dtype != SB_BF16 && p->dtype != SB_F32) { set_error("dtype must be SB_BF16 or SB_F32"); return SB_ERR_INVALID_ARG; }
  if (p->select_mode != SB_SELECT_PER_QHEAD && p->select_mode != SB_SELECT_PER_KVGROUP) {
    set_error("bad select_mode %d", p->select_mode);
    return SB_ERR_INVALID_ARG;
  }
  if (p->block_size != 64 && p->block_size != 128 && p->block_size != 256) {
    set_error("block_size %d unsupported (64, 128 or 256)", p->block_size);
    return SB_ERR_UNSUPPORTED;
  }
  if (p->head_dim != 64 && p->head_dim != 128) { set_error("head_dim %d unsupported (64 or 128)", p->head_dim); return SB_ERR_UNSUPPORTED; }
  g->T = p->total_tokens; g->S = p->num_seqs; g->Hq = p->num_q_heads; g->Hkv = p->num_kv_heads;
  g->G = g->Hq / g->Hkv; g->D = p->head_dim; g->B = p->block_size; g->r = g->B / 64; g->mode = p->select_mode; g->dtype = p->dtype;
  g->Hs = g->mode == SB_SELECT_PER_QHEAD ? g->Hq : g->Hkv;
  if (g->mode == SB_SELECT_PER_KVGROUP && g->G > 8) {
    set_error("SB_SELECT_PER_KVGROUP supports at most 8 query heads per KV head (got %d)", g->G);
    return SB_ERR_UNSUPPORTED;
  }
  g->softmax_scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)g->D);
  g->score_scale = p->score_scale > 0.f ? p->score_scale : g->softmax_scale;
  g->NQB = 0; g->n_max = 0; g->scores_unit = 0; g->nnz_unit = 0; g->bm_words_unit = 0; g->pairs_unit = 0;
  g->NT = 0; g->nt_max = 0; g->nnzT_unit = 0; g->bmT_words_unit = 0;
  if (g->S == 0 || g->T == 0) {
    if (g->S > 0 && p->cu_seqlens_host && p->cu_seqlens_host[g->S] != g->T) { set_error("cu_seqlens[S] != T"); return SB_ERR_INVALID_ARG; }
    if (g->S == 0 && g->T != 0) { set_error("T != 0 with S == 0"); return SB_ERR_INVALID_ARG; }
  }
  if (g->S > 0) {
    if (!p->cu_seqlens_host || !p->topk_host) { set_error("cu_seqlens_host and topk_host are required"); return SB_ERR_INVALID_ARG; }
    const int32_t* cu = p->cu_seqlens_host;
    if (cu[0] != 0 || cu[g->S] != g->T) { set_error("cu_seqlens must start at 0 and end at T"); return SB_ERR_INVALID_ARG; }
    for (int s = 0; s < g->S; ++s) {
      int64_t L = (int64_t)cu[s + 1] - cu[s];
      if (L < 0) { set_error("cu_seqlens decreases at %d", s); return SB_ERR_INVALID_ARG; }
      if (p->topk_host[s] < 1) { set_error("topk[%d] = %d < 1", s, p->topk_host[s]); return SB_ERR_INVALID_ARG; }
      int64_t n = (L + g->B - 1) / g->B;
      if (n > SB_MAX_BLOCKS_PER_SEQ) { set_error("sequence %d has %lld blocks > %d", s, (long long)n, SB_MAX_BLOCKS_PER_SEQ); return SB_ERR_UNSUPPORTED; }
      int64_t k = p->topk_host[s] < n ? p->topk_host[s] : n;
      g->NQB += n;
      if (n > g->n_max) g->n_max = (int)n;
      g->scores_unit += n * n;
      g->nnz_unit += k * n - k * (k - 1) / 2;
      g->bm_words_unit += n * ((n + 31) / 32);
      const int64_t nt = (L + 63) / 64;
      g->NT += nt;
      if (nt > g->nt_max) g->nt_max = (int)nt;
      g->nnzT_unit += tile_entries_before(nt, k, g->r);
      g->bmT_words_unit += nt * ((nt + 31) / 32);
      // unmasked pairs: every past selected block is B x B except that the last query block may have
      // fewer rows; the diagonal block contributes rows(rows+1)/2
      for (int64_t i = 0; i < n; ++i) {
        int64_t rows = (i + 1) * g->B <= L ? g->B : L - i * g->B;
        int64_t c = k < i + 1 ? k : i + 1;
        g->pairs_unit += (c - 1) * rows * g->B + rows * (rows + 1) / 2;
      }
    }
  }
  if ((int64_t)g->Hs * g->nnzT_unit > 0x7fffffffLL || (int64_t)g->Hs * g->NT + 1 > 0x7fffffffLL) {
    set_error("selection too large for int32 row pointers");
    return SB_ERR_UNSUPPORTED;
  }
  return SB_OK;
}

TableOffsets table_offsets(const Geo& g) {
  TableOffsets t{};
  size_t o = 0;
  t.qb_off = o;   o = align_up(o + sizeof(int32_t) * (size_t)(g.S + 1));
  t.sc_off = o;   o = align_up(o + sizeof(int64_t) * (size_t)(g.S + 1));
  t.row_base = o; o = align_up(o + sizeof(int32_t) * (size_t)(g.S + 1));
  t.bm_off = o;   o = align_up(o + sizeof(int64_t) * (size_t)(g.S + 1));
  t.kclamp = o;   o = align_up(o + sizeof(int32_t) * (size_t)(g.S + 1));
  t.qb_seq = o;   o = align_up(o + sizeof(int32_t) * (size_t)(g.NQB + 1));
  t.bytes = o;
  return t;
}

Tables make_tables(const Geo& g, const sb_problem* p, void* base) {
  TableOffsets t = table_offsets(g);
  char* b = (char*)base;
  Tables r;
  r.cu = p->cu_seqlens_dev;
  r.qb_off = (const int32_t*)(b + t.qb_off);
  r.sc_off = (const int64_t*)(b + t.sc_off);
  r.row_base = (const int32_t*)(b + t.row_base);
  r.bm_off = (const int64_t*)(b + t.bm_off);
  r.kclamp = (const int32_t*)(b + t.kclamp);
  r.qb_seq = (const int32_t*)(b + t.qb_seq);
  return r;
}

PlanOffsets plan_offsets(const Geo& gb) {
  const Geo g = tile_geo(gb);  // the plan is laid out for the 64-row tiles the attention kernels work on
  PlanOffsets p{};
  size_t o = 0;
  p.tables = o;   o = align_up(o + table_offsets(g).bytes);
  p.work_fwd = o; o = align_up(o + sizeof(int32_t) * (size_t)(g.Hs * g.NQB + 1));
  p.colcost = o;  o = align_up(o + sizeof(int32_t) * (size_t)(g.Hkv * g.NQB + 1));
  p.bitmap = o;   o = align_up(o + sizeof(uint32_t) * (size_t)(g.Hs * g.bm_words_unit + 1));
  p.items = o;    o = align_up(o + sizeof(WorkItem) * (size_t)(g.Hs * g.NQB + 1));
  p.blk_tables = p.t_rowptr = p.t_idx = o;
  if (gb.r > 1) {
    p.blk_tables = o; o = align_up(o + table_offsets(gb).bytes);
    p.t_rowptr = o;   o = align_up(o + sizeof(int32_t) * (size_t)(g.Hs * g.NQB + 1));
    p.t_idx = o;      o = align_up(o + sizeof(int32_t) * (size_t)(g.Hs * g.nnz_unit + 1));
  }
  const size_t E = (size_t)split_extra_max(g);
  p.bwd_items = o;  o = align_up(o + sizeof(ColItem) * ((size_t)g.Hkv * ((size_t)g.NQB + E) + 1));
  p.counters = o;   o = align_up(o + sizeof(int32_t) * 4);
  p.split_cols = o; o = align_up(o + sizeof(int32_t) * (3 * E + 1));
  p.bytes = o;
  return p;
}

static WsOffsets ws_offsets(const Geo& g, bool bwd) {
  WsOffsets w{};
  size_t o = 0;
  size_t qbytes = g.dtype == SB_F32 ? sizeof(uint16_t) * (size_t)g.T * g.Hq * g.D : 0;
  size_t kbytes = g.dtype == SB_F32 ? sizeof(uint16_t) * (size_t)g.T * g.Hkv * g.D : 0;
  w.cu_busy = o; o = align_up(o + sizeof(uint64_t) * SB_CU_SLOTS);
  w.qc = o;  o = align_up(o + qbytes);
  w.kc = o;  o = align_up(o + kbytes);
  w.vc = o;  o = align_up(o + kbytes);
  w.oc = o;  o = align_up(o + 0);
  w.doc = o; o = align_up(o + (bwd ? qbytes : 0));
  w.drow = o; o = align_up(o + (bwd ? sizeof(float) * (size_t)g.T * g.Hq : 0));
  w.lse2 = o; o = align_up(o + (bwd ? sizeof(float) * ((size_t)g.T * g.Hq + 1) : 0));  // + one +inf sentinel
  w.ticket = o; o = align_up(o + sizeof(int32_t) * 64);
  w.partials = o; o = align_up(o + (bwd ? sizeof(float) * 2 * (size_t)split_extra_max(tile_geo(g)) * 2 * 64 * g.D : 0));  // tile_geo is idempotent
  w.bytes = o;
  return w;
}
WsOffsets fwd_ws_offsets(const Geo& g) { return ws_offsets(g, false); }

WsOffsets bwd_ws_offsets(const Geo& g) { return ws_offsets(g, true); }

size_t scores_ws_bytes(const Geo& g) {
  // tables + pooled Q [NQB][Hq][D] float + pooled K [NQB][Hkv][D] float
  return align_up(table_offsets(g).bytes) + align_up(sizeof(float) * (size_t)g.NQB * g.Hq * g.D) +
         align_up(sizeof(float) * (size_t)g.NQB * g.Hkv * g.D);
}

// One workgroup: prefix sums over sequences, then the query-block -> sequence map.
__global__ __launch_bounds__(1024) void geom_kernel(const int32_t* __restrict__ cu, const int32_t* __restrict__ topk, int S, int B,
                                                    int64_t NQB, int32_t* qb_off, int64_t* sc_off, int32_t* row_base,
                                                    int64_t* bm_off, int32_t* kclamp, int32_t* qb_seq) {
  __shared__ long long wsum[4][16];  // per-wavefront totals of the four scanned columns
  __shared__ long long carry[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid < 4) carry[tid] = 0;
  if (tid == 0) { qb_off[0] = 0; sc_off[0] = 0; row_base[0] = 0; bm_off[0] = 0; }
  __syncthreads();
  for (int base = 0; base < S; base += 1024) {
    int s = base + tid;
    long long v[4] = {0, 0, 0, 0};
    if (s < S) {
      long long L = cu[s + 1] - cu[s];
      long long n = (L + B - 1) / B;
      long long k = topk[s] < n ? topk[s] : n;
      if (k < 1) k = n > 0 ? 1 : 0;
      kclamp[s] = (int32_t)k;
      v[0] = n; v[1] = n * n; v[2] = k * n - k * (k - 1) / 2; v[3] = n * ((n + 31) / 32);
    }
    // inclusive scan of the four columns: inside each wavefront by shuffles, then over the 16 wavefront totals
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const long long t = __shfl_up(v[a], off, 64);
        if (lane >= off) v[a] += t;
      }
      if (lane == 63) wsum[a][wave] = v[a];
    }
    __syncthreads();
    long long before[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      before[a] = 0;
      for (int w = 0; w < wave; ++w) before[a] += wsum[a][w];
    }
    if (s < S) {
      qb_off[s + 1] = (int32_t)(carry[0] + before[0] + v[0]);
      sc_off[s + 1] = carry[1] + before[1] + v[1];
      row_base[s + 1] = (int32_t)(carry[2] + before[2] + v[2]);
      bm_off[s + 1] = carry[3] + before[3] + v[3];
    }
    __syncthreads();
    if (tid < 4) {
      long long total = 0;
      for (int w = 0; w < 16; ++w) total += wsum[tid][w];
      carry[tid] += total;
    }
    __syncthreads();
  }
  __threadfence_block();
  __syncthreads();
  // query block -> sequence by binary search over qb_off (written above by this workgroup)
  for (long long qb = tid; qb < NQB; qb += 1024) {
    int lo = 0, hi = S - 1;  // largest s with qb_off[s] <= qb and n_s > 0  (first s with qb_off[s+1] > qb)
    while (lo < hi) {
      int mid = (lo + hi) >> 1;
      if (qb_off[mid + 1] > qb) hi = mid; else lo = mid + 1;
    }
    qb_seq[qb] = lo;
  }
}

int launch_geom(const Geo& g, const sb_problem* p, void* base, hipStream_t st) {
  if (g.S == 0) return SB_OK;
  if (!p->cu_seqlens_dev || !p->topk_dev) { set_error("cu_seqlens_dev and topk_dev are required"); return SB_ERR_INVALID_ARG; }
  TableOffsets t = table_offsets(g);
  char* b = (char*)base;
  hipLaunchKernelGGL(geom_kernel, dim3(1), dim3(1024), 0, st, p->cu_seqlens_dev, p->topk_dev, g.S, g.B, g.NQB,
                     (int32_t*)(b + t.qb_off), (int64_t*)(b + t.sc_off), (int32_t*)(b + t.row_base),
                     (int64_t*)(b + t.bm_off), (int32_t*)(b + t.kclamp), (int32_t*)(b + t.qb_seq));
  SB_LAUNCH_CHECK("geom_kernel");
  return SB_OK;
}

__global__ __launch_bounds__(256) void fill_words_kernel(uint32_t* __restrict__ dst, size_t n, uint32_t value) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = value;
}

int fill_words(void* dst, size_t bytes, uint32_t value, hipStream_t st) {
  const size_t n = bytes / 4;
  if (n == 0) return SB_OK;
  const size_t blocks = (n + 255) / 256;
  hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, st, (uint32_t*)dst, n, value);
  SB_LAUNCH_CHECK("fill_words_kernel");
  return SB_OK;
}
int fill_zero(void* dst, size_t bytes, hipStream_t st) { return fill_words(dst, bytes, 0u, st); }

}  // namespace sb

using namespace sb;

extern "C" {

const char* sb_last_error(void) { return g_err; }
const char* sb_version(void) { return "libsparsebal 0.1 (gfx950)"; }

int sb_get_layout(const sb_problem* p, sb_layout* out) {
  if (!out) { set_error("null layout"); return SB_ERR_INVALID_ARG; }
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  out->num_qblocks = g.NQB;
  out->sel_heads = g.Hs;
  out->scores_elems = (int64_t)g.Hs * g.scores_unit;
  out->pooled_elems = g.NQB * g.Hkv * g.D;
  out->sel_rows = (int64_t)g.Hs * g.NQB;
  out->sel_nnz = (int64_t)g.Hs * g.nnz_unit;
  out->plan_bytes = (int64_t)plan_offsets(g).bytes;
  out->scores_ws_bytes = (int64_t)scores_ws_bytes(g);
  out->select_ws_bytes = (int64_t)align_up(table_offsets(g).bytes);
  out->fwd_ws_bytes = (int64_t)fwd_ws_offsets(g).bytes;
  out->bwd_ws_bytes = (int64_t)bwd_ws_offsets(g).bytes;
  out->attended_pairs_per_head_sum = g.pairs_unit * g.Hq;
  out->coverage_ws_bytes = (int64_t)coverage_ws_bytes(g);
  return SB_OK;
}

int sb_plan_sections(const sb_problem* p, int64_t* out) {
  if (!out) { set_error("null out"); return SB_ERR_INVALID_ARG; }
  Geo gb;
  int rc = make_geo(p, &gb);
  if (rc != SB_OK) return rc;
  const Geo g = tile_geo(gb);
  const PlanOffsets po = plan_offsets(gb);
  const TableOffsets to = table_offsets(g);
  out[SB_PLAN_QB_OFF] = (int64_t)(po.tables + to.qb_off);
  out[SB_PLAN_BM_OFF] = (int64_t)(po.tables + to.bm_off);
  out[SB_PLAN_QB_SEQ] = (int64_t)(po.tables + to.qb_seq);
  out[SB_PLAN_WORK_FWD] = (int64_t)po.work_fwd;
  out[SB_PLAN_COLCOST] = (int64_t)po.colcost;
  out[SB_PLAN_BITMAP] = (int64_t)po.bitmap;
  out[SB_PLAN_BWD_ITEMS] = (int64_t)po.bwd_items;
  out[SB_PLAN_COUNTERS] = (int64_t)po.counters;
  out[SB_PLAN_SPLIT_COLS] = (int64_t)po.split_cols;
  out[SB_PLAN_BWD_ITEMS_COUNT] = (int64_t)g.Hkv * (g.NQB + split_extra_max(g));
  out[SB_PLAN_SPLIT_WEIGHT] = split_weight(g);
  out[SB_PLAN_SPLIT_MAX] = split_extra_max(g);
  return SB_OK;
}

int sb_keep_ratio_to_topk(const int32_t* cu, int32_t S, int32_t B, const float* rho, int32_t* out) {
  if (S < 0 || B < 1 || (S > 0 && (!cu || !rho || !out))) { set_error("bad arguments"); return SB_ERR_INVALID_ARG; }
  for (int s = 0; s < S; ++s) {
    long long L = (long long)cu[s + 1] - cu[s];
    if (L < 0) { set_error("cu_seqlens decreases at %d", s); return SB_ERR_INVALID_ARG; }
    long long n = (L + B - 1) / B;
    long long k = (long long)ceil((double)rho[s] * (double)n - 1e-6);
    if (k > n) k = n;
    if (k < 1) k = 1;
    out[s] = (int32_t)k;
  }
  return SB_OK;
}

int sb_sel_rowptr_host(const sb_problem* p, int32_t* rowptr) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (!rowptr) { set_error("null rowptr"); return SB_ERR_INVALID_ARG; }
  int64_t pos = 0;
  for (int hs = 0; hs < g.Hs; ++hs) {
    int64_t qb = 0;
    for (int s = 0; s < g.S; ++s) {
      int64_t L = (int64_t)p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
      int64_t n = (L + g.B - 1) / g.B, k = p->topk_host[s] < n ? p->topk_host[s] : n;
      for (int64_t i = 0; i < n; ++i) {
        rowptr[(int64_t)hs * g.NQB + qb + i] = (int32_t)pos;
        pos += k < i + 1 ? k : i + 1;
      }
      qb += n;
    }
  }
  rowptr[(int64_t)g.Hs * g.NQB] = (int32_t)pos;
  return SB_OK;
}

int sb_set_instrumentation(int flag) { g_instrument = flag & 3; return SB_OK; }

int sb_read_kernel_times(double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) { set_error("null argument"); return SB_ERR_INVALID_ARG; }
  std::vector<EventPair> taken[K_NUM];
  {
    std::lock_guard<std::mutex> lock(g_ev_mu);
    for (int k = 0; k < K_NUM; ++k) taken[k].swap(g_events[k]);
  }
  int rc = SB_OK;
  for (int k = 0; k < K_NUM; ++k) {
    total_ms[k] = 0.0; launches[k] = 0;
    for (auto& e : taken[k]) {
      float ms = 0.f;
      if (rc == SB_OK && (hipEventSynchronize(e.b) != hipSuccess || hipEventElapsedTime(&ms, e.a, e.b) != hipSuccess)) {
        set_error("reading a kernel's event pair failed");
        rc = SB_ERR_HIP;
      }
      total_ms[k] += ms; launches[k] += 1;
    }
  }
  std::lock_guard<std::mutex> lock(g_ev_mu);  // the events go back to the free list whether or not they could be read
  for (int k = 0; k < K_NUM; ++k)
    for (auto& e : taken[k]) { g_free_events.push_back(e.a); g_free_events.push_back(e.b); }
  return rc;
}

int sb_read_cu_busy(const void* ws, uint64_t* out, void* stream) {
  if (!ws || !out) { set_error("null argument"); return SB_ERR_INVALID_ARG; }
  SB_CHECK_HIP(hipMemcpyAsync(out, ws, sizeof(uint64_t) * SB_CU_SLOTS, hipMemcpyDeviceToHost, (hipStream_t)stream));
  SB_CHECK_HIP(hipStreamSynchronize((hipStream_t)stream));
  return SB_OK;
}

}  // extern "C"
