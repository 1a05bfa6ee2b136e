// Block-sparse attention forward (paper Eq. 2) on bf16 MFMA with fp32 online softmax.
//
// One workgroup per work item (sequence s, selection head hs, query block i), taken from the
// longest-first work list.  The item's 64 query rows (times up to 4 query heads of the KV group in
// per-KV-group mode) are split into strips of 32 rows, one wavefront per strip.  The K and V tiles
// of the selected key blocks stream through three LDS slots as a sequence of half-tiles
// K0 V0 K1 V1 ...: while half-tile n is consumed, n+1 is landing and n+2 is issued, all by
// asynchronous global->LDS loads that occupy no registers.  Each wavefront computes S^T = K Q^T,
// keeps the running max / sum per query in registers (a query is a C-matrix column, i.e. one lane
// pair), and accumulates O^T += V^T P^T, reading V^T straight out of the row-major V tile with the
// transposing LDS read.
#include "sb_attn_common.h"

namespace sb {

template <int D, bool OUT_F32, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2))) void attn_fwd_kernel(AttnParams P) {
  __shared__ __attribute__((aligned(1024))) bf16 slots[3][64 * D];
  constexpr int LPT = loads_per_tile<D>();
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int64_t row = P.work[blockIdx.x];
  const int hs = (int)(row / P.NQB);
  const int qb = (int)(row - (int64_t)hs * P.NQB);
  const int s = P.qb_seq[qb];
  const int i = qb - P.qb_off[s];
  const int64_t seq0 = P.cu[s];
  const int L = P.cu[s + 1] - P.cu[s];
  // per-KV-group mode: a workgroup serves up to 4 query heads of the group, blockIdx.y picks which
  const int hh = blockIdx.y * (nthr >> 7) + (wave >> 1), strip = wave & 1;
  const bool head_ok = P.mode == SB_SELECT_PER_QHEAD || hh < P.G;
  const int h = P.mode == SB_SELECT_PER_QHEAD ? hs : hs * P.G + (head_ok ? hh : 0);
  const int g = h / P.G;
  const int qloc = strip * 32 + l32;  // this lane's query row inside the block
  const bool qvalid = head_ok && i * 64 + qloc < L;
  const int64_t tq = seq0 + i * 64 + qloc;

  const int e0 = P.rowptr[row], ntiles = P.rowptr[row + 1] - e0;
  // The row's block indices are staged in LDS, kJ at a time: reading them from LDS keeps them off
  // the vector-memory counter that the in-flight tile loads are tracked with.
  constexpr int kJ = 256;
  __shared__ int jbuf[kJ];
  auto stage_indices = [&](int t0) {  // entries t0 .. t0+kJ-1 of the row; all waves call it together
    __syncthreads();
    for (int a = tid; a < kJ; a += nthr) jbuf[a] = t0 + a < ntiles ? P.idx[e0 + t0 + a] : 0;
    __syncthreads();
  };
  // half-tile n: K (n even) or V (n odd) of tile n/2, staged in slot n % 3
  TileLoader<D> loader;
  loader.init(P.Hkv, wave, lane);
  auto issue = [&](int n) {
    const int j = __builtin_amdgcn_readfirstlane(jbuf[(n >> 1) % kJ]);
    loader.issue(slots[n % 3], (n & 1) ? P.v : P.k, seq0 + (int64_t)j * 64, min(64, L - j * 64), P.Hkv, g);
  };
  bf16x8 qf[D / 16];
  {
    const bf16* qp = P.q + (tq * P.Hq + h) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qf[ks] = qvalid ? *(const bf16x8*)(qp + 16 * ks) : zero_bf16x8();
  }
  stage_indices(0);
  // the query fragments must have landed before the tile loads start: from here on the only
  // vector-memory operations in flight are tile loads, which the loop waits for by count
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(qf[ks]));
  issue(0);
  issue(1);

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) oacc[dt] = zero16();
  float m = -__builtin_inff(), l = 0.f;

  for (int t = 0; t < ntiles; ++t) {
    const bool more = t + 1 < ntiles;
    if (more && (t + 1) % kJ == 0) stage_indices(t + 1);  // drains the loads in flight once per kJ tiles
    // ---- K half-tile: loads of V_t may stay in flight
    wait_vmcnt<LPT>();
    __builtin_amdgcn_s_barrier();
    if (more) issue(2 * t + 2);
    const bf16* Ks = slots[(2 * t) % 3];
    f32x16 sacc[2];
    {
      // all 2 x D/16 operand reads are issued before the first MFMA so that LDS latency is paid once
      bf16x8 ka[2][D / 16];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) ka[mt][ks] = lds_row8<D>(Ks, 32 * mt + l32, 2 * ks + hf);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        sacc[mt] = zero16();
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) sacc[mt] = mfma32(ka[mt][ks], qf[ks], sacc[mt]);
      }
    }
    // online softmax on the raw scores: p = exp2(scale*log2e * (s - m)), m = running max of raw scores
    if (t == ntiles - 1) {  // the diagonal block is the last entry of every row: causal mask inside it
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (32 * mt + c_row(v, hf) > qloc) sacc[mt][v] = -__builtin_inff();
    }
    float mx = -__builtin_inff();
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[mt][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m, mx);
    const float alpha = fast_exp2((m - m_new) * P.scale_log2e);
    const float neg_m = -m_new * P.scale_log2e;
    float rs = 0.f;
    bf16x8 pb[4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float pv = fast_exp2(__builtin_fmaf(sacc[mt][v], P.scale_log2e, neg_m));
        rs += pv;
        pb[2 * mt + (v >> 3)][v & 7] = (bf16)pv;
      }
    l = l * alpha + rs;
    m = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // rescale only when some row's max moved
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
    }
    // ---- V half-tile: loads of K_{t+1} may stay in flight
    if (more) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    if (more) issue(2 * t + 3);
    const bf16* Vs = slots[(2 * t + 1) % 3];
    {
      bf16x8 va[D / 32][4];
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) va[dt][kk] = lds_tr_operand<D>(Vs, kk, dt, lane);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) oacc[dt] = mfma32(va[dt][kk], pb[kk], oacc[dt]);
    }
  }

  l += __shfl_xor(l, 32, 64);
  const float inv = 1.0f / l;
  if (qvalid) {
    const int64_t obase = (tq * P.Hq + h) * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int d0 = 32 * dt + 8 * vg + 4 * hf;
        float x0 = oacc[dt][4 * vg] * inv, x1 = oacc[dt][4 * vg + 1] * inv, x2 = oacc[dt][4 * vg + 2] * inv,
              x3 = oacc[dt][4 * vg + 3] * inv;
        if (OUT_F32) {
          *(float4*)((float*)P.o + obase + d0) = make_float4(x0, x1, x2, x3);
        } else {
          bf16x4 y;
          y[0] = (bf16)x0; y[1] = (bf16)x1; y[2] = (bf16)x2; y[3] = (bf16)x3;
          *(bf16x4*)((bf16*)P.o + obase + d0) = y;
        }
      }
    if (hf == 0) P.lse[(int64_t)h * P.T + tq] = (m * P.scale_log2e + __builtin_log2f(l)) * 0.69314718055994531f;
  }
  timer.stop(P);
}

// float -> bf16 (round to nearest even) copy used when the caller's tensors are float
__global__ __launch_bounds__(256) void f32_to_bf16_kernel(const float* __restrict__ src, bf16* __restrict__ dst, int64_t n4) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n4) return;
  float4 x = ((const float4*)src)[idx];
  bf16x4 y;
  y[0] = (bf16)x.x; y[1] = (bf16)x.y; y[2] = (bf16)x.z; y[3] = (bf16)x.w;
  ((bf16x4*)dst)[idx] = y;
}

int convert_f32_to_bf16(const void* src, void* dst, int64_t n, hipStream_t st) {
  const int64_t n4 = n / 4;  // element counts are multiples of head_dim
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, (const float*)src, (bf16*)dst, n4);
  SB_LAUNCH_CHECK("f32_to_bf16_kernel");
  return SB_OK;
}

}  // namespace sb

using namespace sb;

extern "C" int sb_sparse_attn_fwd(const sb_problem* p, const void* q, const void* k, const void* v,
                                  const int32_t* sel_rowptr, const int32_t* sel_idx, const void* plan, void* o,
                                  float* lse, void* ws, void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) return SB_OK;
  if (!q || !k || !v || !sel_rowptr || !sel_idx || !plan || !o || !lse || !ws) { set_error("null argument"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  PlanOffsets po = plan_offsets(g);
  WsOffsets wo = fwd_ws_offsets(g);
  const char* pb = (const char*)plan;
  char* wb = (char*)ws;
  Tables t = make_tables(g, p, (void*)(pb + po.tables));
  AttnParams P{};
  if (g.dtype == SB_F32) {
    if ((rc = convert_f32_to_bf16(q, wb + wo.qc, (int64_t)g.T * g.Hq * g.D, st)) != SB_OK) return rc;
    if ((rc = convert_f32_to_bf16(k, wb + wo.kc, (int64_t)g.T * g.Hkv * g.D, st)) != SB_OK) return rc;
    if ((rc = convert_f32_to_bf16(v, wb + wo.vc, (int64_t)g.T * g.Hkv * g.D, st)) != SB_OK) return rc;
    P.q = (const bf16*)(wb + wo.qc); P.k = (const bf16*)(wb + wo.kc); P.v = (const bf16*)(wb + wo.vc);
  } else {
    P.q = (const bf16*)q; P.k = (const bf16*)k; P.v = (const bf16*)v;
  }
  P.o = o; P.lse = lse;
  P.rowptr = sel_rowptr; P.idx = sel_idx; P.work = (const int32_t*)(pb + po.work_fwd);
  P.cu = t.cu; P.qb_off = t.qb_off; P.qb_seq = t.qb_seq; P.bm_off = t.bm_off;
  P.NQB = g.NQB; P.T = g.T; P.Hq = g.Hq; P.Hkv = g.Hkv; P.G = g.G; P.Hs = g.Hs; P.mode = g.mode;
  P.scale = g.softmax_scale; P.scale_log2e = g.softmax_scale * 1.4426950408889634f;
  P.out_f32 = g.dtype == SB_F32;
  P.cu_busy = nullptr;
  if (g_instrument & 1) {
    SB_CHECK_HIP(hipMemsetAsync(wb + wo.cu_busy, 0, sizeof(uint64_t) * SB_CU_SLOTS, st));
    P.cu_busy = (unsigned long long*)(wb + wo.cu_busy);
  }
  const int G = g.mode == SB_SELECT_PER_QHEAD ? 1 : g.G;
  const int parts = (G + 3) / 4, hpp = (G + parts - 1) / parts;  // query heads per workgroup <= 4
  dim3 grid((unsigned)(g.Hs * g.NQB), (unsigned)parts), block((unsigned)(128 * hpp));
  KernelTimer kt(K_FWD, st);
#define SB_FWD_LAUNCH(DD, FF)                                                                         \
  do {                                                                                                \
    if (hpp == 1) hipLaunchKernelGGL((attn_fwd_kernel<DD, FF, 128>), grid, block, 0, st, P);          \
    else if (hpp == 2) hipLaunchKernelGGL((attn_fwd_kernel<DD, FF, 256>), grid, block, 0, st, P);     \
    else hipLaunchKernelGGL((attn_fwd_kernel<DD, FF, 512>), grid, block, 0, st, P);                   \
  } while (0)
  if (g.D == 128) {
    if (P.out_f32) SB_FWD_LAUNCH(128, true); else SB_FWD_LAUNCH(128, false);
  } else {
    if (P.out_f32) SB_FWD_LAUNCH(64, true); else SB_FWD_LAUNCH(64, false);
  }
#undef SB_FWD_LAUNCH
  SB_LAUNCH_CHECK("attn_fwd_kernel");
  return SB_OK;
}
