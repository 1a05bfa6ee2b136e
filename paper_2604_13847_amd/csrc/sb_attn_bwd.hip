// Block-sparse attention backward (gradient of paper Eq. 2 with the selection held fixed).
//
//   Dr = rowsum(dO * O)                                    (prep kernel)
//   P  = exp(scale * S - LSE),  dP = dO V^T,  dS = P * (dP - Dr)
//   dQ = scale * dS K          query-major kernel, same work items and tile walk as the forward
//   dK = scale * dS^T Q, dV = P^T dO   key-major kernel: one workgroup owns key block (s, g, j),
//        keeps its K/V strip in registers, walks the query blocks that kept j (transpose bitmap,
//        ascending) for every query head of the KV group and accumulates in registers; each output
//        element is written once, in a fixed order, so the result is deterministic.
#include "sb_attn_common.h"

namespace sb {

// ---------------------------------------------------------------------------------------------
template <bool O_F32>
__global__ __launch_bounds__(256) void bwd_prep_kernel(const void* __restrict__ o, const bf16* __restrict__ d_o, int64_t rows,
                                                       int T, int Hq, int D, float* __restrict__ drow) {
  const int lpr = D / 8;  // lanes per (token, head) row, 8 elements each
  const int64_t r = ((int64_t)blockIdx.x * 256 + threadIdx.x) / lpr;
  const int c = threadIdx.x % lpr;
  float acc = 0.f;
  if (r < rows) {
    bf16x8 a = *(const bf16x8*)(d_o + r * D + 8 * c);
    if (O_F32) {
      const float* op = (const float*)o + r * D + 8 * c;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc += (float)a[e] * op[e];
    } else {
      bf16x8 b = *(const bf16x8*)((const bf16*)o + r * D + 8 * c);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
    }
  }
  for (int off = lpr >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (r < rows && c == 0) {
    const int64_t t = r / Hq;
    const int h = (int)(r - t * Hq);
    drow[(int64_t)h * T + t] = acc;
  }
}

// ---------------------------------------------------------------------------------------------
template <int D, bool OUT_F32, int MAXT>
__global__ __launch_bounds__(MAXT) void attn_bwd_dq_kernel(AttnParams P) {
  constexpr int KLD = D + 8, TLD = 64 + 8;
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * KLD];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * KLD];
  __shared__ __attribute__((aligned(16))) bf16 Kt[D * TLD];
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int64_t row = P.work[blockIdx.x];
  const int hs = (int)(row / P.NQB);
  const int qb = (int)(row - (int64_t)hs * P.NQB);
  const int s = P.qb_seq[qb];
  const int i = qb - P.qb_off[s];
  const int64_t seq0 = P.cu[s];
  const int L = P.cu[s + 1] - P.cu[s];
  const int hh = blockIdx.y * (nthr >> 7) + (wave >> 1), strip = wave & 1;
  const bool head_ok = P.mode == SB_SELECT_PER_QHEAD || hh < P.G;
  const int h = P.mode == SB_SELECT_PER_QHEAD ? hs : hs * P.G + (head_ok ? hh : 0);
  const int g = h / P.G;
  const int qloc = strip * 32 + l32;
  const bool qvalid = head_ok && i * 64 + qloc < L;
  const int64_t tq = seq0 + i * 64 + qloc;

  bf16x8 qf[D / 16], dof[D / 16];
  float lse2 = __builtin_inff(), dr = 0.f;  // invalid rows: P = exp2(x - inf) = 0
  {
    const bf16* qp = P.q + (tq * P.Hq + h) * D + 8 * hf;
    const bf16* dp = P.d_o + (tq * P.Hq + h) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      qf[ks] = qvalid ? *(const bf16x8*)(qp + 16 * ks) : zero_bf16x8();
      dof[ks] = qvalid ? *(const bf16x8*)(dp + 16 * ks) : zero_bf16x8();
    }
    if (qvalid) {
      lse2 = P.lse[(int64_t)h * P.T + tq] * 1.4426950408889634f;
      dr = P.drow[(int64_t)h * P.T + tq];
    }
  }
  f32x16 dqacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) dqacc[dt] = zero16();

  const int e0 = P.rowptr[row], e1 = P.rowptr[row + 1];
  for (int e = e0; e < e1; ++e) {
    const int j = P.idx[e];
    const int64_t kv0 = seq0 + (int64_t)j * 64;
    const int kvalid = min(64, L - j * 64);
    __syncthreads();
    load_tile_transposed<D, KLD, TLD>(Kt, Ks, P.k, kv0, kvalid, P.Hkv, g, tid, nthr);
    load_tile_rowmajor<D, KLD>(Vs, P.v, kv0, kvalid, P.Hkv, g, tid, nthr);
    __syncthreads();
    const bool diag = j == i;
    bf16x8 dsb[4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        bf16x8 a = *(const bf16x8*)(Ks + (32 * mt + l32) * KLD + 16 * ks + 8 * hf);
        sacc = mfma32(a, qf[ks], sacc);
      }
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        bf16x8 a = *(const bf16x8*)(Vs + (32 * mt + l32) * KLD + 16 * ks + 8 * hf);
        dpacc = mfma32(a, dof[ks], dpacc);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float pv = fast_exp2(sacc[v] * P.scale_log2e - lse2);
        if (diag && 32 * mt + c_row(v, hf) > qloc) pv = 0.f;
        dsb[2 * mt + (v >> 3)][v & 7] = (bf16)(pv * (dpacc[v] - dr));
      }
    }
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 a = *(const bf16x8*)(Kt + (32 * dt + l32) * TLD + 16 * kk + 8 * hf);
        dqacc[dt] = mfma32(a, dsb[kk], dqacc[dt]);
      }
  }
  if (qvalid) {
    const int64_t obase = (tq * P.Hq + h) * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int d0 = 32 * dt + 8 * vg + 4 * hf;
        float x0 = dqacc[dt][4 * vg] * P.scale, x1 = dqacc[dt][4 * vg + 1] * P.scale, x2 = dqacc[dt][4 * vg + 2] * P.scale,
              x3 = dqacc[dt][4 * vg + 3] * P.scale;
        if (OUT_F32) {
          *(float4*)((float*)P.dq + obase + d0) = make_float4(x0, x1, x2, x3);
        } else {
          bf16x4 y;
          y[0] = (bf16)x0; y[1] = (bf16)x1; y[2] = (bf16)x2; y[3] = (bf16)x3;
          *(bf16x4*)((bf16*)P.dq + obase + d0) = y;
        }
      }
  }
  timer.stop(P);
}

// ---------------------------------------------------------------------------------------------
// Key-major kernel: 2 wavefronts, each owns 32 keys of the block.
template <int D, bool OUT_F32>
__global__ __launch_bounds__(128) void attn_bwd_dkv_kernel(AttnParams P) {
  constexpr int QLD = D + 8, TLD = 64 + 8;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  bf16* Qs = (bf16*)smem;          // [64][QLD]
  bf16* dOs = Qs + 64 * QLD;       // [64][QLD]
  bf16* Qt = dOs + 64 * QLD;       // [D][TLD]
  bf16* dOt = Qt + D * TLD;        // [D][TLD]
  float* lse_s = (float*)(dOt + D * TLD);  // [64] LSE * log2(e), +inf for rows past the sequence end
  float* dr_s = lse_s + 64;                // [64]
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int64_t col = P.work[blockIdx.x];  // g * NQB + global block index
  const int g = (int)(col / P.NQB);
  const int qbj = (int)(col - (int64_t)g * P.NQB);
  const int s = P.qb_seq[qbj];
  const int j = qbj - P.qb_off[s];
  const int n = P.qb_off[s + 1] - P.qb_off[s];
  const int64_t seq0 = P.cu[s];
  const int L = P.cu[s + 1] - P.cu[s];
  const int kloc = wave * 32 + l32;
  const bool kvalid = j * 64 + kloc < L;
  const int64_t tk = seq0 + j * 64 + kloc;

  bf16x8 kf[D / 16], vf[D / 16];
  {
    const bf16* kp = P.k + (tk * P.Hkv + g) * D + 8 * hf;
    const bf16* vp = P.v + (tk * P.Hkv + g) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      kf[ks] = kvalid ? *(const bf16x8*)(kp + 16 * ks) : zero_bf16x8();
      vf[ks] = kvalid ? *(const bf16x8*)(vp + 16 * ks) : zero_bf16x8();
    }
  }
  f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) { dkacc[dt] = zero16(); dvacc[dt] = zero16(); }

  const int words = (n + 31) >> 5;
  const int nsel = P.mode == SB_SELECT_PER_QHEAD ? P.G : 1;   // bitmap columns to walk
  const int hpe = P.mode == SB_SELECT_PER_QHEAD ? 1 : P.G;    // query heads per set bit
  for (int a = 0; a < nsel; ++a) {
    const int hs = P.mode == SB_SELECT_PER_QHEAD ? g * P.G + a : g;
    const uint32_t* bm = P.bitmap + (int64_t)P.Hs * P.bm_off[s] + ((int64_t)hs * n + j) * words;
    for (int wi = j >> 5; wi < words; ++wi) {
      uint32_t bits = bm[wi];
      while (bits) {
        const int b = __builtin_ctz(bits);
        bits &= bits - 1;
        const int i = 32 * wi + b;
        const int64_t q0 = seq0 + (int64_t)i * 64;
        const int qvalid = min(64, L - i * 64);
        const bool diag = i == j;
        for (int hb = 0; hb < hpe; ++hb) {
          const int h = P.mode == SB_SELECT_PER_QHEAD ? hs : g * P.G + hb;
          __syncthreads();
          load_tile_transposed<D, QLD, TLD>(Qt, Qs, P.q, q0, qvalid, P.Hq, h, tid, 128);
          load_tile_transposed<D, QLD, TLD>(dOt, dOs, P.d_o, q0, qvalid, P.Hq, h, tid, 128);
          if (tid < 64) {
            const bool ok = tid < qvalid;
            lse_s[tid] = ok ? P.lse[(int64_t)h * P.T + q0 + tid] * 1.4426950408889634f : __builtin_inff();
            dr_s[tid] = ok ? P.drow[(int64_t)h * P.T + q0 + tid] : 0.f;
          }
          __syncthreads();
          bf16x8 pa[4], dsa[4];
#pragma unroll
          for (int qt = 0; qt < 2; ++qt) {
            f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
              bf16x8 qa = *(const bf16x8*)(Qs + (32 * qt + l32) * QLD + 16 * ks + 8 * hf);
              sacc = mfma32(qa, kf[ks], sacc);
            }
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
              bf16x8 da = *(const bf16x8*)(dOs + (32 * qt + l32) * QLD + 16 * ks + 8 * hf);
              dpacc = mfma32(da, vf[ks], dpacc);
            }
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
              const int qr = 32 * qt + 8 * vg + 4 * hf;  // query rows qr..qr+3 are registers 4vg..4vg+3
              const float4 ls = *(const float4*)(lse_s + qr);
              const float4 dd = *(const float4*)(dr_s + qr);
              const float lsv[4] = {ls.x, ls.y, ls.z, ls.w};
              const float ddv[4] = {dd.x, dd.y, dd.z, dd.w};
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                const int v = 4 * vg + c;
                float pv = fast_exp2(sacc[v] * P.scale_log2e - lsv[c]);
                if (diag && kloc > qr + c) pv = 0.f;
                pa[2 * qt + (v >> 3)][v & 7] = (bf16)pv;
                dsa[2 * qt + (v >> 3)][v & 7] = (bf16)(pv * (dpacc[v] - ddv[c]));
              }
            }
          }
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
              bf16x8 db = *(const bf16x8*)(dOt + (32 * dt + l32) * TLD + 16 * kk + 8 * hf);
              dvacc[dt] = mfma32(pa[kk], db, dvacc[dt]);
              bf16x8 qbv = *(const bf16x8*)(Qt + (32 * dt + l32) * TLD + 16 * kk + 8 * hf);
              dkacc[dt] = mfma32(dsa[kk], qbv, dkacc[dt]);
            }
        }
      }
    }
  }
  // C layout: column = d (32dt + l32), register v = key row c_row(v, hf) of this wavefront's strip
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int kr = wave * 32 + c_row(v, hf);
      if (j * 64 + kr < L) {
        const int64_t off = ((seq0 + j * 64 + kr) * P.Hkv + g) * D + 32 * dt + l32;
        if (OUT_F32) {
          ((float*)P.dk)[off] = dkacc[dt][v] * P.scale;
          ((float*)P.dv)[off] = dvacc[dt][v];
        } else {
          ((bf16*)P.dk)[off] = (bf16)(dkacc[dt][v] * P.scale);
          ((bf16*)P.dv)[off] = (bf16)dvacc[dt][v];
        }
      }
    }
  timer.stop(P);
}

int convert_f32_to_bf16(const void* src, void* dst, int64_t n, hipStream_t st);

template <int D, bool F32>
static int launch_bwd(const Geo& g, const AttnParams& P, hipStream_t st) {
  constexpr int QLD = D + 8, TLD = 64 + 8;
  // query-major dQ
  const int G = g.mode == SB_SELECT_PER_QHEAD ? 1 : g.G;
  const int parts = (G + 3) / 4, hpp = (G + parts - 1) / parts;
  AttnParams Pq = P;
  Pq.work = P.work;  // forward work list
  dim3 grid((unsigned)(g.Hs * g.NQB), (unsigned)parts), block((unsigned)(128 * hpp));
  KernelTimer kt(K_BWD_DQ, st);
  if (hpp == 1) hipLaunchKernelGGL((attn_bwd_dq_kernel<D, F32, 128>), grid, block, 0, st, Pq);
  else if (hpp == 2) hipLaunchKernelGGL((attn_bwd_dq_kernel<D, F32, 256>), grid, block, 0, st, Pq);
  else hipLaunchKernelGGL((attn_bwd_dq_kernel<D, F32, 512>), grid, block, 0, st, Pq);
  SB_LAUNCH_CHECK("attn_bwd_dq_kernel");
  return SB_OK;
}

template <int D, bool F32>
static int launch_dkv(const Geo& g, const AttnParams& P, hipStream_t st) {
  constexpr int QLD = D + 8, TLD = 64 + 8;
  const size_t smem = sizeof(bf16) * (size_t)(2 * 64 * QLD + 2 * D * TLD) + sizeof(float) * 128;
  static bool attr_set = false;
  if (!attr_set) {
    SB_CHECK_HIP(hipFuncSetAttribute((const void*)attn_bwd_dkv_kernel<D, F32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  dim3 grid((unsigned)(g.Hkv * g.NQB)), block(128);
  KernelTimer kt(K_BWD_DKV, st);
  hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, F32>), grid, block, smem, st, P);
  SB_LAUNCH_CHECK("attn_bwd_dkv_kernel");
  return SB_OK;
}

}  // namespace sb

using namespace sb;

extern "C" int sb_sparse_attn_bwd(const sb_problem* p, const void* q, const void* k, const void* v, const void* o,
                                  const float* lse, const void* d_o, const int32_t* sel_rowptr, const int32_t* sel_idx,
                                  const void* plan, void* dq, void* dk, void* dv, void* ws, void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) return SB_OK;
  if (!q || !k || !v || !o || !lse || !d_o || !sel_rowptr || !sel_idx || !plan || !dq || !dk || !dv || !ws) {
    set_error("null argument");
    return SB_ERR_INVALID_ARG;
  }
  hipStream_t st = (hipStream_t)stream;
  PlanOffsets po = plan_offsets(g);
  WsOffsets wo = bwd_ws_offsets(g);
  const char* pb = (const char*)plan;
  char* wb = (char*)ws;
  Tables t = make_tables(g, p, (void*)(pb + po.tables));
  AttnParams P{};
  const bool f32 = g.dtype == SB_F32;
  if (f32) {
    if ((rc = convert_f32_to_bf16(q, wb + wo.qc, (int64_t)g.T * g.Hq * g.D, st)) != SB_OK) return rc;
    if ((rc = convert_f32_to_bf16(k, wb + wo.kc, (int64_t)g.T * g.Hkv * g.D, st)) != SB_OK) return rc;
    if ((rc = convert_f32_to_bf16(v, wb + wo.vc, (int64_t)g.T * g.Hkv * g.D, st)) != SB_OK) return rc;
    if ((rc = convert_f32_to_bf16(d_o, wb + wo.doc, (int64_t)g.T * g.Hq * g.D, st)) != SB_OK) return rc;
    P.q = (const bf16*)(wb + wo.qc); P.k = (const bf16*)(wb + wo.kc); P.v = (const bf16*)(wb + wo.vc);
    P.d_o = (const bf16*)(wb + wo.doc);
  } else {
    P.q = (const bf16*)q; P.k = (const bf16*)k; P.v = (const bf16*)v; P.d_o = (const bf16*)d_o;
  }
  float* drow = (float*)(wb + wo.drow);
  P.lse = (float*)lse; P.drow = drow; P.dq = dq; P.dk = dk; P.dv = dv;
  P.rowptr = sel_rowptr; P.idx = sel_idx;
  P.bitmap = (const uint32_t*)(pb + po.bitmap);
  P.cu = t.cu; P.qb_off = t.qb_off; P.qb_seq = t.qb_seq; P.bm_off = t.bm_off;
  P.NQB = g.NQB; P.T = g.T; P.Hq = g.Hq; P.Hkv = g.Hkv; P.G = g.G; P.Hs = g.Hs; P.mode = g.mode;
  P.scale = g.softmax_scale; P.scale_log2e = g.softmax_scale * 1.4426950408889634f;
  P.out_f32 = f32;
  P.cu_busy = nullptr;
  if (g_instrument & 1) {
    SB_CHECK_HIP(hipMemsetAsync(wb + wo.cu_busy, 0, sizeof(uint64_t) * SB_CU_SLOTS, st));
    P.cu_busy = (unsigned long long*)(wb + wo.cu_busy);
  }
  const int64_t rows = (int64_t)g.T * g.Hq;
  const int rows_per_wg = 256 / (g.D / 8);
  dim3 pgrid((unsigned)((rows + rows_per_wg - 1) / rows_per_wg));
  {
  KernelTimer kt(K_BWD_PREP, st);
  if (f32) hipLaunchKernelGGL(bwd_prep_kernel<true>, pgrid, dim3(256), 0, st, o, P.d_o, rows, g.T, g.Hq, g.D, drow);
  else hipLaunchKernelGGL(bwd_prep_kernel<false>, pgrid, dim3(256), 0, st, o, P.d_o, rows, g.T, g.Hq, g.D, drow);
  }
  SB_LAUNCH_CHECK("bwd_prep_kernel");

  AttnParams Pq = P, Pk = P;
  Pq.work = (const int32_t*)(pb + po.work_fwd);
  Pk.work = (const int32_t*)(pb + po.work_bwd);
  if (g.D == 128) {
    rc = f32 ? launch_bwd<128, true>(g, Pq, st) : launch_bwd<128, false>(g, Pq, st);
    if (rc != SB_OK) return rc;
    rc = f32 ? launch_dkv<128, true>(g, Pk, st) : launch_dkv<128, false>(g, Pk, st);
  } else {
    rc = f32 ? launch_bwd<64, true>(g, Pq, st) : launch_bwd<64, false>(g, Pq, st);
    if (rc != SB_OK) return rc;
    rc = f32 ? launch_dkv<64, true>(g, Pk, st) : launch_dkv<64, false>(g, Pk, st);
  }
  return rc;
}
