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
// Query-major dQ kernel.  Same work items and strips as the forward.  The K and V tiles of the
// selected blocks are double-buffered in LDS as whole tiles: while tile t is consumed, tile t+1 is
// in flight (asynchronous global->LDS loads).  K is read row-wise for S^T = K Q^T and through the
// transposing LDS read for dQ^T += K^T dS^T; V is read row-wise for dP^T = V dO^T.
template <int D, bool OUT_F32, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(MAXT >= 256 ? 2 : 1))) void attn_bwd_dq_kernel(AttnParams P) {
  __shared__ __attribute__((aligned(1024))) bf16 tiles[2][2][64 * D];  // [buffer][K, V]
  constexpr int kJ = 256;
  __shared__ int jbuf[kJ];
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
  const int hh = blockIdx.y * (nthr >> 7) + (wave >> 1), strip = wave & 1;
  const bool head_ok = P.mode == SB_SELECT_PER_QHEAD || hh < P.G;
  const int h = P.mode == SB_SELECT_PER_QHEAD ? hs : hs * P.G + (head_ok ? hh : 0);
  const int g = h / P.G;
  const int qloc = strip * 32 + l32;
  const bool qvalid = head_ok && i * 64 + qloc < L;
  const int64_t tq = seq0 + i * 64 + qloc;
  const int e0 = P.rowptr[row], ntiles = P.rowptr[row + 1] - e0;

  auto stage_indices = [&](int t0) {
    __syncthreads();
    for (int a = tid; a < kJ; a += nthr) jbuf[a] = t0 + a < ntiles ? P.idx[e0 + t0 + a] : 0;
    __syncthreads();
  };
  TileLoader<D> loader;
  loader.init(P.Hkv, wave, lane);
  auto issue = [&](int t) {
    const int j = __builtin_amdgcn_readfirstlane(jbuf[t % kJ]);
    const int64_t kv0 = seq0 + (int64_t)j * 64;
    const int kvalid = min(64, L - j * 64);
    loader.issue(tiles[t & 1][0], P.k, kv0, kvalid, P.Hkv, g);
    loader.issue(tiles[t & 1][1], P.v, kv0, kvalid, P.Hkv, g);
  };

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
  stage_indices(0);
  // everything loaded so far must have landed before the tile loads start (see the forward kernel)
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(qf[ks]), "+v"(dof[ks]));
  asm volatile("" : "+v"(lse2), "+v"(dr));
  issue(0);

  f32x16 dqacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) dqacc[dt] = zero16();

  for (int t = 0; t < ntiles; ++t) {
    const bool more = t + 1 < ntiles;
    if (more && (t + 1) % kJ == 0) stage_indices(t + 1);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();  // tile t has landed for everyone; everyone is done with tile t-1
    if (more) issue(t + 1);
    const bf16* Ks = tiles[t & 1][0];
    const bf16* Vs = tiles[t & 1][1];
    const bool diag = t == ntiles - 1;
    bf16x8 dsb[4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) sacc = mfma32(lds_row8<D>(Ks, 32 * mt + l32, 2 * ks + hf), qf[ks], sacc);
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) dpacc = mfma32(lds_row8<D>(Vs, 32 * mt + l32, 2 * ks + hf), dof[ks], dpacc);
      if (diag) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (32 * mt + c_row(v, hf) > qloc) sacc[v] = -__builtin_inff();
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float pv = fast_exp2(__builtin_fmaf(sacc[v], P.scale_log2e, -lse2));
        dsb[2 * mt + (v >> 3)][v & 7] = (bf16)(pv * (dpacc[v] - dr));
      }
    }
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) dqacc[dt] = mfma32(lds_tr_operand<D>(Ks, kk, dt, lane), dsb[kk], dqacc[dt]);
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
// Key-major dK/dV kernel: 2 wavefronts, each owns 32 keys of key block (s, g, j) and keeps their
// K and V rows in registers.  The Q and dO tiles (plus LSE and Dr) of the query blocks that kept j
// are double-buffered in LDS by asynchronous loads; both are read row-wise (S = Q K^T, dP = dO V^T)
// and through the transposing LDS read (dV += P^T dO, dK += dS^T Q).
// The column's query blocks come from the transpose bitmap, staged in LDS 64 words (2048 query
// blocks) per selection head at a time and walked in ascending order.
template <int D, bool OUT_F32>
__global__ __launch_bounds__(128) void attn_bwd_dkv_kernel(AttnParams P) {
  __shared__ __attribute__((aligned(1024))) bf16 tiles[2][2][64 * D];  // [buffer][Q, dO]
  __shared__ __attribute__((aligned(256))) float rowstat[2][2][64];    // [buffer][LSE, Dr]
  __shared__ uint32_t bm_s[8][64];
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
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

  TileLoader<D> loader;
  loader.init(P.Hq, wave, lane);
  auto issue = [&](int buf, int i, int h) {
    const int64_t q0 = seq0 + (int64_t)i * 64;
    const int qv = min(64, L - i * 64);
    loader.issue(tiles[buf][0], P.q, q0, qv, P.Hq, h);
    loader.issue(tiles[buf][1], P.d_o, q0, qv, P.Hq, h);
    // 64 LSE and 64 Dr values: one 4-byte load per lane, wavefront 0 takes LSE and wavefront 1 Dr
    const float* src = (wave == 0 ? P.lse : P.drow) + (int64_t)h * P.T + q0 + min(lane, qv - 1);
    dma4(src, lds_offset(rowstat[buf][wave]));
  };

  for (int w0 = (j >> 5) & ~63; w0 < words; w0 += 64) {  // chunks of 64 bitmap words
    const int wn = min(64, words - w0);
    __syncthreads();
    for (int a = tid; a < nsel * 64; a += 128) {
      const int sel = a >> 6, w = a & 63;
      const int hs = P.mode == SB_SELECT_PER_QHEAD ? g * P.G + sel : g;
      bm_s[sel][w] = w < wn ? P.bitmap[(int64_t)P.Hs * P.bm_off[s] + ((int64_t)hs * n + j) * words + w0 + w] : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(kf[ks]), "+v"(vf[ks]));
    // iterator over (query block i, query head h) in the order (selection head, i ascending, head)
    int it_sel = 0, it_w = -1, it_hb = 0, it_i = 0;
    uint32_t it_bits = 0;
    auto next = [&](int& i, int& h) -> bool {
      if (it_hb > 0 && it_hb < hpe) { i = it_i; h = g * P.G + it_hb; ++it_hb; return true; }
      while (true) {
        if (it_bits) {
          const int b = __builtin_ctz(it_bits);
          it_bits &= it_bits - 1;
          it_i = 32 * (w0 + it_w) + b;
          i = it_i;
          h = P.mode == SB_SELECT_PER_QHEAD ? g * P.G + it_sel : g * P.G;
          it_hb = 1;
          return true;
        }
        ++it_w;
        if (it_w >= wn) { it_w = 0; ++it_sel; }
        if (it_sel >= nsel) return false;
        it_bits = __builtin_amdgcn_readfirstlane(bm_s[it_sel][it_w]);
      }
    };
    int ci, ch, ni = 0, nh = 0;
    bool have = next(ci, ch);
    if (have) issue(0, ci, ch);
    for (int t = 0; have; ++t) {
      const bool more = next(ni, nh);
      wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      if (more) issue((t + 1) & 1, ni, nh);
      const bf16* Qs = tiles[t & 1][0];
      const bf16* dOs = tiles[t & 1][1];
      const float* lse_s = rowstat[t & 1][0];
      const float* dr_s = rowstat[t & 1][1];
      const int qv = min(64, L - ci * 64);
      const bool diag = ci == j;
      bf16x8 pa[4], dsa[4];
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) sacc = mfma32(lds_row8<D>(Qs, 32 * qt + l32, 2 * ks + hf), kf[ks], sacc);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) dpacc = mfma32(lds_row8<D>(dOs, 32 * qt + l32, 2 * ks + hf), vf[ks], dpacc);
#pragma unroll
        for (int vg = 0; vg < 4; ++vg) {
          const int qr = 32 * qt + 8 * vg + 4 * hf;  // query rows qr..qr+3 are registers 4vg..4vg+3
          const float4 ls = *(const float4*)(lse_s + qr);
          const float4 dd = *(const float4*)(dr_s + qr);
          const float lsv[4] = {ls.x, ls.y, ls.z, ls.w};
          const float ddv[4] = {dd.x, dd.y, dd.z, dd.w};
          if (diag || qv < 64) {  // causal mask inside the diagonal block, rows past the sequence end
#pragma unroll
            for (int c = 0; c < 4; ++c)
              if ((diag && kloc > qr + c) || qr + c >= qv) sacc[4 * vg + c] = -__builtin_inff();
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int v = 4 * vg + c;
            float pv = fast_exp2(__builtin_fmaf(sacc[v], P.scale_log2e, -lsv[c] * 1.4426950408889634f));
            pa[2 * qt + (v >> 3)][v & 7] = (bf16)pv;
            dsa[2 * qt + (v >> 3)][v & 7] = (bf16)(pv * (dpacc[v] - ddv[c]));
          }
        }
      }
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          dvacc[dt] = mfma32(pa[kk], lds_tr_operand<D>(dOs, kk, dt, lane), dvacc[dt]);
          dkacc[dt] = mfma32(dsa[kk], lds_tr_operand<D>(Qs, kk, dt, lane), dkacc[dt]);
        }
      have = more; ci = ni; ch = nh;
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
  dim3 grid((unsigned)(g.Hkv * g.NQB)), block(128);
  KernelTimer kt(K_BWD_DKV, st);
  hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, F32>), grid, block, 0, st, P);
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
