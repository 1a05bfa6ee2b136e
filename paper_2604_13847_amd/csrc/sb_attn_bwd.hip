// Block-sparse attention backward (gradient of paper Eq. 2 with the selection held fixed).
//
//   Dr = rowsum(dO * O)                                    (prologue of the query-major kernel, which owns every row once)
//   P  = exp(scale * S - LSE),  dP = dO V^T,  dS = P * (dP - Dr)
//   dQ = scale * dS K          query-major kernel, same work items and tile walk as the forward
//   dK = scale * dS^T Q, dV = P^T dO   key-major kernel: one workgroup owns key block (s, g, j),
//        keeps its K/V strip in registers, walks the query blocks that kept j (transpose bitmap, last
//        query block first) for every query head of the KV group and accumulates in registers; each output
//        element is written once, in a fixed order, so the result is deterministic.
#include <type_traits>

#include "sb_attn_common.h"

namespace sb {

// ---------------------------------------------------------------------------------------------
// Query-major dQ kernel.  Same work items as the forward.  A workgroup takes one item (sequence,
// selection head, query block) and HPW query heads that share its selection (one in per-query-head
// mode); the K and V tiles of the selected blocks are double-buffered in LDS as whole tiles by
// asynchronous loads and shared by all wavefronts of the workgroup.  A wavefront owns 32 query rows
// of one head and, with the key split KS = 2, one 32-key half of every tile (the two partial dQ of a
// row are added through LDS at the end); Q, dO, LSE and Dr of its rows stay in registers.  Every (token,
// query head) row belongs to exactly one workgroup of this kernel, so its prologue is also where Dr is
// computed (from the dO registers and one read of O) and left, with LSE * log2 e, for the key-major kernel.
// Transposed products put a query in a C-matrix column: S^T = K Q^T, dP^T = V dO^T, so LSE and Dr are
// per-lane scalars and dS^T converts to the B operand of dQ^T += K^T dS^T without cross-lane movement;
// K^T comes from the row-major K tile through the transposing LDS read.
// The register budget (256) lets two wavefronts share a SIMD: one runs its exponentials while the
// other runs matrix instructions.  Operands are fetched from LDS in sets of D/16, a set ahead of use.
template <int D, bool OUT_F32, int KS, int MAXT>
__global__ __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(2))) void attn_bwd_dq_kernel(AttnParams P, int heads) {
  constexpr int TILE_B = 64 * D * 2, ROW_B = D * 2, NOP = D / 16;
  constexpr int NMT = 2 / KS;  // 32-key halves of a tile this wavefront computes
  __shared__ __attribute__((aligned(1024))) bf16 tiles[2][2][64 * D];  // [buffer][K, V]
  constexpr int kJ = 256;
  __shared__ int jbuf[kJ];
  static_assert(KS == 1 || sizeof(tiles) >= (MAXT / 128) * 16 * (D / 32) * 64 * sizeof(float), "partial dQ must fit in the tile buffers");
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int pos = claim_item(blockIdx.x, P.n_items, P.ticket ? P.ticket + blockIdx.y : nullptr);
  if (pos < 0) return;
  const WorkItem item = P.items[pos];
  const int hs = item.hs, i = item.i, L = item.len, e0 = item.e0, ntiles = item.ntiles;
  const int64_t seq0 = item.seq0;
  const int strip = wave & 1, kh = KS == 2 ? (wave >> 1) & 1 : 0;
  const int hh = blockIdx.y * (nthr / (128 * KS)) + wave / (2 * KS);  // query head of the group this wavefront works for
  const bool head_ok = hh < heads;
  const int h = P.mode == SB_SELECT_PER_QHEAD ? hs : hs * P.G + (head_ok ? hh : 0);
  const int g = h / P.G;
  const int qloc = strip * 32 + l32;
  const bool qvalid = head_ok && i * 64 + qloc < L;
  const int64_t tq = seq0 + i * 64 + qloc;

  auto stage_indices = [&](int t0) {
    __syncthreads();
    for (int a = tid; a < kJ; a += nthr) jbuf[a] = t0 + a < ntiles ? P.idx[e0 + t0 + a] : 0;
    __syncthreads();
  };
  TileLoader<D, 4> loader;  // every workgroup of this kernel has at least four wavefronts: they share the tile loads
  loader.init(P.Hkv, wave, lane);
  auto issue = [&](int t) {
    const int j = __builtin_amdgcn_readfirstlane(jbuf[t % kJ]);
    const int64_t kv0 = seq0 + (int64_t)j * 64;
    const int kvalid = min(64, L - j * 64);
    loader.issue(tiles[t & 1][0], P.k, kv0, kvalid, P.Hkv, g);
    loader.issue(tiles[t & 1][1], P.v, kv0, kvalid, P.Hkv, g);
  };

  // B operands: column = query lane%32 of the strip, slots = d 16ks + 8hf + (0..7)
  bf16x8 qf[NOP], dof[NOP];
  float lse2 = __builtin_inff(), dr = 0.f;  // rows that do not exist: P = exp2(x - inf) = 0
  {
    const bf16* qp = P.q + (tq * P.Hq + h) * D + 8 * hf;
    const bf16* dp = P.d_o + (tq * P.Hq + h) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < NOP; ++ks) {
      qf[ks] = qvalid ? *(const bf16x8*)(qp + 16 * ks) : zero_bf16x8();
      dof[ks] = qvalid ? *(const bf16x8*)(dp + 16 * ks) : zero_bf16x8();
    }
    // Dr of the lane's query: its half of the head dimension here, the other half in lane ^ 32
    float part = 0.f;
    if (qvalid) {
      if (OUT_F32) {
        const float* op_ = (const float*)P.o + (tq * P.Hq + h) * D + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < NOP; ++ks) {
          const float4 a = *(const float4*)(op_ + 16 * ks), b = *(const float4*)(op_ + 16 * ks + 4);
          part += (float)dof[ks][0] * a.x + (float)dof[ks][1] * a.y + (float)dof[ks][2] * a.z + (float)dof[ks][3] * a.w;
          part += (float)dof[ks][4] * b.x + (float)dof[ks][5] * b.y + (float)dof[ks][6] * b.z + (float)dof[ks][7] * b.w;
        }
      } else {
        const bf16* op_ = (const bf16*)P.o + (tq * P.Hq + h) * D + 8 * hf;
#pragma unroll
        for (int ks = 0; ks < NOP; ++ks) {
          const bf16x8 ov = *(const bf16x8*)(op_ + 16 * ks);
#pragma unroll
          for (int e = 0; e < 8; ++e) part += (float)dof[ks][e] * (float)ov[e];
        }
      }
      lse2 = P.lse[(int64_t)h * P.T + tq] * 1.4426950408889634f;
    }
    dr = part + __shfl_xor(part, 32, 64);
    if (pos == 0 && blockIdx.y == 0 && tid == 0) P.lse2[(int64_t)P.Hq * P.T] = __builtin_inff();  // read by the key-major kernel in place of the LSE of rows that do not exist
  }
  stage_indices(0);
  // everything loaded so far must have landed before the tile loads start (see the forward kernel)
#pragma unroll
  for (int ks = 0; ks < NOP; ++ks) asm volatile("" : "+v"(qf[ks]), "+v"(dof[ks]));
  asm volatile("" : "+v"(lse2), "+v"(dr));
  issue(0);

  // LDS byte addresses of this lane's operand reads inside buffer 0's K tile, key half kh; the buffer
  // and everything else is a compile-time offset
  const unsigned tiles0 = lds_offset(&tiles[0][0][0]);
  unsigned row_a[NOP], tr_a[D / 32][2];
#pragma unroll
  for (int ks = 0; ks < NOP; ++ks) row_a[ks] = tiles0 + (32 * kh + l32) * ROW_B + 16 * ((2 * ks + hf) ^ chunk_swizzle<D>(l32));
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int r = 8 * half + 4 * hf + ((lane & 15) >> 2), d = 32 * dt + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      tr_a[dt][half] = tiles0 + (32 * kh + r) * ROW_B + 16 * ((d >> 3) ^ chunk_swizzle<D>(r)) + 2 * (d & 7);
    }
  auto ld_row = [&](int ks, unsigned off) __attribute__((always_inline)) {
    return *(const bf16x8 __attribute__((address_space(3)))*)(row_a[ks] + off);
  };
  // A operand of dQ^T += K^T dS^T: row = d (32dt + lane%32), slots = keys 16kk + 8(e/4) + 4hf + e%4 of this wavefront's rows
  auto ld_tr = [&](int kk, int dt, unsigned off) __attribute__((always_inline)) {
    const unsigned o = off + kk * 16 * ROW_B;
    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(tr_a[dt][0] + o));
    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(tr_a[dt][1] + o));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };

  bf16x8 op[NOP];  // one rotating operand set: a register is refilled for the next contraction as soon as it has been consumed

  // A row that keeps only its own block sees few keys: its O is not an average, |O| is of the size of |v|, and the
  // rounding of the stored O (2^-9 relative) moves rowsum(dO * O) by up to ~0.1, which dS = P (dP - Dr) amplifies
  // where one key dominates the row.  For these items Dr is taken from the identity rowsum(dO * O) = sum_j P_j dP_j
  // instead, in fp32 from the one tile the row has, normalised by sum_j P_j (P carries the rounding of the stored LSE).
  if (ntiles == 1) {
    __shared__ float drx[MAXT / 64][64];
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {
      const unsigned ro = mt * 32 * ROW_B;
      f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) op[ks] = ld_row(ks, ro);
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) sacc = mfma32(op[ks], qf[ks], sacc);
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) op[ks] = ld_row(ks, ro + TILE_B);
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) dpacc = mfma32(op[ks], dof[ks], dpacc);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const bool masked = 32 * (mt + kh) + c_row(v, hf) > qloc;  // the tile is the diagonal block
        const float pv = masked ? 0.f : fast_exp2(__builtin_fmaf(sacc[v], P.scale_log2e, -lse2));
        num = __builtin_fmaf(pv, dpacc[v], num);
        den += pv;
      }
    }
    num += __shfl_xor(num, 32, 64);
    den += __shfl_xor(den, 32, 64);
    if (KS == 2) {  // the other key half of the row is with wavefront wave ^ 2
      if (hf == 0) { drx[wave][l32] = num; drx[wave][32 + l32] = den; }
      __syncthreads();
      num += drx[wave ^ 2][l32];
      den += drx[wave ^ 2][32 + l32];
    }
    if (den > 0.f) dr = num / den;
  }
  if (qvalid && kh == 0 && hf == 0) {
    P.drow[(int64_t)h * P.T + tq] = dr;
    P.lse2[(int64_t)h * P.T + tq] = lse2;
  }

  f32x16 dqacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) dqacc[dt] = zero16();

  // The diagonal block is always the last tile of a row: it takes its own instantiation of the tile
  // body, so that the other tiles carry no mask selects.
  auto tile = [&](auto diag_c, auto buf_c, int t) __attribute__((always_inline)) {
    constexpr bool diag = decltype(diag_c)::value;
    // BUF = 0 / 1: the tile's buffer is an immediate offset of every LDS read; BUF = -1: the operand addresses are
    // moved to the other buffer after every tile
    constexpr int BUF = decltype(buf_c)::value;
    constexpr unsigned BO = BUF > 0 ? 2 * TILE_B : 0;
    const bool more = t + 1 < ntiles;
    if (more && (t + 1) % kJ == 0) stage_indices(t + 1);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();  // tile t has landed for everyone; everyone is done with tile t-1
    if (more) issue(t + 1);
    if (BUF < 0 && t > 0) {
      const int dl = (t & 1) ? 2 * TILE_B : -2 * TILE_B;
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) row_a[ks] += dl;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) { tr_a[dt][0] += dl; tr_a[dt][1] += dl; }
    }
#pragma unroll
    for (int mt = 0; mt < NMT; ++mt) {  // keys 32(mt + kh) .. +31 of the tile
      const unsigned ro = BO + mt * 32 * ROW_B;
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) op[ks] = ld_row(ks, ro);  // K rows
      __builtin_amdgcn_sched_barrier(0);
      f32x16 sacc = zero16(), dpacc = zero16();
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) {  // S^T = K Q^T, refilling every operand register with the V row operand
        sacc = mfma32(op[ks], qf[ks], sacc);
        op[ks] = ld_row(ks, ro + TILE_B);
      }
#pragma unroll
      for (int i_ = 0; i_ < NOP; ++i_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) {  // dP^T = V dO^T, refilling with the K^T operands of the dQ step
        dpacc = mfma32(op[ks], dof[ks], dpacc);
        op[ks] = ld_tr(2 * mt + ks / (D / 32), ks % (D / 32), BO);
      }
#pragma unroll
      for (int i_ = 0; i_ < NOP; ++i_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (diag) {  // causal mask inside the diagonal block (also removes keys past the end of the sequence)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (32 * (mt + kh) + c_row(v, hf) > qloc) sacc[v] = -__builtin_inff();
      }
      bf16x8 dsb[2];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float pv = fast_exp2(__builtin_fmaf(sacc[v], P.scale_log2e, -lse2));
        dsb[v >> 3][v & 7] = (bf16)(pv * (dpacc[v] - dr));
      }
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) dqacc[dt] = mfma32(op[q * (D / 32) + dt], dsb[q], dqacc[dt]);
      // the matrix instructions of the first 16 keys run under the pointwise work of the other 16
      __builtin_amdgcn_sched_group_barrier(0x002, 40, 0);
#pragma unroll
      for (int i_ = 0; i_ < D / 32; ++i_) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 40 / (D / 32), 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, D / 32, 0);
    }
  };
  if (KS == 2) {  // two tiles per iteration, so that the buffer of a tile is known at compile time
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    int t = 0;
    for (; t + 2 < ntiles; t += 2) {
      tile(std::false_type(), B0(), t);
      tile(std::false_type(), B1(), t + 1);
    }
    if (t + 2 == ntiles) {
      tile(std::false_type(), B0(), t);
      tile(std::true_type(), B1(), t + 1);
    } else {
      tile(std::true_type(), B0(), t);
    }
  } else {  // a wavefront that computes both key halves has twice the tile body: the copies would not fit the register budget
    using BR = std::integral_constant<int, -1>;
    for (int t = 0; t + 1 < ntiles; ++t) tile(std::false_type(), BR(), t);
    tile(std::true_type(), BR(), ntiles - 1);
  }
  if (KS == 2) {  // add the two key halves of every row: the kh = 1 wavefront hands its partial over
    float* xbuf = (float*)&tiles[0][0][0] + (size_t)(wave >> 2) * 2 * (16 * (D / 32) * 64) + (size_t)strip * (16 * (D / 32) * 64);
    __syncthreads();  // everyone is done with the tile buffers
    if (kh == 1) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) xbuf[(16 * dt + v) * 64 + lane] = dqacc[dt][v];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) dqacc[dt][v] += xbuf[(16 * dt + v) * 64 + lane];
    }
  }
  if (qvalid && kh == 0) {
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
// K and V rows in registers for the whole launch.  The Q and dO tiles (plus the rows' log-sum-exp
// in base 2 and Dr) of the query blocks that kept j are double-buffered in LDS by asynchronous
// loads; both are read row-wise (S = Q K^T, dP = dO V^T) and through the transposing LDS read
// (dV += P^T dO, dK += dS^T Q).
// A tile is processed as two halves of 32 queries, software-pipelined so that the exponentials of
// one half run under the matrix instructions of the other:
//   S,dP(half 0);  S,dP(half 1) | P,dS(half 0);  dV,dK(half 0) | P,dS(half 1);  dV,dK(half 1)
// Tiles that need a mask (the diagonal block, a ragged last query block) take a separate
// instantiation of the tile body, so the common path has no per-element selects or branches.
// The column's tiles are visited query block by query block, from the sequence's last query block
// down to the diagonal, all query heads of the KV group at one query block before the next:
// concurrent columns of one KV head (same XCD) start at the same query block, advance at a similar
// pace and so ask for the same Q/dO tiles at about the same time and meet them in that XCD's L2.
template <int D, bool OUT_F32>
__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(1))) void attn_bwd_dkv_kernel(AttnParams P) {
  constexpr int TILE_B = 64 * D * 2;  // bytes of one Q or dO tile
  constexpr int BUF_B = 2 * TILE_B;   // bytes of one buffer (Q tile, dO tile)
  constexpr int ROW_B = D * 2;
  __shared__ __attribute__((aligned(1024))) bf16 tiles[2][2][64 * D];  // [buffer][Q, dO]
  __shared__ __attribute__((aligned(256))) float rowstat[2][2][64];    // [buffer][LSE * log2(e), Dr]
  constexpr int kCW = 16;            // bitmap words (32 query blocks each) handled per chunk
  __shared__ uint32_t bm_s[8][kCW];  // bitmap words of up to 8 selection heads
  __shared__ uint16_t tl_s[kCW * 32 * 8];  // the chunk's tiles in processing order
  __shared__ int ntl_s;
  const ColItem item = P.bwd_items[blockIdx.x];
  if (item.col < 0) return;  // the item lists are padded to their largest possible length
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int64_t col = item.col;  // g * NQB + global block index
  const int wlo = item.wrange & 0xffff, whi = item.wrange >> 16;  // bitmap words of the column this item covers
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

  // LDS byte addresses of this lane's operand reads inside buffer 0 (the buffer and everything else is an
  // offset: rows 16 apart share the swizzle)
  unsigned row_a[D / 16], tr_a[D / 32][2];
  const unsigned stat_a = lds_offset(&rowstat[0][0][0]) + 16 * hf;
  {
    const unsigned tiles0 = lds_offset(&tiles[0][0][0]);
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) row_a[ks] = tiles0 + l32 * ROW_B + 16 * ((2 * ks + hf) ^ chunk_swizzle<D>(l32));
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int r = 8 * half + 4 * hf + ((lane & 15) >> 2), d = 32 * dt + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        tr_a[dt][half] = tiles0 + r * ROW_B + 16 * ((d >> 3) ^ chunk_swizzle<D>(r)) + 2 * (d & 7);
      }
  }
  auto lds16 = [](unsigned a) __attribute__((always_inline)) { return *(const bf16x8 __attribute__((address_space(3)))*)a; };
  auto lds_f4 = [](unsigned a) __attribute__((always_inline)) { return *(const f32x4 __attribute__((address_space(3)))*)a; };
  constexpr int NOP = D / 16;  // operands (and matrix instructions) per pipeline stage
  // A operands of S = Q K^T / dP = dO V^T: rows 32qt + lane%32 of the tile at byte offset `off`, all of d
  auto ld_rows = [&](bf16x8* dst, unsigned off) __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < NOP; ++ks) dst[ks] = lds16(row_a[ks] + off);
  };
  // B operands of dV += P^T dO / dK += dS^T Q for the query steps kk0, kk0+1: contraction slots =
  // queries 16kk + 8(e/4) + 4hf + e%4, column = d (32dt + lane%32), through the transposing read
  auto ld_tr = [&](bf16x8* dst, unsigned off, int kk0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
        const unsigned o = off + (kk0 + q) * 16 * ROW_B;
        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(tr_a[dt][0] + o));
        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(tr_a[dt][1] + o));
        dst[q * (D / 32) + dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
  };

  TileLoader<D> loader;
  loader.init(P.Hq, wave, lane);
  constexpr int kLoadsPerTile = 2 * TileLoader<D>::LPT + 1;  // asynchronous loads one wavefront issues per tile
  auto issue = [&](int buf, int i, int h) __attribute__((always_inline)) {
    const int64_t q0 = seq0 + (int64_t)i * 64;
    const int qv = min(64, L - i * 64);
    loader.issue(tiles[buf][0], P.q, q0, qv, P.Hq, h);
    loader.issue(tiles[buf][1], P.d_o, q0, qv, P.Hq, h);
    // 64 LSE and 64 Dr values: one 4-byte load per lane, wavefront 0 takes LSE and wavefront 1 Dr
    // (rows past the end of the sequence read the +inf stored behind the LSE array: their P becomes 0)
    const float* src = wave == 0 ? (lane < qv ? P.lse2 + (int64_t)h * P.T + q0 + lane : P.lse2 + (int64_t)P.Hq * P.T)
                                 : P.drow + (int64_t)h * P.T + q0 + min(lane, qv - 1);
    dma4(src, lds_offset(rowstat[buf][wave]));
  };

  f32x16 sacc[2], dpacc[2];
  bf16x8 pa[4], dsa[4];
  bf16x8 opA[NOP], opB[NOP];
  // causal mask inside the diagonal tile (raw scores of queries 32qt .. 32qt+31)
  auto mask_diag = [&](int qt) __attribute__((always_inline)) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (kloc > 32 * qt + c_row(v, hf)) sacc[qt][v] = -__builtin_inff();
  };
  // P = exp2(S c - lse2), dS = P (dP - Dr), both to bf16, for registers 4vg .. 4vg+3 = query rows
  // 32qt + 8vg + 4hf + (0..3).  The rows' statistics are fetched from LDS one stage ahead (ld_stat)
  // so that no stage has to wait for them.
  f32x4 st_ls[2], st_dd[2];
  auto ld_stat = [&](int slot, unsigned so, int qt, int vg) __attribute__((always_inline)) {
    st_ls[slot] = lds_f4(stat_a + so + (32 * qt + 8 * vg) * 4);
    st_dd[slot] = lds_f4(stat_a + so + 256 + (32 * qt + 8 * vg) * 4);
  };
  auto pointwise = [&](int slot, int qt, int vg) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int v = 4 * vg + c;
      const float pv = fast_exp2(__builtin_fmaf(sacc[qt][v], P.scale_log2e, -st_ls[slot][c]));
      pa[2 * qt + (v >> 3)][v & 7] = (bf16)pv;
      dsa[2 * qt + (v >> 3)][v & 7] = (bf16)(pv * (dpacc[qt][v] - st_dd[slot][c]));
    }
  };
#define SB_STAGE_FENCE() __builtin_amdgcn_sched_barrier(0)
// scheduling groups for one stage: NOP x (1 matrix instruction, nds LDS reads, nvalu vector ALU instructions)
#define SB_PIPE(nds, nvalu)                                                     \
  _Pragma("unroll") for (int i_ = 0; i_ < NOP; ++i_) {                          \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          \
    if ((nds) > 0) __builtin_amdgcn_sched_group_barrier(0x100, (nds), 0);       \
    if ((nvalu) > 0) __builtin_amdgcn_sched_group_barrier(0x002, (nvalu), 0);   \
  }

  const int words = (n + 31) >> 5;
  const bool per_qhead = P.mode == SB_SELECT_PER_QHEAD;
  const int nsel = per_qhead ? P.G : 1;      // bitmap columns (selection heads) of this KV head
  const int hpe = per_qhead ? 1 : P.G;       // query heads each set bit stands for
  int tt = 0;                                // tiles of the chunk processed so far: tile tt lives in buffer tt & 1
  for (int sel0 = 0; sel0 < nsel; sel0 += 8) {                  // selection heads in groups of 8
    const int ns8 = min(8, nsel - sel0);
    for (int wend = whi, w0; wend > wlo; wend = w0) {  // chunks of up to kCW bitmap words, last first
      w0 = max(wlo, wend - kCW);
      const int wn = wend - w0;
      // ---- the chunk's tile list: entry = (query block - 32 w0) * 8 + head, ordered by query block, then head.
      // The list is walked backwards (last query block first): every column of a sequence then starts at
      // the same query block and, selecting at a similar density, stays close to its neighbours.
      __syncthreads();
      for (int a = tid; a < ns8 * kCW; a += 128) {
        const int sel = a / kCW, w = a % kCW;
        const int hs = per_qhead ? g * P.G + sel0 + sel : g;
        bm_s[sel][w] = w < wn ? P.bitmap[(int64_t)P.Hs * P.bm_off[s] + ((int64_t)hs * n + j) * words + w0 + w] : 0u;
      }
      __syncthreads();
      if (tid < 64) {  // lane w counts the tiles of word w, a wavefront scan turns counts into list positions
        int cnt = 0;
        if (tid < kCW)
          for (int sel = 0; sel < ns8; ++sel) cnt += __builtin_popcount(bm_s[sel][tid]) * hpe;
        int incl = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const int up = __shfl_up(incl, off, 64);
          if (tid >= off) incl += up;
        }
        if (tid == 63) ntl_s = incl;
        int pos = incl - cnt;
        if (tid < kCW && cnt > 0) {
          uint32_t any = 0;
          for (int sel = 0; sel < ns8; ++sel) any |= bm_s[sel][tid];
          while (any) {
            const int b = __builtin_ctz(any);
            any &= any - 1;
            if (per_qhead) {
              for (int sel = 0; sel < ns8; ++sel)
                if ((bm_s[sel][tid] >> b) & 1u) tl_s[pos++] = (uint16_t)((32 * tid + b) * 8 + sel);
            } else {
              for (int hh = 0; hh < hpe; ++hh) tl_s[pos++] = (uint16_t)((32 * tid + b) * 8 + hh);
            }
          }
        }
      }
      __syncthreads();
      const int ntl = __builtin_amdgcn_readfirstlane(ntl_s);
      if (ntl == 0) continue;
      // the diagonal tiles (query block j itself) are the first of the list, i.e. the last to be processed: count them
      int nd = 0;
      if (j >= 32 * w0 && j < 32 * (w0 + wn)) {
        for (int sel = 0; sel < ns8; ++sel) nd += (int)((bm_s[sel][(j >> 5) - w0] >> (j & 31)) & 1u) * hpe;
        nd = __builtin_amdgcn_readfirstlane(nd);
      }
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(kf[ks]), "+v"(vf[ks]));
      auto entry = [&](int t, int& i, int& h) __attribute__((always_inline)) {
        const int e = __builtin_amdgcn_readfirstlane((int)tl_s[ntl - 1 - t]);
        i = 32 * w0 + (e >> 3);
        h = g * P.G + sel0 + (e & 7);
      };
      // ---- prologue: tiles 0 and 1 in flight, the first operands of tile 0 on their way to registers
      tt = 0;  // every chunk starts in buffer 0 (the barrier above has drained the loads and reads of the previous one)
      {
        int i0, h0;
        entry(0, i0, h0);
        issue(tt & 1, i0, h0);
        if (ntl > 1) {
          entry(1, i0, h0);
          issue((tt + 1) & 1, i0, h0);
          wait_vmcnt<kLoadsPerTile>();
        } else {
          wait_vmcnt<0>();
        }
      }
      __builtin_amdgcn_s_barrier();
      ld_rows(opA, 0);
      // ---- one tile per iteration, eight stages of NOP matrix instructions each; the operands of a
      // stage are fetched from LDS while the previous stage computes, and the pointwise work of one half
      // tile is spread under the matrix instructions of the next stages.  The instruction mix of every
      // stage is pinned with scheduling groups: one matrix instruction, then its share of the LDS reads
      // and of the vector arithmetic.
      // BUF = 0 / 1: the tile's buffer is known at compile time and is an immediate offset of every LDS read;
      // BUF = -1: it is tt & 1 and the offsets are added per tile
      auto tile = [&](auto diag_c, auto buf_c, int t) __attribute__((always_inline)) {
          constexpr bool DIAG = decltype(diag_c)::value;
          constexpr int BUF = decltype(buf_c)::value;
          const int buf = BUF >= 0 ? BUF : (tt & 1);
          const unsigned BO = buf * BUF_B, NBO = (1 - buf) * BUF_B, SO = buf * 512;
          const int e2 = t + 2 < ntl ? (int)tl_s[ntl - 3 - t] : 0;
          // stage 0: S(queries 0..31)
          ld_rows(opB, BO + TILE_B);
          sacc[0] = zero16();
#pragma unroll
          for (int ks = 0; ks < NOP; ++ks) sacc[0] = mfma32(opA[ks], kf[ks], sacc[0]);
          SB_PIPE(1, 0);
          SB_STAGE_FENCE();
          // stage 1: dP(queries 0..31)
          ld_rows(opA, BO + 32 * ROW_B);
          ld_stat(0, SO, 0, 0);
          ld_stat(1, SO, 0, 1);
          dpacc[0] = zero16();
#pragma unroll
          for (int ks = 0; ks < NOP; ++ks) dpacc[0] = mfma32(opB[ks], vf[ks], dpacc[0]);
          SB_PIPE(2, 0);
          SB_STAGE_FENCE();
          // stage 2: S(queries 32..63) | first half of the pointwise work of queries 0..31
          if (DIAG) mask_diag(0);
          ld_rows(opB, BO + TILE_B + 32 * ROW_B);
          sacc[1] = zero16();
#pragma unroll
          for (int ks = 0; ks < NOP; ++ks) sacc[1] = mfma32(opA[ks], kf[ks], sacc[1]);
          pointwise(0, 0, 0);
          pointwise(1, 0, 1);
          SB_PIPE(1, 8);
          SB_STAGE_FENCE();
          ld_stat(0, SO, 0, 2);
          ld_stat(1, SO, 0, 3);
          SB_STAGE_FENCE();
          // stage 3: dP(queries 32..63) | second half
          ld_tr(opA, BO + TILE_B, 0);
          dpacc[1] = zero16();
#pragma unroll
          for (int ks = 0; ks < NOP; ++ks) dpacc[1] = mfma32(opB[ks], vf[ks], dpacc[1]);
          pointwise(0, 0, 2);
          pointwise(1, 0, 3);
          SB_PIPE(2, 8);
          SB_STAGE_FENCE();
          ld_stat(0, SO, 1, 0);
          ld_stat(1, SO, 1, 1);
          SB_STAGE_FENCE();
          // stage 4: dV += P^T dO over queries 0..31 | first half of the pointwise work of queries 32..63
          if (DIAG) mask_diag(1);
          ld_tr(opB, BO, 0);
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) dvacc[dt] = mfma32(pa[q], opA[q * (D / 32) + dt], dvacc[dt]);
          pointwise(0, 1, 0);
          pointwise(1, 1, 1);
          SB_PIPE(2, 8);
          SB_STAGE_FENCE();
          ld_stat(0, SO, 1, 2);
          ld_stat(1, SO, 1, 3);
          SB_STAGE_FENCE();
          // stage 5: dK += dS^T Q over queries 0..31 | second half
          ld_tr(opA, BO + TILE_B, 2);
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) dkacc[dt] = mfma32(dsa[q], opB[q * (D / 32) + dt], dkacc[dt]);
          pointwise(0, 1, 2);
          pointwise(1, 1, 3);
          SB_PIPE(2, 8);
          SB_STAGE_FENCE();
          // stage 6: dV over queries 32..63
          ld_tr(opB, BO, 2);
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) dvacc[dt] = mfma32(pa[2 + q], opA[q * (D / 32) + dt], dvacc[dt]);
          SB_PIPE(2, 0);
          SB_STAGE_FENCE();
          // stage 7: dK over queries 32..63.  Its operands are the last LDS reads of this tile: once they
          // have arrived the buffer is free, and once the next tile has landed everywhere (barrier) its
          // first operands can be fetched under this stage's matrix instructions.
          asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_s_barrier();
          if (t + 2 < ntl) {
            const int e = __builtin_amdgcn_readfirstlane(e2);
            issue(buf, 32 * w0 + (e >> 3), g * P.G + sel0 + (e & 7));
          }
          SB_STAGE_FENCE();
          ld_rows(opA, NBO);  // (after the last tile of the chunk this reads a stale buffer and is not used)
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) dkacc[dt] = mfma32(dsa[2 + q], opB[q * (D / 32) + dt], dkacc[dt]);
          SB_PIPE(1, 0);
          SB_STAGE_FENCE();
          ++tt;
      };
      {
        using B0 = std::integral_constant<int, 0>;
        using B1 = std::integral_constant<int, 1>;
        using BR = std::integral_constant<int, -1>;
        const int nn = ntl - nd;  // tiles without a mask: in pairs, the chunk starts in buffer 0
        int t = 0;
        for (; t + 2 <= nn; t += 2) {
          tile(std::false_type(), B0(), t);
          tile(std::false_type(), B1(), t + 1);
        }
        if (t < nn) tile(std::false_type(), B0(), t++);
        for (; t < ntl; ++t) tile(std::true_type(), BR(), t);  // the diagonal tiles
      }

    }
  }
#undef SB_PIPE
#undef SB_STAGE_FENCE
  // C layout: column = d (32dt + l32), register v = key row c_row(v, hf) of this wavefront's strip
  if (item.slot >= 0) {  // a part of a split column: leave the fp32 partial sums for the reduction
    float* part = P.partials + (size_t)item.slot * (2 * 64 * D);
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int kr = wave * 32 + c_row(v, hf);
        part[kr * D + 32 * dt + l32] = dkacc[dt][v];
        part[(64 + kr) * D + 32 * dt + l32] = dvacc[dt][v];
      }
    timer.stop(P);
    return;
  }
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

// dK/dV of the split columns: the parts' fp32 partial sums added in part order (last query blocks first), then the
// scale and the rounding of the unsplit path.  One workgroup per split column.
template <int D, bool OUT_F32>
__global__ __launch_bounds__(256) void attn_bwd_dkv_reduce_kernel(AttnParams P) {
  const int si = blockIdx.x;
  if (si >= P.counters[1]) return;
  const int64_t col = P.split_cols[3 * si];
  const int slot0 = P.split_cols[3 * si + 1], np = P.split_cols[3 * si + 2];
  const int g = (int)(col / P.NQB);
  const int qbj = (int)(col - (int64_t)g * P.NQB);
  const int s = P.qb_seq[qbj];
  const int j = qbj - P.qb_off[s];
  const int64_t seq0 = P.cu[s];
  const int rows = min(64, P.cu[s + 1] - P.cu[s] - j * 64);
  const float* part = P.partials + (size_t)slot0 * (2 * 64 * D);
  for (int e = threadIdx.x; e < rows * D; e += 256) {
    float dk = 0.f, dv = 0.f;
    for (int p = 0; p < np; ++p) {
      dk += part[(size_t)p * (2 * 64 * D) + e];
      dv += part[(size_t)p * (2 * 64 * D) + 64 * D + e];
    }
    const int kr = e / D, d = e % D;
    const int64_t off = ((seq0 + j * 64 + kr) * P.Hkv + g) * D + d;
    if (OUT_F32) {
      ((float*)P.dk)[off] = dk * P.scale;
      ((float*)P.dv)[off] = dv;
    } else {
      ((bf16*)P.dk)[off] = (bf16)(dk * P.scale);
      ((bf16*)P.dv)[off] = (bf16)dv;
    }
  }
}

int convert_f32_to_bf16(const void* src, void* dst, int64_t n, hipStream_t st);

template <int D, bool F32>
static int launch_bwd(const Geo& g, const AttnParams& P, hipStream_t st) {
  // query-major dQ: one workgroup per (item, part of the item's query heads); 2 * KS wavefronts per head
  const int heads = g.mode == SB_SELECT_PER_QHEAD ? 1 : g.G;
  const int parts = (heads + 3) / 4, hpp = (heads + parts - 1) / parts;  // heads per workgroup: 1..4
  dim3 grid((unsigned)ticketed_grid(P.n_items, P.ticket != nullptr), (unsigned)parts);
  KernelTimer kt(K_BWD_DQ, st);
  if (hpp == 1) hipLaunchKernelGGL((attn_bwd_dq_kernel<D, F32, 2, 256>), grid, dim3(256), 0, st, P, heads);
  else if (hpp == 2) hipLaunchKernelGGL((attn_bwd_dq_kernel<D, F32, 2, 512>), grid, dim3(512), 0, st, P, heads);
  else hipLaunchKernelGGL((attn_bwd_dq_kernel<D, F32, 1, 512>), grid, dim3(128 * hpp), 0, st, P, heads);
  SB_LAUNCH_CHECK("attn_bwd_dq_kernel");
  return SB_OK;
}

template <int D, bool F32>
static int launch_dkv(const Geo& g, const AttnParams& P, hipStream_t st) {
  const int64_t extra = split_extra_max(g);
  const int64_t n_items = (int64_t)g.Hkv * (g.NQB + extra);
  if (n_items > 0x7fffffffll) { set_error("too many key-major items for one launch"); return SB_ERR_INVALID_ARG; }
  dim3 grid((unsigned)n_items), block(128);
  KernelTimer kt(K_BWD_DKV, st);
  hipLaunchKernelGGL((attn_bwd_dkv_kernel<D, F32>), grid, block, 0, st, P);
  SB_LAUNCH_CHECK("attn_bwd_dkv_kernel");
  if (extra > 0) {  // at most `extra` columns are split; workgroups beyond the actual count return at once
    hipLaunchKernelGGL((attn_bwd_dkv_reduce_kernel<D, F32>), dim3((unsigned)extra), dim3(256), 0, st, P);
    SB_LAUNCH_CHECK("attn_bwd_dkv_reduce_kernel");
  }
  return SB_OK;
}

}  // namespace sb

using namespace sb;

extern "C" int sb_sparse_attn_bwd(const sb_problem* p, const void* q, const void* k, const void* v, const void* o,
                                  const float* lse, const void* d_o, const int32_t* sel_rowptr, const int32_t* sel_idx,
                                  const void* plan, void* dq, void* dk, void* dv, void* ws, void* stream) {
  Geo gb;
  int rc = make_geo(p, &gb);
  if (rc != SB_OK) return rc;
  if (gb.S == 0 || gb.T == 0 || gb.NQB == 0) return SB_OK;
  const Geo g = tile_geo(gb);  // the kernels work on 64-row tiles; for larger selection blocks the plan holds the tile-level selection
  if (!q || !k || !v || !o || !lse || !d_o || !sel_rowptr || !sel_idx || !plan || !dq || !dk || !dv || !ws) {
    set_error("null argument");
    return SB_ERR_INVALID_ARG;
  }
  hipStream_t st = (hipStream_t)stream;
  PlanOffsets po = plan_offsets(gb);
  WsOffsets wo = bwd_ws_offsets(g);
  const char* pb = (const char*)plan;
  char* wb = (char*)ws;
  Tables t = make_tables(g, p, (void*)(pb + po.tables));
  AttnParams P{};
  const bool f32 = g.dtype == SB_F32;
  if (f32) {
    KernelTimer kt(K_BWD_PREP, st);  // float32 inputs only: the conversions to the kernels' operand type
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
  float* lse2 = (float*)(wb + wo.lse2);
  P.o = (void*)o; P.lse = (float*)lse; P.drow = drow; P.lse2 = lse2; P.dq = dq; P.dk = dk; P.dv = dv;
  P.rowptr = gb.r == 1 ? sel_rowptr : (const int32_t*)(pb + po.t_rowptr);
  P.idx = gb.r == 1 ? sel_idx : (const int32_t*)(pb + po.t_idx);
  P.items = (const WorkItem*)(pb + po.items);
  P.bitmap = (const uint32_t*)(pb + po.bitmap);
  P.bwd_items = (const ColItem*)(pb + po.bwd_items);
  P.split_cols = (const int32_t*)(pb + po.split_cols);
  P.counters = (const int32_t*)(pb + po.counters);
  P.partials = (float*)(wb + wo.partials);
  P.cu = t.cu; P.qb_off = t.qb_off; P.qb_seq = t.qb_seq; P.bm_off = t.bm_off;
  P.NQB = g.NQB; P.T = g.T; P.Hq = g.Hq; P.Hkv = g.Hkv; P.G = g.G; P.Hs = g.Hs; P.mode = g.mode;
  P.scale = g.softmax_scale; P.scale_log2e = g.softmax_scale * 1.4426950408889634f;
  P.out_f32 = f32;
  P.cu_busy = nullptr;
  if (g_instrument & 1) {
    if ((rc = fill_zero(wb + wo.cu_busy, sizeof(uint64_t) * SB_CU_SLOTS, st)) != SB_OK) return rc;
    P.cu_busy = (unsigned long long*)(wb + wo.cu_busy);
  }
  // The query-major launch hands one item in sixteen out by ticket (see claim_item).  The key-major launch does not: its
  // items are few and very unequal, and a heavy one that is held back for the tail lengthens the launch (measured: +23 %
  // on the 32768-token batch, -1 % on the 262144-token one).
  const int heads = g.mode == SB_SELECT_PER_QHEAD ? 1 : g.G;
  const int64_t n_items = (int64_t)g.Hs * g.NQB;
  if (n_items > 0x3fffffffll) { set_error("too many work items for one launch"); return SB_ERR_INVALID_ARG; }
  P.n_items = (int)n_items;
  P.ticket = nullptr;
  AttnParams Pq = P, Pk = P;
  if (use_tickets(n_items) && heads <= kTicketSlots) {
    Pq.ticket = (int*)(wb + wo.ticket);
    if ((rc = fill_zero(Pq.ticket, sizeof(int32_t) * kTicketSlots, st)) != SB_OK) return rc;
  }
  Pq.work = (const int32_t*)(pb + po.work_fwd);
  Pk.work = nullptr;  // the key-major kernel reads bwd_items
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
