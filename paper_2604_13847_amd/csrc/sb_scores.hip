// Routing scores (paper section 2.2, MoBA indexer): mean-pool the blocks of K and Q, then
// score = score_scale * <pooled Q block i, pooled K block j> for past blocks j < i.
// Both kernels are HBM-bound: K and Q are read once, the score matrix is written once.
#include "sb_internal.h"

namespace sb {

__device__ inline float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Mean over the valid tokens of one block, for 4 adjacent columns per thread.
// grid = (NQB, ceil(H*D / 1024)); X is [T][H*D]; out is [NQB][H*D] float.
template <bool F32>
__global__ __launch_bounds__(256) void pool_kernel(const void* __restrict__ X, int cols, const int32_t* __restrict__ cu,
                                                   const int32_t* __restrict__ qb_off, const int32_t* __restrict__ qb_seq,
                                                   int B, float* __restrict__ out) {
  const int qb = blockIdx.x;
  const int c0 = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (c0 >= cols) return;
  const int s = qb_seq[qb];
  const int j = qb - qb_off[s];
  const int L = cu[s + 1] - cu[s];
  const int first = j * B, last = min((j + 1) * B, L);
  const int64_t row0 = (int64_t)cu[s] + first;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (F32) {
    const float* p = (const float*)X + row0 * cols + c0;
#pragma unroll 8
    for (int r = 0; r < last - first; ++r) {
      float4 v = *(const float4*)(p + (int64_t)r * cols);
      a0 += v.x; a1 += v.y; a2 += v.z; a3 += v.w;
    }
  } else {
    const uint16_t* p = (const uint16_t*)X + row0 * cols + c0;
#pragma unroll 8
    for (int r = 0; r < last - first; ++r) {
      uint2 v = *(const uint2*)(p + (int64_t)r * cols);
      a0 += bf16_bits_to_float(v.x & 0xffffu); a1 += bf16_bits_to_float(v.x >> 16);
      a2 += bf16_bits_to_float(v.y & 0xffffu); a3 += bf16_bits_to_float(v.y >> 16);
    }
  }
  const float inv = 1.0f / (float)(last - first);
  *(float4*)(out + (int64_t)qb * cols + c0) = make_float4(a0 * inv, a1 * inv, a2 * inv, a3 * inv);
}

// One workgroup per (tile of 64 query blocks of one sequence, selection head).  It walks the key
// block tiles (32 key blocks each) up to its own diagonal, computing 64x32 scores per step from
// LDS-staged pooled vectors, and writes -infinity for every j >= i of its rows.
// tile table: grid.x indexes (sequence, i-tile) pairs through a search over it_off (prefix of ceil(n_s/64)).
template <int D>
__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ qbar, const float* __restrict__ kbar,
                                                    const int32_t* __restrict__ cu, const int32_t* __restrict__ qb_off,
                                                    const int64_t* __restrict__ sc_off, int S, int Hq, int Hkv, int Hs,
                                                    int G, int mode, float scale, float* __restrict__ scores) {
  constexpr int LD = D + 4;  // padded row length (floats) of the LDS tiles
  __shared__ float qs[64 * LD];
  __shared__ float ks[32 * LD];
  __shared__ int sh_s, sh_it;
  const int tid = threadIdx.x;
  if (tid == 0) {  // locate (sequence, i-tile) of this workgroup
    int t = blockIdx.x, s = 0;
    for (; s < S; ++s) {
      int nt = (qb_off[s + 1] - qb_off[s] + 63) >> 6;
      if (t < nt) break;
      t -= nt;
    }
    sh_s = s; sh_it = t;
  }
  __syncthreads();
  const int s = sh_s, it = sh_it;
  if (s >= S) return;
  const int hs = blockIdx.y;
  const int n = qb_off[s + 1] - qb_off[s];
  const int64_t qb0 = qb_off[s];
  float* out = scores + (int64_t)Hs * sc_off[s] + (int64_t)hs * n * n;
  const int i0 = it * 64;
  const int rows = min(64, n - i0);
  const int heads = mode == SB_SELECT_PER_QHEAD ? 1 : G;
  const int h0 = mode == SB_SELECT_PER_QHEAD ? hs : hs * G;
  const int g = h0 / G;
  // stage the pooled query tile (summed over the group's heads in per-KV-group mode)
  for (int u = tid; u < 64 * (D / 4); u += 256) {
    int r = u / (D / 4), c = (u % (D / 4)) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r < rows)
      for (int hh = 0; hh < heads; ++hh) {
        float4 v = *(const float4*)(qbar + ((qb0 + i0 + r) * Hq + h0 + hh) * D + c);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    *(float4*)(qs + r * LD + c) = acc;
  }
  const int ti = tid >> 4, tj = tid & 15;  // thread computes rows ti*4..+3, columns tj and tj+16
  const float ninf = -__builtin_inff();
  for (int jt = 0; jt <= 2 * it + 1; ++jt) {
    const int j0 = jt * 32;
    if (j0 >= n) break;
    const int colsv = min(32, n - j0);
    __syncthreads();
    for (int u = tid; u < 32 * (D / 4); u += 256) {
      int r = u / (D / 4), c = (u % (D / 4)) * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < colsv) v = *(const float4*)(kbar + ((qb0 + j0 + r) * Hkv + g) * D + c);
      *(float4*)(ks + r * LD + c) = v;
    }
    __syncthreads();
    float acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) acc[a][b] = 0.f;
#pragma unroll 4
    for (int d = 0; d < D; d += 4) {
      float4 qv[4], kv[2];
#pragma unroll
      for (int a = 0; a < 4; ++a) qv[a] = *(const float4*)(qs + (ti * 4 + a) * LD + d);
#pragma unroll
      for (int b = 0; b < 2; ++b) kv[b] = *(const float4*)(ks + (tj + 16 * b) * LD + d);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          acc[a][b] = fmaf(qv[a].x, kv[b].x, acc[a][b]);
          acc[a][b] = fmaf(qv[a].y, kv[b].y, acc[a][b]);
          acc[a][b] = fmaf(qv[a].z, kv[b].z, acc[a][b]);
          acc[a][b] = fmaf(qv[a].w, kv[b].w, acc[a][b]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      int i = i0 + ti * 4 + a;
      if (i >= n) continue;
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        int j = j0 + tj + 16 * b;
        if (j < n) out[(int64_t)i * n + j] = j < i ? scale * acc[a][b] : ninf;
      }
    }
  }
  // columns right of the own tile are all in the future
  const int jstart = (it + 1) * 64;
  for (int r = 0; r < rows; ++r)
    for (int j = jstart + tid; j < n; j += 256) out[(int64_t)(i0 + r) * n + j] = ninf;
}

}  // namespace sb

using namespace sb;

extern "C" int sb_block_scores(const sb_problem* p, const void* q, const void* k, float* kbar_out, float* scores_out,
                               void* ws, void* stream) {
  Geo g;
  int rc = make_geo(p, &g);
  if (rc != SB_OK) return rc;
  if (g.S == 0 || g.T == 0 || g.NQB == 0) return SB_OK;
  if (!q || !k || !scores_out || !ws) { set_error("null q, k, scores_out or ws"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  rc = launch_geom(g, p, ws, st);
  if (rc != SB_OK) return rc;
  Tables t = make_tables(g, p, ws);
  char* b = (char*)ws + align_up(table_offsets(g).bytes);
  float* qbar = (float*)b;
  float* kbar = (float*)(b + align_up(sizeof(float) * (size_t)g.NQB * g.Hq * g.D));
  const int qcols = g.Hq * g.D, kcols = g.Hkv * g.D;
  dim3 gq((unsigned)g.NQB, (unsigned)((qcols + 1023) / 1024)), gk((unsigned)g.NQB, (unsigned)((kcols + 1023) / 1024));
  {
  KernelTimer kt(K_POOL, st);
  if (g.dtype == SB_F32) {
    hipLaunchKernelGGL(pool_kernel<true>, gq, dim3(256), 0, st, q, qcols, t.cu, t.qb_off, t.qb_seq, g.B, qbar);
    hipLaunchKernelGGL(pool_kernel<true>, gk, dim3(256), 0, st, k, kcols, t.cu, t.qb_off, t.qb_seq, g.B, kbar);
  } else {
    hipLaunchKernelGGL(pool_kernel<false>, gq, dim3(256), 0, st, q, qcols, t.cu, t.qb_off, t.qb_seq, g.B, qbar);
    hipLaunchKernelGGL(pool_kernel<false>, gk, dim3(256), 0, st, k, kcols, t.cu, t.qb_off, t.qb_seq, g.B, kbar);
  }
  }
  SB_LAUNCH_CHECK("pool_kernel");
  if (kbar_out)
    SB_CHECK_HIP(hipMemcpyAsync(kbar_out, kbar, sizeof(float) * (size_t)g.NQB * g.Hkv * g.D, hipMemcpyDeviceToDevice, st));
  // number of (sequence, i-tile) pairs
  int64_t tiles = 0;
  for (int s = 0; s < g.S; ++s) {
    int64_t L = (int64_t)p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
    int64_t n = (L + g.B - 1) / g.B;
    tiles += (n + 63) / 64;
  }
  dim3 gs((unsigned)tiles, (unsigned)g.Hs);
  KernelTimer kt(K_SCORE, st);
  if (g.D == 128)
    hipLaunchKernelGGL(score_kernel<128>, gs, dim3(256), 0, st, qbar, kbar, t.cu, t.qb_off, t.sc_off, g.S, g.Hq, g.Hkv,
                       g.Hs, g.G, g.mode, g.score_scale, scores_out);
  else
    hipLaunchKernelGGL(score_kernel<64>, gs, dim3(256), 0, st, qbar, kbar, t.cu, t.qb_off, t.sc_off, g.S, g.Hq, g.Hkv,
                       g.Hs, g.G, g.mode, g.score_scale, scores_out);
  SB_LAUNCH_CHECK("score_kernel");
  return SB_OK;
}
