// Routing scores (paper section 2.2, MoBA indexer): mean-pool the blocks of K and Q, then
// score = score_scale * <pooled Q block i, pooled K block j> for past blocks j < i.
// Pooling is HBM-bound (K and Q are read once); the score tiles run on the fp32 matrix cores and
// write the score matrix once.
#include "sb_internal.h"
#include "sb_score_tile.h"

namespace sb {

__device__ inline float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Mean over the valid tokens of one block, for 8 (bf16) or 4 (float) adjacent columns per thread: 16-byte loads, eight
// rows in flight per thread.  grid = (NQB, ceil(H*D / (256 * columns per thread))); X is [T][H*D]; out is [NQB][H*D] float.
template <bool F32>
__global__ __launch_bounds__(256) void pool_kernel(const void* __restrict__ X, int cols, const int32_t* __restrict__ cu,
                                                   const int32_t* __restrict__ qb_off, const int32_t* __restrict__ qb_seq,
                                                   int B, float* __restrict__ out) {
  constexpr int CPT = F32 ? 4 : 8;  // columns per thread
  const int qb = blockIdx.x;
  const int c0 = (blockIdx.y * 256 + threadIdx.x) * CPT;
  if (c0 >= cols) return;
  const int s = qb_seq[qb];
  const int j = qb - qb_off[s];
  const int L = cu[s + 1] - cu[s];
  const int first = j * B, last = min((j + 1) * B, L);
  const int64_t row0 = (int64_t)cu[s] + first;
  float a[CPT];
#pragma unroll
  for (int e = 0; e < CPT; ++e) a[e] = 0.f;
  if (F32) {
    const float* p = (const float*)X + row0 * cols + c0;
#pragma unroll 8
    for (int r = 0; r < last - first; ++r) {
      float4 v = *(const float4*)(p + (int64_t)r * cols);
      a[0] += v.x; a[1] += v.y; a[2] += v.z; a[3] += v.w;
    }
  } else {
    const uint16_t* p = (const uint16_t*)X + row0 * cols + c0;
#pragma unroll 8
    for (int r = 0; r < last - first; ++r) {
      const uint4 v = *(const uint4*)(p + (int64_t)r * cols);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        a[2 * e] += bf16_bits_to_float(w[e] & 0xffffu);
        a[2 * e + 1] += bf16_bits_to_float(w[e] >> 16);
      }
    }
  }
  const float inv = 1.0f / (float)(last - first);
  float* o = out + (int64_t)qb * cols + c0;
#pragma unroll
  for (int e = 0; e < CPT; e += 4) *(float4*)(o + e) = make_float4(a[e] * inv, a[e + 1] * inv, a[e + 2] * inv, a[e + 3] * inv);
}

// Score tiles on the fp32 matrix cores (the selection is taken on fp32 scores, so the operands stay
// fp32).  One workgroup per (64 query blocks of one sequence, chunk of up to kScChunk * 64 key
// blocks, selection head): the pooled query tile is staged in LDS once, the pooled key tiles one
// after the other; each of the four wavefronts keeps 16 query rows in registers and computes the
// four 16 x 16 tiles of its rows in every 64 x 64 score tile.  Tiles right of the diagonal are
// -infinity without being computed, and the last chunk of a row tile also fills every column to
// its right with -infinity, so that the whole n x n matrix is defined.  Splitting the columns over
// workgroups keeps the longest workgroup short however long the sequence is.
constexpr int kScChunk = 4;

// workgroups of a sequence with nt row tiles: sum over it < nt of (it / kScChunk + 1)
__host__ __device__ inline int64_t score_items(int64_t nt) {
  const int64_t q = nt / kScChunk, r = nt % kScChunk;
  return kScChunk * q * (q + 1) / 2 + r * (q + 1);
}

template <int D>
__global__ __launch_bounds__(256) void score_kernel(const float* __restrict__ qbar, const float* __restrict__ kbar,
                                                    const int32_t* __restrict__ qb_off, const int64_t* __restrict__ sc_off,
                                                    int S, int Hq, int Hkv, int Hs, int G, int mode, float scale,
                                                    float* __restrict__ scores) {
  constexpr int LD = D + 4;  // padded row length (floats) of the LDS tiles
  __shared__ float qs[64 * LD];
  __shared__ float ks[64 * LD];
  __shared__ int sh_s, sh_it, sh_jc;
  const int tid = threadIdx.x;
  if (tid == 0) {  // locate (sequence, row tile, column chunk) of this workgroup
    int64_t x = blockIdx.x;
    int s = 0, it = 0;
    for (; s < S; ++s) {
      const int64_t c = score_items((qb_off[s + 1] - qb_off[s] + 63) >> 6);
      if (x < c) break;
      x -= c;
    }
    if (s < S)
      for (;; ++it) {
        const int c = it / kScChunk + 1;
        if (x < c) break;
        x -= c;
      }
    sh_s = s; sh_it = it; sh_jc = (int)x;
  }
  __syncthreads();
  const int s = sh_s, it = sh_it, jc = sh_jc;
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
    const int r = u / (D / 4), c = (u % (D / 4)) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r < rows)
      for (int hh = 0; hh < heads; ++hh) {
        const float4 v = *(const float4*)(qbar + ((qb0 + i0 + r) * Hq + h0 + hh) * D + c);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    *(float4*)(qs + r * LD + c) = acc;
  }
  const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, kq = lane >> 4;
  const float ninf = -__builtin_inff();
  float a[D / 4];  // this lane's quarter of query row 16 * wave + l16 (filled once the tile is staged)
  bool have_a = false;
  // A key tile is fetched into registers one tile ahead (its loads are in flight while the tile before it is being
  // multiplied) and written to LDS between the two barriers.
  constexpr int PF = 64 * (D / 4) / 256;  // float4 per thread and key tile
  float4 pf[PF];
  auto fetch = [&](int jt) __attribute__((always_inline)) {
    const int j0 = jt * 64, colsv = min(64, n - j0);
#pragma unroll
    for (int x = 0; x < PF; ++x) {
      const int u = tid + 256 * x, r = u / (D / 4), cc = (u % (D / 4)) * 4;
      pf[x] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (r < colsv) pf[x] = *(const float4*)(kbar + ((qb0 + j0 + r) * Hkv + g) * D + cc);
    }
  };
  auto computed = [&](int jt) { return jt * 64 < n && jt <= it; };  // key tiles that are multiplied (a prefix of the chunk)
  if (computed(jc * kScChunk)) fetch(jc * kScChunk);
  for (int c = 0; c < kScChunk; ++c) {
    const int jt = jc * kScChunk + c, j0 = jt * 64;
    if (j0 >= n) break;
    if (jt > it) {  // entirely in the future of these rows
      for (int u = tid; u < rows * 64; u += 256) {
        const int r = u >> 6, j = j0 + (u & 63);
        if (j < n) out[(int64_t)(i0 + r) * n + j] = ninf;
      }
      continue;
    }
    __syncthreads();  // the previous key tile has been consumed (and, the first time, the query tile is staged)
    if (!have_a) {
      load_quarter<D>(a, qs + (16 * wave + l16) * LD, kq);
      have_a = true;
    }
#pragma unroll
    for (int x = 0; x < PF; ++x) {
      const int u = tid + 256 * x, r = u / (D / 4), cc = (u % (D / 4)) * 4;
      *(float4*)(ks + r * LD + cc) = pf[x];
    }
    if (c + 1 < kScChunk && computed(jt + 1)) fetch(jt + 1);
    __syncthreads();
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) {
      const int j = j0 + 16 * c4 + l16;
      const bool future = j0 + 16 * c4 > i0 + 16 * wave + 15;  // the whole 16 x 16 tile lies right of the diagonal
      f32x4s acc = {0.f, 0.f, 0.f, 0.f};
      if (!future) {
        float b[D / 4];
        load_quarter<D>(b, ks + (16 * c4 + l16) * LD, kq);
        acc = score_tile16<D>(a, b);
      }
      if (j < n) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int i = i0 + 16 * wave + 4 * kq + v;
          if (i < n) out[(int64_t)i * n + j] = j < i ? scale * acc[v] : ninf;
        }
      }
    }
  }
  if (jc == it / kScChunk) {  // last chunk of this row tile: every column to its right is in the future
    const int jstart = (jc + 1) * kScChunk * 64;
    for (int r = 0; r < rows; ++r)
      for (int j = jstart + tid; j < n; j += 256) out[(int64_t)(i0 + r) * n + j] = ninf;
  }
}

// Mean-pools Q and K into the workspace behind the geometry tables.
int launch_pool(const Geo& g, const sb_problem* p, const Tables& t, const void* q, const void* k, float* kbar_out, void* ws,
                hipStream_t st, float** qbar_p, float** kbar_p) {
  (void)p;
  char* b = (char*)ws + align_up(table_offsets(g).bytes);
  float* qbar = (float*)b;
  float* kbar = (float*)(b + align_up(sizeof(float) * (size_t)g.NQB * g.Hq * g.D));
  const int qcols = g.Hq * g.D, kcols = g.Hkv * g.D;
  const int per_wg = 256 * (g.dtype == SB_F32 ? 4 : 8);  // columns per workgroup (head_dim is a multiple of 8)
  dim3 gq((unsigned)g.NQB, (unsigned)((qcols + per_wg - 1) / per_wg)), gk((unsigned)g.NQB, (unsigned)((kcols + per_wg - 1) / per_wg));
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
  *qbar_p = qbar;
  *kbar_p = kbar;
  return SB_OK;
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
  float *qbar = nullptr, *kbar = nullptr;
  if ((rc = launch_pool(g, p, t, q, k, kbar_out, ws, st, &qbar, &kbar)) != SB_OK) return rc;
  int64_t items = 0;  // (sequence, row tile, column chunk) triples
  for (int s = 0; s < g.S; ++s) {
    const int64_t L = (int64_t)p->cu_seqlens_host[s + 1] - p->cu_seqlens_host[s];
    const int64_t n = (L + g.B - 1) / g.B;
    items += score_items((n + 63) / 64);
  }
  if (items > 0x7fffffffll) { set_error("too many score tiles for one launch"); return SB_ERR_INVALID_ARG; }
  dim3 gs((unsigned)items, (unsigned)g.Hs);
  KernelTimer kt(K_SCORE, st);
  if (g.D == 128)
    hipLaunchKernelGGL(score_kernel<128>, gs, dim3(256), 0, st, qbar, kbar, t.qb_off, t.sc_off, g.S, g.Hq, g.Hkv, g.Hs, g.G,
                       g.mode, g.score_scale, scores_out);
  else
    hipLaunchKernelGGL(score_kernel<64>, gs, dim3(256), 0, st, qbar, kbar, t.qb_off, t.sc_off, g.S, g.Hq, g.Hkv, g.Hs, g.G,
                       g.mode, g.score_scale, scores_out);
  SB_LAUNCH_CHECK("score_kernel");
  return SB_OK;
}
