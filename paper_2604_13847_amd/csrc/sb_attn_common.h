// Device helpers shared by the forward and backward attention kernels (gfx950, wave64).
//
// MFMA used: v_mfma_f32_32x32x16_bf16.  Operand layout per lane (half = lane/32):
//   A (32 x 16): row = lane%32, the 8 elements are contraction slots (half, 0..7)
//   B (16 x 32): col = lane%32, the 8 elements are contraction slots (half, 0..7)
//   C (32 x 32): col = lane%32, register v is row 8*(v/4) + 4*half + v%4
// A and B only have to agree on which contraction index sits in slot (half, e); the kernels choose
// that mapping freely (see key_of_slot below).
#pragma once

#include "sb_internal.h"

namespace sb {

struct AttnParams {
  const bf16* q; const bf16* k; const bf16* v; const bf16* d_o;
  void* o;            // forward output (bf16 or float per out_f32)
  float* lse;         // [Hq][T]
  const float* drow;  // [Hq][T] rowsum(dO * O)
  void* dq; void* dk; void* dv;
  const int32_t* rowptr; const int32_t* idx; const int32_t* work;
  const uint32_t* bitmap;
  const int32_t* cu; const int32_t* qb_off; const int32_t* qb_seq; const int64_t* bm_off;
  int64_t NQB;
  int T, Hq, Hkv, G, Hs, mode;
  float scale, scale_log2e;
  int out_f32;
  unsigned long long* cu_busy;  // null when instrumentation is off
};

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ inline f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

__device__ inline bf16x8 zero_bf16x8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (bf16)0.f;
  return z;
}

// Row (0..31) of C register v for a lane in half `hf`.
__device__ inline int c_row(int v, int hf) { return 8 * (v >> 2) + 4 * hf + (v & 3); }

// A 64-long contraction axis (keys or queries of one block) is walked in 4 steps of 16; step kk,
// slot (hf, e) holds element 16*kk + 8*(e/4) + 4*hf + e%4, which is exactly the row of C register
// 8*(kk%2)+e of the (kk/2)-th 32x32 tile: a C tile converts to an A/B operand without any shuffle.
// In LDS the transposed tiles keep that element at position 16*kk + 8*hf + e (position_of_quad), so
// the 8 slots of a lane are one 16-byte read.
__device__ inline int position_of_quad(int quad) {  // quad = element/4 (0..15) -> position/4
  return (quad & ~3) | ((quad & 1) << 1) | ((quad >> 1) & 1);
}

__device__ inline uint4 ld16(const void* p) { return *(const uint4*)p; }

// Cooperative copy of a 64 x D bf16 tile (rows `row0..row0+valid-1` of a [T][H][D] tensor, head h;
// rows >= valid are zero) into LDS, row-major with padded row length LD.
template <int D, int LD>
__device__ inline void load_tile_rowmajor(bf16* dst, const bf16* src, int64_t row0, int valid, int H, int h, int tid, int nthr) {
  for (int u = tid; u < 64 * (D / 8); u += nthr) {
    const int r = u / (D / 8), c = u % (D / 8);
    uint4 x = make_uint4(0, 0, 0, 0);
    if (r < valid) x = ld16(src + ((row0 + r) * H + h) * D + 8 * c);
    *(uint4*)(dst + r * LD + 8 * c) = x;
  }
}

// Same tile written transposed: dst[d][position(row)] with row length LDT (>= 64), so that a lane
// reading 8 consecutive elements of a d-row gets its 8 contraction slots.  Optionally also writes
// the row-major copy (dst_rm != nullptr) from the same loads.
template <int D, int LD, int LDT>
__device__ inline void load_tile_transposed(bf16* dst_t, bf16* dst_rm, const bf16* src, int64_t row0, int valid, int H, int h,
                                            int tid, int nthr) {
  for (int u = tid; u < 16 * (D / 8); u += nthr) {
    const int c = u % (D / 8), quad = u / (D / 8);
    uint4 x[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 4 * quad + r;
      x[r] = make_uint4(0, 0, 0, 0);
      if (row < valid) x[r] = ld16(src + ((row0 + row) * H + h) * D + 8 * c);
      if (dst_rm) *(uint4*)(dst_rm + row * LD + 8 * c) = x[r];
    }
    const int pos = 4 * position_of_quad(quad);
    const uint32_t* w0 = (const uint32_t*)&x[0];
    const uint32_t* w1 = (const uint32_t*)&x[1];
    const uint32_t* w2 = (const uint32_t*)&x[2];
    const uint32_t* w3 = (const uint32_t*)&x[3];
#pragma unroll
    for (int dw = 0; dw < 4; ++dw) {  // dword dw holds d = 8c + 2dw (low half) and 8c + 2dw + 1 (high half)
      uint2 lo, hi;
      lo.x = (w0[dw] & 0xffffu) | (w1[dw] << 16);
      lo.y = (w2[dw] & 0xffffu) | (w3[dw] << 16);
      hi.x = (w0[dw] >> 16) | (w1[dw] & 0xffff0000u);
      hi.y = (w2[dw] >> 16) | (w3[dw] & 0xffff0000u);
      *(uint2*)(dst_t + (8 * c + 2 * dw) * LDT + pos) = lo;
      *(uint2*)(dst_t + (8 * c + 2 * dw + 1) * LDT + pos) = hi;
    }
  }
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct BusyTimer {
  long long t0;
  __device__ inline void start(const AttnParams& P) {
    if (P.cu_busy && threadIdx.x == 0) t0 = wall_clock64();
  }
  __device__ inline void stop(const AttnParams& P) {
    if (P.cu_busy && threadIdx.x == 0) atomicAdd(&P.cu_busy[__smid() & (SB_CU_SLOTS - 1)], (unsigned long long)(wall_clock64() - t0));
  }
};

}  // namespace sb
