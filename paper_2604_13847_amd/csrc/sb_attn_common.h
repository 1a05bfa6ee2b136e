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
  float* drow;        // [Hq][T] rowsum(dO * O): written by the dQ kernel, read by the dK/dV kernel
  float* lse2;        // [Hq][T] lse * log2(e), likewise; entry [Hq*T] is +inf (stands in for rows that do not exist)
  void* dq; void* dk; void* dv;
  const int32_t* rowptr; const int32_t* idx; const int32_t* work;
  const WorkItem* items;  // descriptors of the query-major items, in work order
  const uint32_t* bitmap;
  const ColItem* bwd_items;    // key-major items (whole columns or parts of heavy ones), see ColItem
  const int32_t* split_cols;   // (column, first partial slot, parts) of the split columns; counters[1] of them
  const int32_t* counters;
  float* partials;             // [slot][dK, dV][64][D] fp32 partial sums of the parts of split columns
  const int32_t* cu; const int32_t* qb_off; const int32_t* qb_seq; const int64_t* bm_off;
  int64_t NQB;
  int T, Hq, Hkv, G, Hs, mode;
  float scale, scale_log2e;
  int out_f32;
  unsigned long long* cu_busy;  // null when instrumentation is off
  // Work distribution (see claim_item)
  int* ticket;        // [kTicketSlots] counters, zero at launch; null: every item is taken by position
  int n_items;        // query-major items
};
constexpr int kTicketSlots = 64;    // one counter per head plane of a query-major launch

// Which item does the workgroup at position `pos` of a launch work on?
// Workgroup ids are dealt to the 8 XCDs in turn, so every XCD gets the same number of workgroups whatever its pace, and
// the XCDs do differ by several percent (the L2 hit rate depends on which heads an XCD serves, and the dies themselves
// differ): a launch that ties every item to a position ends when the slowest XCD is through its share.  So one item in
// sixteen (the last 8 of every 128 in list order, a cross-section of the whole list) is held back: the other items are
// tied to the leading positions, in list order and on the XCD they would have had anyway, and the held-back ones form
// the tail of the launch, handed out by ticket to whichever workgroup asks first.  The launch has twice as many tail
// workgroups as tail items: a fast XCD gets through more of them, and those that find the tail empty exit at once.
// Which workgroup computes an item never changes its result.
// Returns the item's index in the list or -1; every thread of the workgroup must call it (it has a barrier).
__device__ inline int claim_item(int pos, int n_items, int* counter) {
  if (!counter) return pos < n_items ? pos : -1;
  const int groups = n_items >> 7, held = groups << 3;  // held-back items: indices 128 q + 120 .. 128 q + 127
  if (pos < n_items - held) return pos < 120 * groups ? (pos / 120 << 7) + pos % 120 : pos + held;
  __shared__ int sh_claim;
  if (threadIdx.x == 0) sh_claim = atomicAdd(counter, 1);
  __syncthreads();
  const int t = sh_claim;
  return t < held ? ((t >> 3) << 7) + 120 + (t & 7) : -1;
}

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


// ---------------------------------------------------------------------------------------------
// Asynchronous tile staging.  A 64 x D bf16 tile lives in LDS unpadded (row r at byte r*2D), with
// the 16-byte chunks of each row permuted by chunk_swizzle(r): chunk c of row r sits at chunk
// c ^ chunk_swizzle(r).  The permutation makes both access patterns of the MFMA operands free of
// bank conflicts: (a) 16 lanes reading the same chunk of 16 consecutive rows, (b) a transposing
// read where 16 lanes cover 4 consecutive rows x 32 bytes.
// Tiles are written by global_load_lds_dwordx4: each lane fetches 16 bytes from its own global
// address and the wavefront's 1 KiB lands at M0 + 16*lane, so no registers are spent on data in
// flight.  The instruction is issued through inline asm on purpose: the waits are placed by hand
// (wait_vmcnt) so that loads stay in flight across the compute on the previous tile.
template <int D>
__device__ inline int chunk_swizzle(int r) {
  // D = 128 (16 chunks, one row = all 64 banks): the two low row bits pick the 64-byte quarter of the
  // row, the next two the chunk inside it.  A transposing read (32 lanes = 4 rows x 64 bytes) then
  // covers 8 distinct 32-byte bank groups and a row-wise read (16 rows, same chunk) 16 distinct chunks.
  if (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  // D = 64 (8 chunks, two rows = all banks): row bit 0 already selects the bank half.
  return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
}

__device__ inline unsigned lds_offset(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) char*)p;
}

__device__ inline void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_base) : "memory", "m0");
}

// 4 bytes per lane: the wavefront's 256 bytes land at lds_base + 4*lane
__device__ inline void dma4(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" : : "v"(gptr), "s"(lds_base) : "memory", "m0");
}

// s_waitcnt vmcnt(N) only (the other counters stay unconstrained).  The memory clobber keeps the
// compiler from moving LDS reads of the awaited tile above the wait.
template <int N>
__device__ inline void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// Per-lane byte offsets (from the tile's first row, head h) of the loads a loader wavefront issues
// for a tile: wavefront w takes the LPT consecutive KiB (LPT * w + a) of the tile, a = 0 .. LPT-1, i.e.
// tile rows (LPT * w + a) * RPI .. +RPI-1.  The offsets depend only on the lane and on the tensor's row
// pitch, so they are computed once per kernel.
template <int D, int NW = 2>  // NW: wavefronts (0 .. NW-1 of the workgroup) that share the loads of a tile
struct TileLoader {
  static constexpr int C = D / 8;      // 16-byte chunks per row
  static constexpr int RPI = 64 / C;   // rows covered by one wavefront-wide load
  static constexpr int LPT = (D / 8) / NW;  // loads per loader wavefront per tile
  static_assert(LPT >= 1 && LPT * NW * RPI == 64, "the loader wavefronts must cover the 64 rows exactly");
  // Consecutive loads of a wavefront land 1 KiB apart in LDS, so up to four of them share one M0 value: the
  // instruction's immediate offset moves both the global and the LDS address, and voff is pre-biased for it.
  static constexpr int GRP = LPT % 4 == 0 ? 4 : (LPT % 2 == 0 ? 2 : 1);
  unsigned voff[LPT];
  int rl, pc;  // row within a load's group of RPI rows, 16-byte chunk of this lane
  int wave;
  __device__ inline void init(int H, int wave_, int lane) {
    wave = wave_;
    rl = lane / C;
    pc = lane % C;
#pragma unroll
    for (int a = 0; a < LPT; ++a) {
      const int r = (LPT * (wave & (NW - 1)) + a) * RPI + rl;
      voff[a] = (unsigned)(r * H * D * 2 + 16 * (pc ^ chunk_swizzle<D>(r))) - 1024u * (a % GRP);
    }
  }
  // Issue the copy of rows row0 .. row0+63 (head h) of `src` into `slot`.  Rows >= valid repeat the
  // last valid row; their data is always masked by the consumer.  Wavefronts 0 .. NW-1 issue LPT loads
  // each, the others none.  Full tiles (the common case) use a scalar base address plus the
  // precomputed lane offsets, so no vector arithmetic is spent per load.
  __device__ inline void issue(bf16* slot, const bf16* src, int64_t row0, int valid, int H, int h) const {
    if (wave >= NW) return;
    const unsigned base = lds_offset(slot) + LPT * (wave & (NW - 1)) * 1024;  // this wavefront's part of the tile
    const char* tile = (const char*)(src + (row0 * H + h) * D);
    if (valid >= 64) {
      const unsigned long long tv = (unsigned long long)tile;  // wave-uniform: move it to scalar registers
      // (readfirstlane returns int: go through unsigned so that the low half is not sign-extended)
      const unsigned t_hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(tv >> 32));
      const unsigned t_lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(tv & 0xffffffffull));
      const unsigned long long ts = ((unsigned long long)t_hi << 32) | (unsigned long long)t_lo;
      // The base is copied by a scalar instruction first: a scalar register written by a vector instruction
      // (readfirstlane) must not be read by a vector-memory instruction within 5 wait states, while scalar reads of
      // it are interlocked.  M0 needs one wait state (s_nop 0) before the load that uses it.
      unsigned long long sbase;
#pragma unroll
      for (int a = 0; a < LPT; a += GRP) {
        if (GRP == 4)
          asm volatile("s_mov_b64 %0, %6\n\ts_mov_b32 m0, %5\n\ts_nop 0\n\t"
                       "global_load_lds_dwordx4 %1, %0\n\t"
                       "global_load_lds_dwordx4 %2, %0 offset:1024\n\t"
                       "global_load_lds_dwordx4 %3, %0 offset:2048\n\t"
                       "global_load_lds_dwordx4 %4, %0 offset:3072"
                       : "=&s"(sbase) : "v"(voff[a]), "v"(voff[a + 1]), "v"(voff[a + 2]), "v"(voff[a + 3]), "s"(base + a * 1024), "s"(ts) : "memory", "m0");
        else if (GRP == 2)
          asm volatile("s_mov_b64 %0, %4\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\t"
                       "global_load_lds_dwordx4 %1, %0\n\t"
                       "global_load_lds_dwordx4 %2, %0 offset:1024"
                       : "=&s"(sbase) : "v"(voff[a]), "v"(voff[a + 1]), "s"(base + a * 1024), "s"(ts) : "memory", "m0");
        else
          asm volatile("s_mov_b64 %0, %3\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                       : "=&s"(sbase) : "v"(voff[a]), "s"(base + a * 1024), "s"(ts) : "memory", "m0");
      }
    } else {
#pragma unroll
      for (int a = 0; a < LPT; ++a) {  // ragged tile (rare): the lane offsets are recomputed instead of being kept in registers
        const int r = (LPT * (wave & (NW - 1)) + a) * RPI + rl;
        dma16(tile + (int64_t)min(r, valid - 1) * H * D * 2 + 16 * (pc ^ chunk_swizzle<D>(r)), base + a * 1024);
      }
    }
  }
};
// One wavefront copies a strip of 32 rows of one head of a [T][H][D] tensor into an LDS slot of its
// own, with the same swizzled layout as above.  `strip` points at the first row's head slice (it is
// wave-uniform), `valid` is the number of rows of the strip that exist (<= 0 when the whole strip
// lies past the end of the sequence): missing rows repeat the sequence's last row, and the consumer
// masks them.
// Full strips (the common case) are issued four loads at a time: the instruction's immediate
// offset moves both the global and the LDS address, so one M0 value serves four consecutive KiB of
// the slot and the per-lane global offsets are pre-biased by the same amount.  A wavefront issues
// one instruction per four clocks at best, so every instruction saved here is time the wavefront
// can spend issuing MFMAs.
template <int D>
struct StripLoader {
  static constexpr int C = D / 8;        // 16-byte chunks per row
  static constexpr int RPI = 64 / C;     // rows covered by one wavefront-wide load
  static constexpr int LPS = 32 / RPI;   // loads per strip
  static_assert(LPS % 4 == 0, "loads are issued in groups of four");
  unsigned voff[LPS];                    // lane offset of load a, minus 1024 * (a % 4)
  int rl, pc;                            // row within a load's group of RPI rows, 16-byte chunk of this lane
  int pitch;                             // bytes between consecutive rows
  __device__ inline void init(int H, int lane) {
    rl = lane / C;
    pc = lane % C;
    pitch = H * D * 2;
#pragma unroll
    for (int a = 0; a < LPS; ++a) {
      const int r = a * RPI + rl;
      // r * pitch >= 1024 * a * H, so the bias never makes the offset negative
      voff[a] = (unsigned)(r * pitch + 16 * (pc ^ chunk_swizzle<D>(r)) - 1024 * (a & 3));
    }
  }
  // all 32 rows exist; `strip` must be wave-uniform
  __device__ inline void issue_full(unsigned slot, const char* strip) const {
    const unsigned long long tv = (unsigned long long)strip;
    // (readfirstlane returns int: go through unsigned so that the low half is not sign-extended)
    const unsigned t_hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(tv >> 32));
    const unsigned t_lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(tv & 0xffffffffull));
    const unsigned long long ts = ((unsigned long long)t_hi << 32) | (unsigned long long)t_lo;
    // The base is copied by a scalar instruction first: a scalar register written by a vector
    // instruction (readfirstlane) must not be read by a vector-memory instruction within 5 wait
    // states, while scalar reads of it are interlocked.  M0 needs one wait state (s_nop 0) before
    // the load that uses it.
#pragma unroll
    for (int a = 0; a < LPS; a += 4) {
      unsigned long long base;
      asm volatile("s_mov_b64 %0, %6\n\ts_mov_b32 m0, %5\n\ts_nop 0\n\t"
                   "global_load_lds_dwordx4 %1, %0\n\t"
                   "global_load_lds_dwordx4 %2, %0 offset:1024\n\t"
                   "global_load_lds_dwordx4 %3, %0 offset:2048\n\t"
                   "global_load_lds_dwordx4 %4, %0 offset:3072"
                   : "=&s"(base) : "v"(voff[a]), "v"(voff[a + 1]), "v"(voff[a + 2]), "v"(voff[a + 3]), "s"(slot + a * 1024), "s"(ts) : "memory", "m0");
    }
  }
  __device__ inline void issue(unsigned slot, const char* strip, int valid) const {
    if (valid >= 32) {
      issue_full(slot, strip);
    } else {
#pragma unroll
      for (int a = 0; a < LPS; ++a) {  // ragged strip (rare): the lane offsets are recomputed instead of being kept in registers
        const int r = a * RPI + rl;
        dma16(strip + (int64_t)min(r, valid - 1) * pitch + 16 * (pc ^ chunk_swizzle<D>(r)), slot + a * 1024);
      }
    }
  }
};
template <int D>
constexpr int loads_per_tile() { return D / 16; }

// 8 consecutive elements (chunk c) of row r
template <int D>
__device__ inline bf16x8 lds_row8(const bf16* slot, int r, int c) {
  return *(const bf16x8*)(slot + r * D + 8 * (c ^ chunk_swizzle<D>(r)));
}

// Transposing read (ds_read_b64_tr_b16): within each group of 16 lanes, lane x supplies the address
// of 4 consecutive elements of row r0 + x/4 starting at column dbase + 4*(x%4), and receives the 4
// elements of column dbase + x from rows r0 .. r0+3.
template <int D>
__device__ inline bf16x4 lds_tr4(const bf16* slot, int r0, int dbase, int lane16) {
  const int r = r0 + (lane16 >> 2), d = dbase + 4 * (lane16 & 3);
  const bf16* p = slot + r * D + 8 * ((d >> 3) ^ chunk_swizzle<D>(r)) + (d & 7);
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)p);
}

// A/B operand whose 8 contraction slots are rows 16*kk + 8*(e/4) + 4*hf + e%4 of the tile and whose
// MFMA row/column is tile column 32*dt + lane%32.
template <int D>
__device__ inline bf16x8 lds_tr_operand(const bf16* slot, int kk, int dt, int lane) {
  const int hf = lane >> 5, lane16 = lane & 15, dbase = 32 * dt + 16 * ((lane >> 4) & 1);
  bf16x4 lo = lds_tr4<D>(slot, 16 * kk + 4 * hf, dbase, lane16);
  bf16x4 hi = lds_tr4<D>(slot, 16 * kk + 8 + 4 * hf, dbase, lane16);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// x * f for an accumulator element that lives in an accumulation register.  Written as one opaque
// block so that the copies to and from the arithmetic registers stay inside the (rarely taken)
// branch that needs them instead of being hoisted into the main loop.
__device__ inline float scale_acc(float x, float f) {
  float tmp;
  asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1" : "+a"(x), "=&v"(tmp) : "v"(f));
  return x;
}

// max(a, b, c) in one instruction.  Written as asm because the compiler's fmax first quiets a possible
// signalling NaN in every operand it has not produced itself (an extra instruction per value read
// back from an accumulator); a NaN operand is simply dropped by the hardware instruction.
__device__ inline float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// acc + p[0] + p[1] in one instruction (fp32 accumulation of two bf16 values)
__device__ inline float sum2(bf16x2 p, float acc) {
  bf16x2 one;
  one[0] = (bf16)1.0f;
  one[1] = (bf16)1.0f;
  return __builtin_amdgcn_fdot2_f32_bf16(p, one, acc, false);
}

// max of x over the two lanes l and l + 32 (both receive it): one lane-half swap, no LDS round trip
__device__ inline float max_across_halves(float x) {
  const unsigned u = __float_as_uint(x);
  // returns {own low half | partner's low half, partner's high half | own high half}: element 0 holds
  // the low half's value in every lane, element 1 the high half's
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
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
