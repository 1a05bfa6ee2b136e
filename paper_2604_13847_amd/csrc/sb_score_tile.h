// Pieces shared by the score kernel, the selection kernel and the kernel that does both (paper
// section 2.2): the 16 x 16 score tile on the fp32 matrix cores, the order-preserving key of a
// score, and the per-row selection that one wavefront carries out on keys held in LDS.
// Every path that produces a score goes through score_tile16 with the same operands in the same
// order, and every path that selects goes through select_row, so the paths agree bit for bit.
#pragma once

#include "sb_internal.h"

namespace sb {

typedef float f32x4s __attribute__((ext_vector_type(4)));

// One 16 x 16 tile of dot products <pooled query row, pooled key row> on v_mfma_f32_16x16x4_f32.
// Lane (r = lane % 16, kq = lane / 16) supplies, of query row r in a[] and of key row r in b[], the
// elements 16 u + 4 kq + e (u < D/16, e < 4) at position 4 u + e: the four lanes of a row then read
// 64 consecutive bytes with each 16-byte load.  Instruction t = 4 u + e contracts elements
// 16 u + e + {0, 4, 8, 12}.  Result: the lane holds key column lane % 16 of query rows
// 4 * (lane / 16) + v, v = 0..3.
template <int D>
__device__ inline f32x4s score_tile16(const float (&a)[D / 4], const float (&b)[D / 4]) {
  f32x4s acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < D / 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], acc, 0, 0, 0);
  return acc;
}

// this lane's share of a row of D floats (16-byte aligned) into registers
template <int D>
__device__ inline void load_quarter(float (&dst)[D / 4], const float* __restrict__ row, int kq) {
#pragma unroll
  for (int u = 0; u < D / 16; ++u) {
    const float4 v = *(const float4*)(row + 16 * u + 4 * kq);
    dst[4 * u] = v.x; dst[4 * u + 1] = v.y; dst[4 * u + 2] = v.z; dst[4 * u + 3] = v.w;
  }
}
template <int D>
__device__ inline void add_quarter(float (&dst)[D / 4], const float* __restrict__ row, int kq) {
#pragma unroll
  for (int u = 0; u < D / 16; ++u) {
    const float4 v = *(const float4*)(row + 16 * u + 4 * kq);
    dst[4 * u] += v.x; dst[4 * u + 1] += v.y; dst[4 * u + 2] += v.z; dst[4 * u + 3] += v.w;
  }
}

// Total order of the selection as an unsigned key: score descending = key descending; -0 and +0
// share a key; NaN sorts below everything.
__device__ inline uint32_t order_key(float x) {
  if (x != x) return 0u;
  if (x == 0.0f) x = 0.0f;
  uint32_t b = __float_as_uint(x);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// LDS operations of one wavefront are carried out in issue order, so a wavefront that works alone
// on its own LDS region needs no barrier between phases: only the compiler has to keep the order.
__device__ inline void wave_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Closed-form start of row i (sequence budget k) in the selection CSR, relative to the sequence's base.
__device__ inline int64_t sel_rows_before(int i, int k) {
  const int m0 = min(i, k);  // rows i' < i with i'+1 <= k contribute i'+1, the rest contribute k
  return (int64_t)m0 * (m0 + 1) / 2 + (int64_t)(i - m0) * k;
}

// One wavefront chooses the `need` best of keys[0..m) (0 < need < m; ties to the lower index) and
// writes their indices in ascending order to out[0..need), then i to out[need].  keys and hist (256
// bins) are this wavefront's own LDS; the keys must be visible to it on entry.
// The threshold (the need-th largest key, and how many keys equal to it are kept) comes from one of
// two exact searches.  Small budgets: a histogram of the keys' distance from the row's largest key in
// steps of 2^17 (keys of floats are logarithmic, so 255 such bins span the top four octaves whatever
// the scale of the scores), then a ranking of the few keys in the bin that holds the threshold.
// Otherwise, or when the threshold lies outside those bins or its bin holds more than 64 keys: a radix
// select over all 32 bits, 8 bits per pass.
constexpr int kDistShift = 17;

__device__ inline void select_row(const uint32_t* keys, int* hist, int lane, int m, int need, int i, int32_t* __restrict__ out) {
  const unsigned long long lt = (1ull << lane) - 1ull;
  uint32_t thr = 0;
  int remaining = 0;
  bool found_thr = false;
  if (need * 4 <= m) {
    uint32_t kmax = 0;
    for (int j = lane; j < m; j += 64) kmax = max(kmax, keys[j]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off, 64));
#pragma unroll
    for (int a = 0; a < 4; ++a) hist[lane + 64 * a] = 0;
    wave_lds_fence();
    for (int j = lane; j < m; j += 64) {
      const uint32_t d = (kmax - keys[j]) >> kDistShift;
      if (d < 255u) atomicAdd(&hist[d], 1);
    }
    wave_lds_fence();
    // lane L owns bins 4L .. 4L+3 (ascending distance = descending key; bin 255 is never counted)
    int v[4], sum = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) { v[a] = hist[4 * lane + a]; sum += v[a]; }
    int incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off, 64);
      if (lane >= off) incl += t;
    }
    int run = incl - sum, bin = -1, above = 0, cnt = 0;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      if (run < need && need <= run + v[a]) { bin = 4 * lane + a; above = run; cnt = v[a]; }
      run += v[a];
    }
    const unsigned long long found = __builtin_amdgcn_ballot_w64(bin >= 0);  // at most one lane
    if (found) {
      const int src = __builtin_ctzll(found);
      bin = __builtin_amdgcn_readlane(bin, src);
      above = __builtin_amdgcn_readlane(above, src);
      cnt = __builtin_amdgcn_readlane(cnt, src);
      if (cnt <= 64) {
        // the keys of that bin, in index order, one per lane (staged through the histogram's LDS)
        wave_lds_fence();
        uint32_t* cand = (uint32_t*)hist;
        int pos = 0;
        for (int j0 = 0; j0 < m; j0 += 64) {
          const int j = j0 + lane;
          const uint32_t kk = j < m ? keys[j] : 0u;
          const bool is_c = j < m && ((kmax - kk) >> kDistShift) == (uint32_t)bin;
          const unsigned long long bc = __builtin_amdgcn_ballot_w64(is_c);
          if (is_c) cand[pos + __builtin_popcountll(bc & lt)] = kk;
          pos += __builtin_popcountll(bc);
        }
        wave_lds_fence();
        const bool valid = lane < cnt;
        const uint32_t mine = valid ? cand[lane] : 0u;
        int rank = 0;  // candidates ahead of mine in the total order
        for (int c = 0; c < cnt; ++c) {
          const uint32_t kc = (uint32_t)__builtin_amdgcn_readlane((int)mine, c);
          rank += (kc > mine || (kc == mine && c < lane)) ? 1 : 0;
        }
        const int rem = need - above;  // 1 .. cnt: that many of the bin's keys are kept
        const unsigned long long at = __builtin_amdgcn_ballot_w64(valid && rank == rem - 1);  // exactly one lane
        thr = (uint32_t)__shfl((int)mine, __builtin_ctzll(at), 64);
        remaining = rem - __builtin_popcountll(__builtin_amdgcn_ballot_w64(valid && mine > thr));
        found_thr = true;
      }
    }
    wave_lds_fence();  // the histogram is cleared again below
  }
  if (!found_thr) {
    // radix select, 8 bits per pass: the need-th largest key
    uint32_t prefix = 0, mask = 0;
    remaining = need;
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
    thr = prefix;
  }
  // keys > thr are all kept; of the keys == thr the `remaining` lowest indices are kept; output in index order
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

// Pooling of Q and K into the workspace (and kbar_out, if given); qbar/kbar receive the two pooled arrays.
int launch_pool(const Geo& g, const sb_problem* p, const Tables& t, const void* q, const void* k, float* kbar_out, void* ws,
                hipStream_t st, float** qbar, float** kbar);

}  // namespace sb
