// Block-sparse attention forward (paper Eq. 2) on bf16 MFMA with fp32 online softmax.
//
// One workgroup of two wavefronts per work item (sequence s, query head, query block i), taken from
// the longest-first work list.  The two wavefronts split every selected key block by KEYS: wavefront
// w owns keys 32w .. 32w+31 of each block and all 64 query rows, and runs an online softmax of its
// own over its half of the keys (running max, running sum and an unnormalised O per wavefront); the
// two partial results are merged once, at the end, through LDS.  Because a wavefront only ever
// touches its own key strips, it stages them itself (asynchronous global->LDS loads into a private
// ring of strips K0 V0 K1 V1 ..., three strips ahead) and the main loop has no barrier at all.
// Each K / V^T operand read from LDS feeds two MFMAs (one per 32-query half), which halves the LDS
// traffic per flop compared with a split by query rows.
// S^T = K Q^T puts a query in a C-matrix column, so the softmax statistics are per lane and the
// probabilities convert to the B operand of O^T += V^T P^T without any cross-lane movement; V^T is
// read straight out of the row-major V strip with the transposing LDS read.
#include <type_traits>

#include "sb_attn_common.h"

namespace sb {

template <int D, bool OUT_F32>
__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(1))) void attn_fwd_kernel(AttnParams P, int n_items, int heads) {
  constexpr int NS = 4;          // strips in a wavefront's ring
  constexpr int SLOT = 32 * D;   // elements per strip
  constexpr int LPS = StripLoader<D>::LPS;
  constexpr float kLazy = 8.0f;  // see the softmax below
  __shared__ __attribute__((aligned(1024))) bf16 ring[2][NS][SLOT];
  static_assert(sizeof(bf16) * NS * SLOT >= (16 * (D / 32) + 2) * 64 * sizeof(float), "merge buffer must fit in a ring");
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  // Workgroup id -> (position in the work list, query head of the group).  In per-KV-group mode the
  // `heads` query heads of an item take ids that are 8 apart, so they run on the same XCD (ids are
  // dealt round-robin to the 8 XCDs) and share its L2 for the K/V strips.
  int pos = (int)(blockIdx.x / (8u * heads)) * 8 + (int)(blockIdx.x & 7u);
  const int hh = (int)(blockIdx.x >> 3) % heads;
  pos = claim_item(pos, n_items, P.ticket ? P.ticket + hh : nullptr);
  if (pos < 0) return;
  const WorkItem item = P.items[pos];
  const int hs = item.hs, i = item.i, L = item.len, e0 = item.e0, ntiles = item.ntiles;
  const int64_t seq0 = item.seq0;
  const int h = P.mode == SB_SELECT_PER_QHEAD ? hs : hs * P.G + hh;
  const int g = P.mode == SB_SELECT_PER_QHEAD ? hs / P.G : hs;

  // query fragments of both 32-row halves: qf[b][ks] = Q[32b + lane%32][16ks + 8*(lane/32) .. +7]
  bf16x8 qf[2][D / 16];
  bool qvalid[2];
  int64_t tq[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int qloc = 32 * b + l32;
    qvalid[b] = i * 64 + qloc < L;
    tq[b] = seq0 + i * 64 + qloc;
    const bf16* qp = P.q + (tq[b] * P.Hq + h) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qf[b][ks] = qvalid[b] ? *(const bf16x8*)(qp + 16 * ks) : zero_bf16x8();
  }
  // The row's block indices live in one register across the wavefront (lane a holds entry jb0 + a),
  // refilled every ~64 tiles; a refill waits for all loads in flight, which is rare enough.  Requests
  // run at most two entries behind the newest one, so the window keeps two entries of slack.
  int jb0 = 0;
  int jreg = lane < ntiles ? P.idx[e0 + lane] : 0;
  auto refill = [&](int first) __attribute__((always_inline)) {
    jb0 = first;
    jreg = jb0 + lane < ntiles ? P.idx[e0 + jb0 + lane] : 0;
    // wait here, inside the caller's branch: otherwise the compiler puts a full wait at the join after
    // it, which would drain the strip loads in flight every time
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  };
  auto block_of = [&](int x) __attribute__((always_inline)) {
    if (x - jb0 >= 64) refill(x - 2);
    return __builtin_amdgcn_readlane(jreg, x - jb0);
  };
  // The wavefront's strips (rows 32*wave .. +31 of a selected block's K or V) are loaded in the order
  // in which the pipelined loop below consumes them:
  //   c = 0: K_0;   c = 2i+1: K_{i+1};   c = 2i+2: V_i;   c = 2*ntiles-1 (the last): V_{ntiles-1}
  // Strip c lives in ring slot c % NS and is issued as soon as strip c - NS has been read.
  StripLoader<D> loader;
  loader.init(P.Hkv, lane);
  const int nstrips = 2 * ntiles;
  const char* const k0 = (const char*)(P.k + ((seq0 + 32 * wave) * P.Hkv + g) * D);  // this wavefront's strip of block 0
  const char* const v0 = (const char*)(P.v + ((seq0 + 32 * wave) * P.Hkv + g) * D);
  const unsigned block_pitch = 64u * (unsigned)P.Hkv * D * 2;  // bytes from one key block to the next
  const unsigned ring0 = lds_offset(&ring[wave][0][0]);
  const int Lw = L - 32 * wave;  // rows of the sequence from this wavefront's strip of block 0 on
  auto issue_strip = [&](int slot, bool is_v, int tile) __attribute__((always_inline)) {
    const int j = block_of(tile);
    loader.issue(ring0 + slot * (SLOT * 2), (is_v ? v0 : k0) + (unsigned long long)(unsigned)j * block_pitch, Lw - j * 64);
  };
  int issued = -1;  // newest strip issued so far
  auto try_issue = [&](int c) __attribute__((always_inline)) {
    if (c >= nstrips) return;
    const bool is_v = c == nstrips - 1 || (c != 0 && (c & 1) == 0);
    const int tile = c == 0 ? 0 : c == nstrips - 1 ? ntiles - 1 : (c & 1) ? (c + 1) >> 1 : (c >> 1) - 1;
    issue_strip(c % NS, is_v, tile);
    issued = c;
  };
  // waits until strip c has landed (loads complete in order, so the newer ones may stay in flight)
  auto wait_strip = [&](int c) __attribute__((always_inline)) {
    const int younger = issued - c;
    if (younger >= 3) wait_vmcnt<3 * LPS>();
    else if (younger == 2) wait_vmcnt<2 * LPS>();
    else if (younger == 1) wait_vmcnt<LPS>();
    else wait_vmcnt<0>();
  };
  // LDS addresses of this lane's operand reads within slot 0 of the wavefront's ring; the slot is a
  // compile-time offset wherever the loop is unrolled
  unsigned k_addr[D / 16], v_addr[D / 32][2];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) k_addr[ks] = ring0 + l32 * (D * 2) + 16 * ((2 * ks + hf) ^ chunk_swizzle<D>(l32));
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int r = 8 * half + 4 * hf + ((lane & 15) >> 2), d = 32 * dt + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      v_addr[dt][half] = ring0 + r * (D * 2) + 16 * ((d >> 3) ^ chunk_swizzle<D>(r)) + 2 * (d & 7);
    }
  bf16x8 ka[D / 16], va[D / 32][2];
  auto read_k = [&](int slot) __attribute__((always_inline)) {  // operands of S^T = K Q^T: K rows of this wavefront, all of d
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) ka[ks] = *(const bf16x8 __attribute__((address_space(3)))*)(k_addr[ks] + slot * (SLOT * 2));
  };
  // operands of O^T += V^T P^T through the transposing read: contraction slots of step kk are the
  // keys 16kk + 8*(e/4) + 4*(lane/32) + e%4 (rows 16 apart share the swizzle, so kk is a plain offset)
  auto read_v = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(v_addr[dt][0] + slot * (SLOT * 2) + kk * 16 * (D * 2)));
        bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(v_addr[dt][1] + slot * (SLOT * 2) + kk * 16 * (D * 2)));
        va[dt][kk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
  };
  // the query fragments and indices must have landed before the strip loads start: from here on the
  // only vector-memory operations in flight are strip loads, which the loop waits for by count
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(qf[b][ks]));
  asm volatile("" : "+v"(jreg));

  f32x16 oacc[D / 32][2];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) oacc[dt][0] = oacc[dt][1] = zero16();
  float m[2] = {-__builtin_inff(), -__builtin_inff()}, l[2] = {0.f, 0.f};
  f32x16 sa[2][2];  // raw scores of the current and the next tile (ping-pong)
  bf16x8 pb[2][2];
  float alpha[2];

  auto scores = [&](f32x16* dst) __attribute__((always_inline)) {  // dst = K Q^T for the strip whose operands are in ka
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      dst[b] = zero16();
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) dst[b] = mfma32(ka[ks], qf[b][ks], dst[b]);
    }
  };
  // online softmax on raw scores sc: p = exp2(scale*log2e * (s - m)) -> pb, running sums updated
  auto softmax = [&](const f32x16* sc) __attribute__((always_inline)) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      float mx = max3(sc[b][0], sc[b][1], sc[b][2]);
#pragma unroll
      for (int v = 3; v < 15; v += 2) mx = max3(mx, sc[b][v], sc[b][v + 1]);
      mx = max_across_halves(fmaxf(mx, sc[b][15]));
      // Lazy running maximum: the reference m[b] used in the exponent follows the true maximum only
      // when that has grown by more than kLazy (in log2 units), so p stays below 2^kLazy and the
      // accumulated O needs rescaling only then.  The result is the same up to rounding (O and the
      // row sum carry the same factor), and the rescale branch becomes rare instead of the rule.
      const bool first = m[b] == -__builtin_inff();  // nothing accumulated yet for this query: nothing to rescale
      const bool move = first | ((mx - m[b]) * P.scale_log2e > kLazy);
      const float m_new = move ? fmaxf(m[b], mx) : m[b];
      // a wavefront may have seen no unmasked key yet for a query (its strip of the diagonal block can
      // be entirely above the diagonal): keep the exponent finite then
      const float m_use = m_new == -__builtin_inff() ? 0.f : m_new;
      alpha[b] = first ? 1.0f : fast_exp2((m[b] - m_use) * P.scale_log2e);
      const float neg_m = -m_use * P.scale_log2e;
#pragma unroll
      for (int v = 0; v < 16; ++v) pb[b][v >> 3][v & 7] = (bf16)fast_exp2(__builtin_fmaf(sc[b][v], P.scale_log2e, neg_m));
      // the row sum adds up the probabilities as rounded to bf16, i.e. exactly the weights the
      // accumulation below applies, two per instruction
      float rs = l[b] * alpha[b];
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
      {
        const bf16x8 x = pb[b][kk];
        rs = sum2(__builtin_shufflevector(x, x, 0, 1), rs);
        rs = sum2(__builtin_shufflevector(x, x, 2, 3), rs);
        rs = sum2(__builtin_shufflevector(x, x, 4, 5), rs);
        rs = sum2(__builtin_shufflevector(x, x, 6, 7), rs);
      }
      l[b] = rs;
      m[b] = m_new;
    }
  };
  auto rescale = [&]() __attribute__((always_inline)) {
    if (__builtin_amdgcn_ballot_w64((alpha[0] != 1.0f) | (alpha[1] != 1.0f)) != 0) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[dt][b][v] = scale_acc(oacc[dt][b][v], alpha[b]);
    }
  };
  auto accumulate = [&]() __attribute__((always_inline)) {  // O^T += V^T P^T with the operands in va and pb
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int b = 0; b < 2; ++b) oacc[dt][b] = mfma32(va[dt][kk], pb[b][kk], oacc[dt][b]);
  };

  // ---- prologue: S_0, and the K operands of tile 1
#pragma unroll
  for (int c = 0; c < NS; ++c) try_issue(c);
  wait_strip(0);
  read_k(0);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  try_issue(NS);
  scores(sa[0]);
  if (ntiles > 1) {
    wait_strip(1);
    read_k(1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    try_issue(NS + 1);
  }
  // ---- steady state: step t turns S_t into P_t while the MFMAs of S_{t+1} run, then accumulates
  // P_t V_t while the operands of S_{t+2} are fetched.  The loop is unrolled by two so that ring
  // slots and the score ping-pong are compile-time; steps far enough from the end of the row
  // (STEADY) know how many loads are in flight and that every strip they prefetch exists.
  auto step = [&](auto par_c, auto steady_c, int t) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_c)::value;  // t % 2
    constexpr bool STEADY = decltype(steady_c)::value;
    constexpr int SV = (2 * PAR + 2) % NS, SK = (2 * PAR + 3) % NS;  // slots of strips 2t+2 (V_t) and 2t+3 (K_{t+2})
    if (STEADY) wait_vmcnt<3 * LPS>(); else wait_strip(2 * t + 2);
    read_v(SV);
    scores(sa[PAR ^ 1]);
    softmax(sa[PAR]);
    // The probabilities of the first 16 keys are pinned above the rescale branch so that their
    // exponentials overlap the score MFMAs; those of the other 16 may sink below it and overlap the
    // first half of the accumulation MFMAs.
    asm volatile("" : "+v"(pb[0][0]), "+v"(pb[1][0]));
    rescale();
    if (STEADY) {
      wait_vmcnt<2 * LPS>();
      read_k(SK);
    } else if (t + 2 < ntiles) {
      wait_strip(2 * t + 3);
      read_k(SK);
    }
    __builtin_amdgcn_sched_barrier(0x47F);  // the LDS reads stay above the MFMAs: they must be done before their slot is refilled below
    accumulate();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the slots about to be refilled have been read
    if (STEADY) {  // tiles t+2 and t+4 are not the row's last, so their blocks are complete; the window holds them
      loader.issue_full(ring0 + SV * (SLOT * 2), v0 + (unsigned long long)(unsigned)__builtin_amdgcn_readlane(jreg, t + 2 - jb0) * block_pitch);
      loader.issue_full(ring0 + SK * (SLOT * 2), k0 + (unsigned long long)(unsigned)__builtin_amdgcn_readlane(jreg, t + 4 - jb0) * block_pitch);
      issued = 2 * t + 3 + NS;
    } else {
      try_issue(2 * t + 2 + NS);
      try_issue(2 * t + 3 + NS);
    }
  };
  using std::integral_constant;
  int t = 0;
  for (; t + 6 < ntiles; t += 2) {  // both steps prefetch tiles <= t + 5, none of them the row's last (the only one that can be ragged)
    if (t + 5 - jb0 >= 64) refill(t + 2);
    step(integral_constant<int, 0>(), integral_constant<bool, true>(), t);
    step(integral_constant<int, 1>(), integral_constant<bool, true>(), t + 1);
  }
  for (; t + 1 < ntiles; t += 2) {
    step(integral_constant<int, 0>(), integral_constant<bool, false>(), t);
    if (t + 2 < ntiles) step(integral_constant<int, 1>(), integral_constant<bool, false>(), t + 1);
  }
  // ---- last tile: the diagonal block, causal mask inside it
  if ((ntiles - 1) & 1) {
    sa[0][0] = sa[1][0];
    sa[0][1] = sa[1][1];
  }
  wait_strip(nstrips - 1);
  read_v((nstrips - 1) % NS);
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (32 * wave + c_row(v, hf) > 32 * b + l32) sa[0][b][v] = -__builtin_inff();
  softmax(sa[0]);
  rescale();
  accumulate();

  // ---- merge the two key halves: wavefront w finalises query half w and hands the other half over
  l[0] += __shfl_xor(l[0], 32, 64);
  l[1] += __shfl_xor(l[1], 32, 64);
  float* xbuf = (float*)&ring[wave][0][0];            // this wavefront's outgoing partial, [register][lane]
  const float* ybuf = (const float*)&ring[wave ^ 1][0][0];  // the partner's
  constexpr int NR = 16 * (D / 32);
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    if (b != wave) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) xbuf[(16 * dt + v) * 64 + lane] = oacc[dt][b][v];
      xbuf[NR * 64 + lane] = m[b];
      xbuf[(NR + 1) * 64 + lane] = l[b];
    }
  }
  __syncthreads();
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    if (b == wave) {
      const float m2 = ybuf[NR * 64 + lane], l2 = ybuf[(NR + 1) * 64 + lane];
      const float mt = fmaxf(m[b], m2);  // finite for every existing query: its own key is never masked
      const float w1 = fast_exp2((m[b] - mt) * P.scale_log2e), w2 = fast_exp2((m2 - mt) * P.scale_log2e);
      const float lt = l[b] * w1 + l2 * w2;
      const float inv = 1.0f / lt;
      const float c1 = w1 * inv, c2 = w2 * inv;
      if (qvalid[b]) {
        const int64_t obase = (tq[b] * P.Hq + h) * D;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int vg = 0; vg < 4; ++vg) {
            const int d0 = 32 * dt + 8 * vg + 4 * hf;
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = oacc[dt][b][4 * vg + e] * c1 + ybuf[(16 * dt + 4 * vg + e) * 64 + lane] * c2;
            if (OUT_F32) {
              *(float4*)((float*)P.o + obase + d0) = make_float4(x[0], x[1], x[2], x[3]);
            } else {
              bf16x4 y;
              y[0] = (bf16)x[0]; y[1] = (bf16)x[1]; y[2] = (bf16)x[2]; y[3] = (bf16)x[3];
              *(bf16x4*)((bf16*)P.o + obase + d0) = y;
            }
          }
        if (hf == 0) P.lse[(int64_t)h * P.T + tq[b]] = (mt * P.scale_log2e + __builtin_log2f(lt)) * 0.69314718055994531f;
      }
    }
  }
  timer.stop(P);
}

// ---------------------------------------------------------------------------------------------
// Forward kernel for per-KV-group selection: the query heads of a KV group share a work item, so one
// workgroup takes 3 or 4 of them and they share the item's K/V tiles in LDS (whole tiles,
// double-buffered by asynchronous loads) instead of fetching them once per head.  Two wavefronts per
// query head; a wavefront owns 32 query rows and all 64 keys of every selected tile, as two 32-key
// halves with one online-softmax step each.  The register budget (256) lets two wavefronts share a
// SIMD, so one runs its exponentials while the other runs matrix instructions; one operand set
// rotates through both contractions (K rows, then V^T through the transposing read, each register
// refilled right after the MFMA that consumed it).
template <int D, bool OUT_F32>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2))) void attn_fwd_group_kernel(AttnParams P, int heads) {
  constexpr int TILE_B = 64 * D * 2, ROW_B = D * 2, NOP = D / 16;
  constexpr float kLazy = 8.0f;
  __shared__ __attribute__((aligned(1024))) bf16 tiles[2][2][64 * D];  // [buffer][K, V]
  constexpr int kJ = 256;
  __shared__ int jbuf[kJ];
  BusyTimer timer;
  timer.start(P);
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
  const int pos = claim_item(blockIdx.x, P.n_items, P.ticket ? P.ticket + blockIdx.y : nullptr);
  if (pos < 0) return;
  const WorkItem item = P.items[pos];
  const int hs = item.hs, i = item.i, L = item.len, e0 = item.e0, ntiles = item.ntiles;
  const int64_t seq0 = item.seq0;
  const int strip = wave & 1;
  const int hh = blockIdx.y * (nthr / 128) + (wave >> 1);  // query head of the group this wavefront works for
  const bool head_ok = hh < heads;
  const int h = hs * P.G + (head_ok ? hh : 0);  // per-KV-group mode: the item's selection head is the KV head
  const int g = hs;
  const int qloc = strip * 32 + l32;
  const bool qvalid = head_ok && i * 64 + qloc < L;
  const int64_t tq = seq0 + i * 64 + qloc;

  auto stage_indices = [&](int t0) {
    __syncthreads();
    for (int a = tid; a < kJ; a += nthr) jbuf[a] = t0 + a < ntiles ? P.idx[e0 + t0 + a] : 0;
    __syncthreads();
  };
  TileLoader<D, 4> loader;  // a workgroup has six or eight wavefronts: the first four share the tile loads
  loader.init(P.Hkv, wave, lane);
  auto issue = [&](int t) {
    const int j = __builtin_amdgcn_readfirstlane(jbuf[t % kJ]);
    const int64_t kv0 = seq0 + (int64_t)j * 64;
    const int kvalid = min(64, L - j * 64);
    loader.issue(tiles[t & 1][0], P.k, kv0, kvalid, P.Hkv, g);
    loader.issue(tiles[t & 1][1], P.v, kv0, kvalid, P.Hkv, g);
  };

  // B operand of S^T = K Q^T: column = query lane%32 of the strip, slots = d 16ks + 8hf + (0..7)
  bf16x8 qf[NOP];
  {
    const bf16* qp = P.q + (tq * P.Hq + h) * D + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < NOP; ++ks) qf[ks] = qvalid ? *(const bf16x8*)(qp + 16 * ks) : zero_bf16x8();
  }
  stage_indices(0);
  // everything loaded so far must have landed before the tile loads start: from here on the only
  // vector-memory operations in flight are tile loads, which the loop waits for by count
#pragma unroll
  for (int ks = 0; ks < NOP; ++ks) asm volatile("" : "+v"(qf[ks]));
  issue(0);

  const unsigned tiles0 = lds_offset(&tiles[0][0][0]);
  unsigned row_a[NOP], tr_a[D / 32][2];
#pragma unroll
  for (int ks = 0; ks < NOP; ++ks) row_a[ks] = tiles0 + l32 * ROW_B + 16 * ((2 * ks + hf) ^ chunk_swizzle<D>(l32));
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int r = 8 * half + 4 * hf + ((lane & 15) >> 2), d = 32 * dt + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      tr_a[dt][half] = tiles0 + TILE_B + r * ROW_B + 16 * ((d >> 3) ^ chunk_swizzle<D>(r)) + 2 * (d & 7);
    }
  auto ld_row = [&](int ks, unsigned off) __attribute__((always_inline)) {
    return *(const bf16x8 __attribute__((address_space(3)))*)(row_a[ks] + off);
  };
  // A operand of O^T += V^T P^T: row = d (32dt + lane%32), slots = keys 16kk + 8(e/4) + 4hf + e%4 of this wavefront's rows
  auto ld_tr = [&](int kk, int dt, unsigned off) __attribute__((always_inline)) {
    const unsigned o = off + kk * 16 * ROW_B;
    bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(tr_a[dt][0] + o));
    bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(tr_a[dt][1] + o));
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) oacc[dt] = zero16();
  float m = -__builtin_inff(), l = 0.f;
  bf16x8 op[NOP];

  // The diagonal block is always the last tile of a row: it takes its own instantiation of the tile
  // body, so that the other tiles carry no mask selects.
  auto tile = [&](auto diag_c, auto buf_c, int t) __attribute__((always_inline)) {
    constexpr bool diag = decltype(diag_c)::value;
    constexpr unsigned BO = decltype(buf_c)::value * 2 * TILE_B;  // the tile's buffer, as an immediate offset of every LDS read
    const bool more = t + 1 < ntiles;
    if (more && (t + 1) % kJ == 0) stage_indices(t + 1);
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();  // tile t has landed for everyone; everyone is done with tile t-1
    if (more) issue(t + 1);
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {  // keys 32mt .. 32mt+31 of the tile
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) op[ks] = ld_row(ks, BO + mt * 32 * ROW_B);  // K rows
      __builtin_amdgcn_sched_barrier(0);
      f32x16 sacc = zero16();
#pragma unroll
      for (int ks = 0; ks < NOP; ++ks) {  // S^T = K Q^T, refilling every operand register with a V^T operand
        sacc = mfma32(op[ks], qf[ks], sacc);
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
          if (32 * mt + c_row(v, hf) > qloc) sacc[v] = -__builtin_inff();
      }
      // max3 below is inline asm, whose reads of the matrix instructions' results the compiler's hazard recogniser
      // does not see: a vector instruction may read a register written by an 8-pass matrix instruction only 12 wait
      // states after it.  (The masked tile goes through compiler-visible selects first.)  Without the wait a lane now
      // and then took a stale value into its running maximum: harmless for the result's accuracy (the softmax does
      // not depend on the reference point) but not bitwise repeatable.
      if (!diag) asm volatile("s_nop 7\n\ts_nop 3" : "+v"(sacc));
      // online softmax with a lazy running maximum: the reference m follows the true maximum only when
      // that has grown by more than kLazy (in log2 units), so p stays below 2^kLazy and the accumulated
      // O is rescaled only then; O and the row sum carry the same factor, so the result is the same
      float mx = max3(sacc[0], sacc[1], sacc[2]);
#pragma unroll
      for (int v = 3; v < 15; v += 2) mx = max3(mx, sacc[v], sacc[v + 1]);
      mx = max_across_halves(fmaxf(mx, sacc[15]));
      const bool first = m == -__builtin_inff();  // nothing accumulated yet for this query
      const bool move = first | ((mx - m) * P.scale_log2e > kLazy);
      const float m_new = move ? fmaxf(m, mx) : m;
      const float m_use = m_new == -__builtin_inff() ? 0.f : m_new;  // no unmasked key seen yet: keep the exponent finite
      const float alpha = first ? 1.0f : fast_exp2((m - m_use) * P.scale_log2e);
      const float neg_m = -m_use * P.scale_log2e;
      bf16x8 pb[2];
#pragma unroll
      for (int v = 0; v < 16; ++v) pb[v >> 3][v & 7] = (bf16)fast_exp2(__builtin_fmaf(sacc[v], P.scale_log2e, neg_m));
      float rs = l * alpha;  // the row sum adds the probabilities as rounded to bf16, the weights the accumulation applies
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 x = pb[kk];
        rs = sum2(__builtin_shufflevector(x, x, 0, 1), rs);
        rs = sum2(__builtin_shufflevector(x, x, 2, 3), rs);
        rs = sum2(__builtin_shufflevector(x, x, 4, 5), rs);
        rs = sum2(__builtin_shufflevector(x, x, 6, 7), rs);
      }
      l = rs;
      m = m_new;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[dt][v] *= alpha;
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) oacc[dt] = mfma32(op[kk * (D / 32) + dt], pb[kk], oacc[dt]);
    }
  };
  {  // two tiles per iteration, so that the buffer of a tile is known at compile time
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
  }

  l += __shfl_xor(l, 32, 64);  // the two lane halves hold different keys of the same query
  if (qvalid) {
    const float inv = 1.0f / l;  // l > 0 for every existing query: its own key is never masked
    const int64_t obase = (tq * P.Hq + h) * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int d0 = 32 * dt + 8 * vg + 4 * hf;
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = oacc[dt][4 * vg + e] * inv;
        if (OUT_F32) {
          *(float4*)((float*)P.o + obase + d0) = make_float4(x[0], x[1], x[2], x[3]);
        } else {
          bf16x4 y;
          y[0] = (bf16)x[0]; y[1] = (bf16)x[1]; y[2] = (bf16)x[2]; y[3] = (bf16)x[3];
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
  Geo gb;
  int rc = make_geo(p, &gb);
  if (rc != SB_OK) return rc;
  if (gb.S == 0 || gb.T == 0 || gb.NQB == 0) return SB_OK;
  const Geo g = tile_geo(gb);  // the kernels work on 64-row tiles; for larger selection blocks the plan holds the tile-level selection
  if (!q || !k || !v || !sel_rowptr || !sel_idx || !plan || !o || !lse || !ws) { set_error("null argument"); return SB_ERR_INVALID_ARG; }
  hipStream_t st = (hipStream_t)stream;
  PlanOffsets po = plan_offsets(gb);
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
  P.rowptr = gb.r == 1 ? sel_rowptr : (const int32_t*)(pb + po.t_rowptr);
  P.idx = gb.r == 1 ? sel_idx : (const int32_t*)(pb + po.t_idx); P.work = (const int32_t*)(pb + po.work_fwd);
  P.items = (const WorkItem*)(pb + po.items);
  P.cu = t.cu; P.qb_off = t.qb_off; P.qb_seq = t.qb_seq; P.bm_off = t.bm_off;
  P.NQB = g.NQB; P.T = g.T; P.Hq = g.Hq; P.Hkv = g.Hkv; P.G = g.G; P.Hs = g.Hs; P.mode = g.mode;
  P.scale = g.softmax_scale; P.scale_log2e = g.softmax_scale * 1.4426950408889634f;
  P.out_f32 = g.dtype == SB_F32;
  P.cu_busy = nullptr;
  if (g_instrument & 1) {
    if ((rc = fill_zero(wb + wo.cu_busy, sizeof(uint64_t) * SB_CU_SLOTS, st)) != SB_OK) return rc;
    P.cu_busy = (unsigned long long*)(wb + wo.cu_busy);
  }
  const int heads = g.mode == SB_SELECT_PER_QHEAD ? 1 : g.G;  // query heads that share a work item
  const int64_t n_items = (int64_t)g.Hs * g.NQB;
  if (n_items > 0x3fffffffll) { set_error("too many work items for one launch"); return SB_ERR_INVALID_ARG; }
  const int parts = (heads + 3) / 4, hpp = (heads + parts - 1) / parts;  // the group kernel takes `hpp` heads per workgroup
  const bool tickets = use_tickets(n_items) && heads <= kTicketSlots;
  P.n_items = (int)n_items; P.ticket = nullptr;
  KernelTimer kt(K_FWD, st);
  if (tickets) {
    P.ticket = (int*)(wb + wo.ticket);
    if ((rc = fill_zero(P.ticket, sizeof(int32_t) * kTicketSlots, st)) != SB_OK) return rc;
  }
  const int64_t n_slots = ticketed_grid(n_items, tickets);  // workgroups per head plane
  if (hpp >= 3 && parts * hpp == heads) {  // heads share K/V tiles in LDS; with a head slot left idle the per-head kernel is faster
    dim3 grid((unsigned)n_slots, (unsigned)parts), block(128 * hpp);
#define SB_FWD_LAUNCH(DD, FF) hipLaunchKernelGGL((attn_fwd_group_kernel<DD, FF>), grid, block, 0, st, P, heads)
    if (g.D == 128) {
      if (P.out_f32) SB_FWD_LAUNCH(128, true); else SB_FWD_LAUNCH(128, false);
    } else {
      if (P.out_f32) SB_FWD_LAUNCH(64, true); else SB_FWD_LAUNCH(64, false);
    }
#undef SB_FWD_LAUNCH
  } else {
    const int64_t n_wg = n_slots * heads;
    if (n_wg > 0x7fffffffll) { set_error("too many work items for one launch"); return SB_ERR_INVALID_ARG; }
    dim3 grid((unsigned)n_wg), block(128);
#define SB_FWD_LAUNCH(DD, FF) hipLaunchKernelGGL((attn_fwd_kernel<DD, FF>), grid, block, 0, st, P, (int)n_items, heads)
    if (g.D == 128) {
      if (P.out_f32) SB_FWD_LAUNCH(128, true); else SB_FWD_LAUNCH(128, false);
    } else {
      if (P.out_f32) SB_FWD_LAUNCH(64, true); else SB_FWD_LAUNCH(64, false);
    }
#undef SB_FWD_LAUNCH
  }
  SB_LAUNCH_CHECK("attn_fwd_kernel");
  return SB_OK;
}
