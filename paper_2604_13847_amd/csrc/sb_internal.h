// Internal declarations shared by the translation units of libsparsebal (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <string>
#include <vector>

#include "sparsebal.h"

namespace sb {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

void set_error(const char* fmt, ...);

#define SB_CHECK_HIP(expr)                                                         \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                        \
      ::sb::set_error("%s failed: %s", #expr, hipGetErrorString(e_));              \
      return SB_ERR_HIP;                                                           \
    }                                                                              \
  } while (0)

#define SB_LAUNCH_CHECK(name)                                                      \
  do {                                                                             \
    hipError_t e_ = hipGetLastError();                                             \
    if (e_ != hipSuccess) {                                                        \
      ::sb::set_error("launch of %s failed: %s", name, hipGetErrorString(e_));     \
      return SB_ERR_HIP;                                                           \
    }                                                                              \
  } while (0)

// Host-side geometry derived from sb_problem in O(S).
struct Geo {
  int T = 0, S = 0, Hq = 0, Hkv = 0, G = 1, D = 0, B = 64, Hs = 0, mode = 0, dtype = 0;
  float softmax_scale = 0.f, score_scale = 0.f;
  int64_t NQB = 0;          // total query blocks
  int n_max = 0;            // largest n_s
  int64_t scores_unit = 0;  // sum n_s^2 (per selection head)
  int64_t nnz_unit = 0;     // sum_s (k n - k(k-1)/2) (per selection head)
  int64_t bm_words_unit = 0;  // sum_s n_s * ceil(n_s/32) (per selection head)
  int64_t pairs_unit = 0;   // unmasked (query,key) pairs per query head
  // The attention kernels always work on 64-row tiles.  With a selection block of B = 64*r rows a kept
  // block stands for r consecutive key tiles and a query block for r query tiles (see plan_expand_kernel).
  int r = 1;                // tiles per block
  int64_t NT = 0;           // total 64-row tiles
  int nt_max = 0;           // largest tile count of a sequence
  int64_t nnzT_unit = 0;    // tile-level selection entries per selection head
  int64_t bmT_words_unit = 0;  // sum_s nt_s * ceil(nt_s/32)
};
// The same problem as the attention kernels see it: 64-row blocks, tile counts in the block fields.
inline Geo tile_geo(const Geo& g) {
  Geo t = g;
  t.B = 64; t.r = 1; t.NQB = g.NT; t.n_max = g.nt_max; t.nnz_unit = g.nnzT_unit; t.bm_words_unit = g.bmT_words_unit;
  return t;
}
// Tile-level selection entries of the first `it` query tiles of a sequence with budget k (in blocks):
// query tile it' of block I = it'/r keeps r tiles for each of its min(k, I+1)-1 earlier blocks plus the
// tiles r*I .. it' of its own block.
inline __host__ __device__ int64_t tile_entries_before(int64_t it, int64_t k, int64_t r) {
  const int64_t I = it / r, a = it % r;
  const int64_t sumc = I <= k ? I * (I - 1) / 2 : k * (k - 1) / 2 + (I - k) * (k - 1);  // sum_{I'<I} (min(k, I'+1) - 1)
  const int64_t cI = (k < I + 1 ? k : I + 1) - 1;
  return r * r * sumc + I * (r * (r + 1) / 2) + a * cI * r + a * (a + 1) / 2;
}

// Validates p and fills g; returns SB_OK or an error (message set).
int make_geo(const sb_problem* p, Geo* g);

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
constexpr int kMaxDevices = 64;  // per-device state (attributes set, symbol addresses) is kept for this many ordinals

// Device tables computed by geom_kernel from cu_seqlens_dev / topk_dev.
struct TableOffsets {
  size_t qb_off;     // int32 [S+1]   prefix of n_s
  size_t sc_off;     // int64 [S+1]   prefix of n_s^2
  size_t row_base;   // int32 [S+1]   prefix of c-sums (k n - k(k-1)/2)
  size_t bm_off;     // int64 [S+1]   prefix of n_s*ceil(n_s/32)
  size_t kclamp;     // int32 [S]     min(k_s, n_s)
  size_t qb_seq;     // int32 [NQB]   sequence of each query block
  size_t bytes;
};
TableOffsets table_offsets(const Geo& g);

struct Tables {  // device pointers into a tables area
  const int32_t* cu;
  const int32_t* qb_off;
  const int64_t* sc_off;
  const int32_t* row_base;
  const int64_t* bm_off;
  const int32_t* kclamp;
  const int32_t* qb_seq;
};
Tables make_tables(const Geo& g, const sb_problem* p, void* base);
int launch_geom(const Geo& g, const sb_problem* p, void* base, hipStream_t st);

// Layout of the opaque plan buffer.
struct PlanOffsets {
  size_t tables;     // TableOffsets area
  size_t work_fwd;   // int32 [Hs*NQB]   row ids, longest first
  size_t colcost;    // int32 [Hkv*NQB]  tiles in each key-major column (summed over the group's heads)
  size_t bwd_items;  // ColItem [Hkv*(NQB+E)]  key-major items: entry r*Hkv + g is the r-th heaviest item of KV head g (col = -1: none)
  size_t counters;   // int32 [4]  {partial slots in use, split columns}, zeroed by every plan call
  size_t split_cols; // int32 [3*E]  (column, first partial slot, parts) of every split column
  size_t bitmap;     // uint32 [Hs * bm_words_unit] transpose bitmap: bit i of column (s,hs,j)
  size_t items;      // WorkItem [Hs*NQB]  descriptors of the query-major items, in work_fwd order
  // only for selection blocks larger than a tile (r > 1); everything above is then at tile level
  size_t blk_tables; // TableOffsets area of the block-level geometry
  size_t t_rowptr;   // int32 [Hs*NT+1]  tile-level selection CSR
  size_t t_idx;      // int32 [Hs*nnzT]
  size_t bytes;
};
constexpr int kBwdBins = 4096;
// A key-major column (s, g, j) is one work item unless it is heavier than split_weight() tiles: then it is cut, at the
// granularity of 32 query blocks, into parts of at least that weight that are separate work items; the parts leave
// fp32 partial dK/dV in the backward workspace and a reduction adds them in part order.  The bounds below follow from
// "every part but a column's last has at least split_weight() tiles": at most split_extra_max() parts close, so there are
// at most that many split columns, that many items more than columns (per KV head and overall), and twice that many
// partial slots.  All three are functions of the problem's sizes alone, so the host can size buffers and grids.
struct ColItem {
  int32_t col;     // g * NQB + global block index of the key block, or -1
  int32_t wrange;  // bitmap words [lo, hi) of the column this item covers: lo | hi << 16
  int32_t slot;    // partial slot of this part, or -1: the item is the whole column and writes dK/dV itself
  int32_t weight;  // (query block, query head) tiles of the item
};
static_assert(sizeof(ColItem) == 16, "ColItem is loaded as 4 dwords");
inline int64_t bwd_total_tiles(const Geo& tg) { return (int64_t)tg.Hq * tg.nnz_unit; }  // tg = tile_geo(...)
inline int split_weight(const Geo& tg) { const int64_t w = (bwd_total_tiles(tg) + 4095) / 4096; return (int)(w < 512 ? 512 : w); }
inline int split_extra_max(const Geo& tg) { return (int)(bwd_total_tiles(tg) / split_weight(tg)); }
// Everything a query-major workgroup needs to know about its item, so that it starts with one
// 32-byte load instead of a chain of dependent table lookups.
struct WorkItem {
  int32_t row;     // hs * NQB + query block (index into sel_rowptr)
  int32_t seq0;    // first token of the sequence
  int32_t len;     // tokens in the sequence
  int32_t i;       // query block inside the sequence
  int32_t e0;      // first selection entry of the row
  int32_t ntiles;  // selected blocks of the row
  int32_t hs;      // selection head
  int32_t s;       // sequence
};
static_assert(sizeof(WorkItem) == 32, "WorkItem is loaded as 8 dwords");
PlanOffsets plan_offsets(const Geo& g);

struct WsOffsets {
  size_t cu_busy;    // uint64 [SB_CU_SLOTS]
  size_t qc, kc, vc, oc, doc;  // bf16 copies when dtype == SB_F32 (0 size otherwise)
  size_t drow;       // float [Hq][T]
  size_t lse2;       // float [Hq][T]
  size_t ticket;     // int32 [64] work tickets of the query-major attention kernels (kTicketSlots)
  size_t partials;   // float [2*E][dK, dV][64][D]  partial sums of the parts of split key-major columns
  size_t bytes;
};
WsOffsets fwd_ws_offsets(const Geo& g);
WsOffsets bwd_ws_offsets(const Geo& g);
// Workgroups to launch for a list of n items when one item in sixteen is handed out by ticket at the end of the launch
// (see claim_item in sb_attn_common.h): two tail workgroups per held-back item, the total a multiple of 8.
constexpr int64_t kTicketMinItems = 4096;  // shorter lists are dealt by position only
inline bool use_tickets(int64_t n) { return n >= kTicketMinItems; }
inline int64_t ticketed_grid(int64_t n, bool tickets) { return (n + (tickets ? (n >> 7) << 3 : 0) + 7) / 8 * 8; }
size_t scores_ws_bytes(const Geo& g);
size_t coverage_ws_bytes(const Geo& g);

// Zero `bytes` (a multiple of 4) at `dst` with a small kernel on `st`: unlike a memset node this is safe to record
// into a HIP graph.
int fill_zero(void* dst, size_t bytes, hipStream_t st);
int fill_words(void* dst, size_t bytes, uint32_t value, hipStream_t st);

extern std::atomic<int> g_instrument;  // bit 0: per-CU busy ticks, bit 1: HIP events around each kernel

// HIP-event bracket around one kernel launch on its own stream (only when bit 1 is set).
enum KernelSlot { K_POOL = 0, K_SCORE, K_TOPK, K_PLAN, K_FWD, K_BWD_PREP, K_BWD_DQ, K_BWD_DKV, K_COVERAGE, K_SCORE_SELECT, K_NUM };
static_assert(K_NUM == SB_NUM_KERNELS, "kernel slots");
struct KernelTimer {
  int slot; hipStream_t st; void* start = nullptr;
  KernelTimer(int slot, hipStream_t st);
  ~KernelTimer();
};

}  // namespace sb
