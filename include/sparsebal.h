/*
 * libsparsebal — packed (varlen), causal, GQA dynamic block-sparse attention, forward and
 * backward, with a per-sequence sparsity budget.  MI355X (gfx950) only.
 *
 * The computation is the block-sparse attention of the SparseBalance paper (arXiv 2604.13847),
 * section 2.2: keys/values are cut into fixed-size blocks, a routing score relates each query
 * block to the mean of each key block (the MoBA indexer the paper reuses), the Top-K blocks are
 * kept, and attention is one softmax over the kept keys (Eq. 2; Eq. 1 when every block is kept).
 * The budget k (number of kept blocks) is set per sequence, which is what the paper's dynamic
 * sparsity tuning (section 4.1, Algorithm 1 output) feeds into the kernel.
 *
 * Conventions
 *   - Every function returns SB_OK (0) or a negative error; sb_last_error() gives thread-local text.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *   - The caller owns every buffer, including workspaces; the library never allocates or frees
 *     device memory and never synchronises the stream.  All device work is enqueued on the
 *     hipStream_t passed as `stream` (a null pointer is the default stream).  Host arrays are read
 *     during the call only.
 *   - Layouts are row-major and contiguous, last index fastest:
 *       Q, O, dO, dQ : [T][Hq][D]     K, V, dK, dV : [T][Hkv][D]     LSE : [Hq][T] float
 *     Block j of sequence s covers packed rows cu[s]+j*B .. min(cu[s]+(j+1)*B, cu[s+1])-1; blocks
 *     are aligned to the sequence start and never straddle sequences.
 *     n_s = ceil(L_s/B) blocks per sequence, NQB = sum_s n_s, qb_off[s] = sum_{t<s} n_t.
 *   - Selection heads Hs: Hq in SB_SELECT_PER_QHEAD (one block list per query head) or Hkv in
 *     SB_SELECT_PER_KVGROUP (one list shared by the Hq/Hkv query heads of a KV head; its score is
 *     the sum of their scores).  Query head h reads KV head h / (Hq/Hkv).
 *   - scores: per sequence a dense [Hs][n_s][n_s] float block at element offset Hs*sum_{t<s} n_t^2;
 *     entry (hs,i,j) with j >= i is -infinity.
 *   - Selection CSR: row id = hs*NQB + qb_off[s] + i has c(s,i) = min(k_s, i+1) entries, the block
 *     indices (local to the sequence) kept by query block i, ascending, the last being i itself.
 *     sel_rowptr is therefore a closed form of cu_seqlens and topk.
 *   - No call takes the size of a buffer: every `ws`, `plan` and output must have at least the size sb_get_layout
 *     reports for the same problem; an undersized buffer is overrun, not detected.
 *   - A `ws` buffer is scratch of one call at a time (tables, counters, converted operands): calls that may overlap in
 *     time (different streams) need buffers of their own; calls ordered on one stream may share one.  The library keeps
 *     no device state between calls besides what `plan` and `ws` hold (and the built-in scratch of sb_select_topk_static).
 *   - Supported: block_size 64, 128 or 256; head_dim 64 or 128; Hq % Hkv == 0; n_s <= SB_MAX_BLOCKS_PER_SEQ;
 *     in SB_SELECT_PER_KVGROUP Hq/Hkv <= 8; selection entries and rows (at the granularity of 64-token tiles) must
 *     fit 32-bit row pointers.  Anything else returns SB_ERR_UNSUPPORTED.
 *   - Degenerate inputs: empty sequences are allowed; T == 0 or S == 0 is a no-op returning SB_OK;
 *     k_s > n_s is clamped to n_s; k_s < 1 is an error.
 */
#ifndef SPARSEBAL_H
#define SPARSEBAL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SB_OK 0
#define SB_ERR_INVALID_ARG (-1)
#define SB_ERR_UNSUPPORTED (-2)
#define SB_ERR_WORKSPACE_TOO_SMALL (-3) /* sb_select_topk_static: the problem's tables exceed the built-in scratch */
#define SB_ERR_HIP (-4)

#define SB_BF16 0 /* Q,K,V,O,dO,dQ,dK,dV are bfloat16 */
#define SB_F32 1  /* they are float; the attention kernels round them to bfloat16 on entry */

#define SB_SELECT_PER_QHEAD 0
#define SB_SELECT_PER_KVGROUP 1

#define SB_MAX_BLOCKS_PER_SEQ 16384

typedef struct sb_problem {
  int32_t total_tokens, num_seqs;          /* T, S */
  int32_t num_q_heads, num_kv_heads;       /* Hq, Hkv */
  int32_t head_dim, block_size;            /* D, B */
  int32_t dtype;                           /* SB_BF16 | SB_F32 */
  int32_t select_mode;                     /* SB_SELECT_PER_QHEAD | SB_SELECT_PER_KVGROUP */
  float softmax_scale;                     /* the 1/sqrt(d) of Eq. 1-2; <= 0 means 1/sqrt(head_dim) */
  float score_scale;                       /* factor on the routing score; <= 0 means softmax_scale */
  const int32_t *cu_seqlens_host;          /* host [S+1], cu[0] = 0, non-decreasing, cu[S] = T */
  const int32_t *cu_seqlens_dev;           /* dev  [S+1], same values */
  const int32_t *topk_host;                /* host [S], budget k_s >= 1 counting the diagonal block */
  const int32_t *topk_dev;                 /* dev  [S], same values */
} sb_problem;

/* Sizes a caller needs before allocating; filled on the host from sb_problem alone. */
typedef struct sb_layout {
  int64_t num_qblocks;   /* NQB */
  int64_t sel_heads;     /* Hs */
  int64_t scores_elems;  /* floats in `scores` */
  int64_t pooled_elems;  /* floats in `kbar_out`: NQB*Hkv*D */
  int64_t sel_rows;      /* Hs*NQB; sel_rowptr holds sel_rows+1 int32 */
  int64_t sel_nnz;       /* int32 entries in sel_idx */
  int64_t plan_bytes;    /* bytes of the `plan` buffer of sb_plan_worklist */
  int64_t scores_ws_bytes, select_ws_bytes, fwd_ws_bytes, bwd_ws_bytes; /* bytes of the `ws` arguments */
  int64_t attended_pairs_per_head_sum; /* sum over query heads of unmasked (query,key) pairs,
                                          the diagonal block counted as its causal triangle */
  int64_t coverage_ws_bytes; /* bytes of the `ws` argument of sb_score_coverage */
} sb_layout;

/* Host only.  Validates the problem and fills `out`. */
int sb_get_layout(const sb_problem *p, sb_layout *out);

/* Host only.  Budget from a keep ratio: k_s = clamp(ceil(rho_s*n_s - 1e-6), 1, n_s), one budget per
 * sequence (the budget is a count of selected blocks, paper section 2.2). */
int sb_keep_ratio_to_topk(const int32_t *cu_seqlens_host, int32_t S, int32_t block_size,
                          const float *keep_ratio_host, int32_t *topk_out_host);

/* Host only.  Writes the closed-form CSR row pointers (sel_rows+1 int32) to a host array. */
int sb_sel_rowptr_host(const sb_problem *p, int32_t *rowptr_out_host);

/* Routing scores (paper section 2.2, MoBA indexer): score[s][hs][i][j] = score_scale *
 * < mean of Q over query block i , mean of K over key block j > for j < i (summed over the group's
 * query heads in SB_SELECT_PER_KVGROUP), -infinity for j >= i.  Means are over the valid tokens of a
 * block.  q, k: dev, dtype per p->dtype.  kbar_out: dev [NQB][Hkv][D] float or null.  scores_out:
 * dev, scores_elems floats.  ws: dev, scores_ws_bytes. */
int sb_block_scores(const sb_problem *p, const void *q, const void *k, float *kbar_out, float *scores_out,
                    void *ws, void *stream);

/* Top-K block selection (paper section 2.2): for every row (s,hs,i) keep the diagonal block i plus
 * the c(s,i)-1 best past blocks j < i under the total order (score descending, then block index
 * ascending; -0 == +0; NaN below every number).  Bit-exact function of `scores`.  Writes
 * sel_rowptr_out (dev, sel_rows+1 int32) and sel_idx_out (dev, sel_nnz int32).  ws: dev, select_ws_bytes. */
int sb_select_topk(const sb_problem *p, const float *scores, int32_t *sel_rowptr_out, int32_t *sel_idx_out,
                   void *ws, void *stream);

/* sb_select_topk for callers that cannot allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus `ws`, same results bit for bit.  The
 * geometry tables that `ws` holds in sb_select_topk live in a device array built into the library (SB_STATIC_SELECT_WS_BYTES
 * per GPU, held until the process ends); a problem whose tables (select_ws_bytes of sb_layout) do not fit returns
 * SB_ERR_WORKSPACE_TOO_SMALL and enqueues nothing.  The call allocates and frees nothing.  All calls on one GPU share that
 * array: calls on different streams of one GPU that overlap in time race; calls on one stream are ordered.  The first
 * call on a device looks up the array's address (a host-side query, no allocation); make it outside graph capture. */
#define SB_STATIC_SELECT_WS_BYTES (1 << 20)
int sb_select_topk_static(const sb_problem *p, const float *scores, int32_t *sel_rowptr_out, int32_t *sel_idx_out,
                          void *stream);

/* The indexer and the Top-K selection as one step (paper section 2.2).  Arguments as for
 * sb_block_scores and sb_select_topk; ws: dev, scores_ws_bytes.  sel_rowptr_out and sel_idx_out are
 * bit-identical to calling the two separately, whichever form is used:
 *   scores_out != NULL  the score matrix is written as by sb_block_scores (it stays available for the
 *                       budget controller below) and the selection is taken from it;
 *   scores_out == NULL  one kernel computes each row's scores on chip and selects there: the score
 *                       matrix (scores_elems floats) is neither allocated nor written nor read back.
 *                       A sequence so long that a single row of keys does not fit the compute unit's
 *                       local memory returns SB_ERR_UNSUPPORTED (not reachable below
 *                       SB_MAX_BLOCKS_PER_SEQ on gfx950). */
int sb_score_select(const sb_problem *p, const void *q, const void *k, float *kbar_out, float *scores_out,
                    int32_t *sel_rowptr_out, int32_t *sel_idx_out, void *ws, void *stream);

/* Work plan for the attention kernels: query-major work items (s,hs,i) ordered by decreasing
 * selected-block count (longest first, as in balanced partitioning by workload weight, paper
 * section 4.3), the key-major transpose of the selection (for every (s,hs,j) the set of query
 * blocks that kept j) and key-major items ordered by decreasing weight; a column that very many query blocks
 * kept (an attention sink) is cut into several items of bounded weight, so that no single workgroup becomes the
 * straggler the paper's section 3.2 describes.  plan_out: dev, plan_bytes, opaque; it is valid for this problem and
 * this selection only. */
int sb_plan_worklist(const sb_problem *p, const int32_t *sel_rowptr, const int32_t *sel_idx, void *plan_out,
                     void *stream);

/* Host only; for tests and tools that check the plan's properties (every item once, longest first, the transpose is a
 * transpose).  Writes byte offsets into the plan buffer and three sizes to out[SB_PLAN_NUM_SECTIONS]:
 *   QB_OFF   int32 [S+1]      first 64-token tile of every sequence
 *   BM_OFF   int64 [S+1]      first bitmap word of every sequence (per selection head), n_s * ceil(n_s/32) words each
 *   QB_SEQ   int32 [NQB]      sequence of every tile
 *   WORK_FWD int32 [Hs*NQB]   selection rows (hs * NQB + tile) in launch order, longest first
 *   COLCOST  int32 [Hkv*NQB]  (query block, query head) tiles of every key-major column g * NQB + tile
 *   BITMAP   uint32           bit i of word (s, hs, j, i/32): query tile i of head hs kept key tile j
 *   BWD_ITEMS 4 x int32 each  key-major items in launch order: column (or -1: none), bitmap words lo | hi << 16 the item
 *                             covers, partial slot (or -1: the item is the whole column), tiles; BWD_ITEMS_COUNT entries
 *   COUNTERS int32 [2]        partial slots in use, split columns
 *   SPLIT_COLS 3 x int32 each column, first partial slot, parts
 *   SPLIT_WEIGHT              a column with more tiles than this is cut into parts of at least this many
 * (NQB counts 64-token tiles, whatever the selection block size.) */
#define SB_PLAN_QB_OFF 0
#define SB_PLAN_BM_OFF 1
#define SB_PLAN_QB_SEQ 2
#define SB_PLAN_WORK_FWD 3
#define SB_PLAN_COLCOST 4
#define SB_PLAN_BITMAP 5
#define SB_PLAN_BWD_ITEMS 6
#define SB_PLAN_COUNTERS 7
#define SB_PLAN_SPLIT_COLS 8
#define SB_PLAN_BWD_ITEMS_COUNT 9
#define SB_PLAN_SPLIT_WEIGHT 10
#define SB_PLAN_SPLIT_MAX 11
#define SB_PLAN_NUM_SECTIONS 12
int sb_plan_sections(const sb_problem *p, int64_t *out);

/* Forward (Eq. 2): for every query row r of query block i and query head h,
 * O_r = sum_j softmax_j(softmax_scale * q_r.k_j) v_j over the keys j of the selected blocks that are
 * not in r's future; LSE_r = log sum_j exp(softmax_scale * q_r.k_j).  Any valid selection is
 * accepted (ascending, unique, <= i, containing i).  o: dev like q; lse: dev [Hq][T] float;
 * ws: dev, fwd_ws_bytes. */
int sb_sparse_attn_fwd(const sb_problem *p, const void *q, const void *k, const void *v,
                       const int32_t *sel_rowptr, const int32_t *sel_idx, const void *plan, void *o, float *lse,
                       void *ws, void *stream);

/* Backward of Eq. 2 with the selection held fixed: dQ, dK, dV from dO (dK, dV summed over the
 * query heads of each KV head).  o and lse are the forward's outputs.  Deterministic: every output
 * element is accumulated by one workgroup in a fixed order.  ws: dev, bwd_ws_bytes. */
int sb_sparse_attn_bwd(const sb_problem *p, const void *q, const void *k, const void *v, const void *o,
                       const float *lse, const void *d_o, const int32_t *sel_rowptr, const int32_t *sel_idx,
                       const void *plan, void *dq, void *dk, void *dv, void *ws, void *stream);

/* ---- budget controller (paper sections 4.1 and 4.2): what sets topk[] before the calls above ----
 *
 * Coverage curves of the routing scores (section 4.1, Eq. 4).  For query block i of sequence s and one
 * selection head, the scores of the earlier blocks j < i are normalised by a softmax and sorted in
 * descending order into importance scores r_1 >= r_2 >= ... (sum 1); a budget k keeps the diagonal
 * block plus the k-1 best earlier blocks, so the row covers the sum of its min(k-1, i) largest r.
 * C_s(k), k = 1..n_s, is the mean of that over the sequence's query blocks and selection heads:
 * non-decreasing, C_s(1) = 1/n_s, C_s(n_s) = 1.  `scores`: dev, as written by sb_block_scores (finite
 * for j < i).  coverage_out: dev, NQB floats, C_s(k) at qb_off[s] + k - 1.  ws: dev, coverage_ws_bytes.
 * Deterministic (fixed summation order). */
int sb_score_coverage(const sb_problem *p, const float *scores, float *coverage_out, void *ws, void *stream);

/* Profiled latency table M[x, k] (section 4.2, Eq. 10): latency[a*num_budgets + b] is the measured
 * latency at length lengths[a] (tokens) and budget budgets[b] (blocks); both grids strictly
 * increasing.  All pointers are host pointers; the caller owns them. */
typedef struct sb_perf_table {
  int32_t num_lengths, num_budgets;
  const float *lengths;
  const float *budgets;
  const float *latency;
} sb_perf_table;

/* Host only.  Perf.predict (Eq. 8): the table interpolated linearly in length and in budget, clamped
 * at its edges. */
int sb_perf_predict(const sb_perf_table *t, double length, double budget, double *latency_out);

/* Host only.  Perf.align (Eq. 9): the largest integer budget in 1..max_budget whose predicted latency
 * does not exceed target_latency; 1 if none does. */
int sb_perf_align(const sb_perf_table *t, double length, double target_latency, int32_t max_budget,
                  int32_t *budget_out);

/* Host only.  Workload-aware dynamic sparsity tuning (section 4.1, Algorithm 1) with every packed
 * sequence as one micro-batch.  p->topk_host are the base budgets k_base.  T_anchor is the minimum,
 * mean or maximum (Eq. 3) of the predicted latencies at the base budgets; k_anchor = Perf.align(L_s,
 * T_anchor) in 1..n_s; the final budget is k_anchor unless C_s(k_base) - C_s(k_anchor) exceeds
 * threshold_p (Eq. 5), in which case it is the smallest k with C_s(k_base) - C_s(k) <= threshold_p.
 * coverage_host: host copy of sb_score_coverage's output.  topk_final_out: host [S];
 * topk_anchor_out (host [S]) and t_anchor_out may be null.  Empty sequences keep their base budget. */
#define SB_ANCHOR_MIN 0
#define SB_ANCHOR_MEAN 1
#define SB_ANCHOR_MAX 2
int sb_dst_tune(const sb_problem *p, const float *coverage_host, const sb_perf_table *perf, int anchor,
                double threshold_p, int32_t *topk_final_out, int32_t *topk_anchor_out, double *t_anchor_out);

/* ---- sparsity-aware batching (paper section 4.3, Algorithm 2); host only, CPU side of the data loader ----
 *
 * Sparsity predictor Spar: for each sequence-length bin b (bin_edges[b] <= L < bin_edges[b+1], lengths
 * outside clamp to the first / last bin) an exponential moving average of the final budgets the
 * tuning step produced: ema[b] <- decay*ema[b] + (1-decay)*k per sample, in order; the first sample of
 * a bin initialises it (seen[b] = 1).  sb_spar_predict returns ema[b], or k_base while the bin has
 * seen nothing.  ema: [num_bins] float, seen: [num_bins] bytes, bin_edges: [num_bins+1]; caller-owned. */
int sb_spar_update(float *ema, uint8_t *seen, const float *bin_edges, int32_t num_bins, double decay,
                   const int32_t *lengths, const int32_t *k_final, int32_t n);
int sb_spar_predict(const float *ema, const uint8_t *seen, const float *bin_edges, int32_t num_bins,
                    int32_t length, double k_base, double *k_out);

/* `bin_packing`: balanced partition of n weights into num_bins bins by the longest-first greedy
 * (decreasing weight, ties to the lower index; each to the least loaded bin, ties to the lower bin).
 * bin_of_out[i] is the bin of sample i.  Bin sizes are not constrained. */
int sb_balanced_partition(const double *weights, int32_t n, int32_t num_bins, int32_t *bin_of_out);

/* Algorithm 2: W[i] = Perf.predict(lengths[i], k_pred[i]); samples are split over dp_size DP ranks, then
 * the samples of dp_rank over num_microbatches micro-batches (= gbs / (mbs * N)).  weights_out (nullable),
 * dp_bin_out, mb_bin_out: [n]; mb_bin_out is -1 for the samples of other ranks. */
int sb_sab_batches(const sb_perf_table *perf, const int32_t *lengths, const double *k_pred, int32_t n,
                   int32_t dp_size, int32_t dp_rank, int32_t num_microbatches, double *weights_out,
                   int32_t *dp_bin_out, int32_t *mb_bin_out);

/* Instrumentation (measurement only; off by default).  `flag` is a bit set:
 *   SB_INSTR_CU_BUSY  the attention kernels add, for every workgroup, its run time in ticks of the
 *                     100 MHz constant clock to a per-compute-unit slot inside `ws`; sb_read_cu_busy
 *                     copies the SB_CU_SLOTS slots of the last forward or backward call that used
 *                     `ws` to host memory (it synchronises the stream).  This is the per-CU busy time
 *                     whose max/mean is the imbalance measure of the paper's Eq. 11 applied to CUs.
 *   SB_INSTR_KERNEL_EVENTS  every kernel launch is bracketed by HIP events on the launch stream;
 *                     sb_read_kernel_times waits for them, writes per-kernel total milliseconds and
 *                     launch counts (SB_NUM_KERNELS entries each, host) and resets the record.  The
 *                     events are recycled: once a few steps have run, a timed launch creates none.
 * The flag and the event record are process-wide (one mutex guards them): calls from several threads
 * are safe, their records interleave.  bwd_dkv also covers the reduction of split key-major columns. */
#define SB_CU_SLOTS 512
#define SB_INSTR_CU_BUSY 1
#define SB_INSTR_KERNEL_EVENTS 2
#define SB_NUM_KERNELS 10 /* pool, score, topk, plan, fwd, bwd_prep, bwd_dq, bwd_dkv, coverage, score_select; bwd_prep is the
                             conversion of float32 inputs in the backward call (nothing for bf16 inputs); score_select is the
                             single kernel of sb_score_select without scores_out */
int sb_set_instrumentation(int flag);
int sb_read_cu_busy(const void *ws, uint64_t *busy_out_host, void *stream);
int sb_read_kernel_times(double *total_ms_host, int64_t *launches_host);

const char *sb_last_error(void);
const char *sb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPARSEBAL_H */
