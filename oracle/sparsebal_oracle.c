/*
 * CPU checker for packed, causal, GQA block-sparse attention with per-sequence budgets.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is compared against.  It shares no code, header, table or helper with the GPU
 * path and must never be called from it.  Inputs are float32 arrays (the caller rounds
 * them to the GPU's storage type first); every sum is accumulated in double and every
 * result is returned in double.  No blocking, fusion or reordering beyond the definitions.
 *
 * What is defined where (paper = "SparseBalance", arXiv 2604.13847):
 *   - dense attention softmax(Q K^T / sqrt(d)) V                        : section 2.2, Eq. 1
 *   - block-sparse attention softmax(Q K[I]^T / sqrt(d)) V[I], one joint
 *     softmax over the gathered keys                                    : section 2.2, Eq. 2
 *   - K/V cut into fixed-size blocks; routing metric = relevance of the
 *     query to the mean of each key block; Top-K blocks are kept        : section 2.2 (MoBA indexer)
 *   - budget k = number of selected blocks                              : section 2.2, last paragraph
 * Readings taken where the paper is silent are stated at each function.
 *
 * Parity status: every function below is pinned by CPU tests against closed forms, brute
 * force on small inputs, dense attention (Eq. 1) and finite differences.  Agreement with
 * the numerics of the implementation the paper's authors ran is "parity unpinned": the
 * paper prints no attention values.
 *
 * Layouts (row-major, last index fastest):
 *   Q, dO, O, dQ : [T][Hq][D]      K, V, dK, dV : [T][Hkv][D]      LSE : [Hq][T]
 *   block j of sequence s covers packed rows cu[s]+j*B .. min(cu[s]+(j+1)*B, cu[s+1])-1
 *   n_s = ceil(L_s / B); NQB = sum n_s; qb_off[s] = sum_{t<s} n_t
 *   selection heads Hs = Hq (mode 0: one selection per query head) or Hkv (mode 1: one
 *   selection shared by the query heads of a KV group)
 *   scores : per sequence a dense [Hs][n_s][n_s] block at offset Hs * sum_{t<s} n_t^2
 *   selection CSR: row id = hs*NQB + qb_off[s] + i; entries are block indices local to the
 *   sequence, ascending, the last one being i itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct orc_shape {
  int32_t T, S, Hq, Hkv, D, B;
  int32_t mode;          /* 0: selection per query head, 1: per KV group */
  const int32_t *cu;     /* [S+1] */
} orc_shape;

static int nblocks(const orc_shape *sh, int s) {
  int L = sh->cu[s + 1] - sh->cu[s];
  return (L + sh->B - 1) / sh->B;
}
static int sel_heads(const orc_shape *sh) { return sh->mode == 0 ? sh->Hq : sh->Hkv; }
static int64_t total_qblocks(const orc_shape *sh) {
  int64_t n = 0;
  for (int s = 0; s < sh->S; ++s) n += nblocks(sh, s);
  return n;
}
static int64_t qb_offset(const orc_shape *sh, int s) {
  int64_t n = 0;
  for (int t = 0; t < s; ++t) n += nblocks(sh, t);
  return n;
}
static int64_t score_offset(const orc_shape *sh, int s) {
  int64_t n = 0;
  for (int t = 0; t < s; ++t) n += (int64_t)nblocks(sh, t) * nblocks(sh, t);
  return n * sel_heads(sh);
}
/* selection head that query head h reads its block list from */
static int sel_head_of(const orc_shape *sh, int h) {
  int G = sh->Hq / sh->Hkv;
  return sh->mode == 0 ? h : h / G;
}

int64_t orc_num_qblocks(const orc_shape *sh) { return total_qblocks(sh); }
int64_t orc_scores_elems(const orc_shape *sh) { return score_offset(sh, sh->S); }

/* Budget from a keep ratio: the budget is a block count per sequence (section 2.2); a ratio
 * rho of the sequence's n blocks is read as k = ceil(rho*n - 1e-6) clamped to [1, n], one
 * value per sequence.  The 1e-6 absorbs float32 representation error of rho. */
int orc_keep_ratio_to_topk(const int32_t *cu, int S, int B, const float *rho, int32_t *k_out) {
  for (int s = 0; s < S; ++s) {
    int L = cu[s + 1] - cu[s];
    int n = (L + B - 1) / B;
    double x = ceil((double)rho[s] * (double)n - 1e-6);
    int k = (int)x;
    if (k < 1) k = 1;
    if (k > n) k = n;
    k_out[s] = (n == 0) ? 1 : k;
  }
  return 0;
}

/* Mean representation of each block (section 2.2): mean over the VALID tokens of the block.
 * X is [T][H][D]; out is [NQB][H][D]. */
int orc_block_mean(const orc_shape *sh, const float *X, int H, double *out) {
  int D = sh->D, B = sh->B;
  for (int s = 0; s < sh->S; ++s) {
    int L = sh->cu[s + 1] - sh->cu[s];
    int64_t qb0 = qb_offset(sh, s);
    for (int j = 0; j < nblocks(sh, s); ++j) {
      int first = j * B, last = (j + 1) * B < L ? (j + 1) * B : L;
      for (int h = 0; h < H; ++h)
        for (int d = 0; d < D; ++d) {
          double acc = 0.0;
          for (int t = first; t < last; ++t) acc += (double)X[((int64_t)(sh->cu[s] + t) * H + h) * D + d];
          out[((qb0 + j) * H + h) * D + d] = acc / (double)(last - first);
        }
    }
  }
  return 0;
}

/* Routing scores.  Token level (section 2.2): logit(t, h, j) = q_{t,h} . mean(K block j of
 * KV head g(h)).  The score of query BLOCK i is the mean of that logit over the block's valid
 * query tokens, times score_scale; in mode 1 the scores of the G query heads of a KV group
 * are added.  Only strictly past blocks j < i compete; j >= i is written as -infinity (the
 * block's own diagonal is always kept and the future is masked). */
int orc_block_scores(const orc_shape *sh, const float *Q, const float *K, double score_scale, double *scores) {
  int D = sh->D, B = sh->B, Hq = sh->Hq, Hkv = sh->Hkv, G = Hq / Hkv, Hs = sel_heads(sh);
  int64_t NQB = total_qblocks(sh);
  double *kbar = (double *)malloc(sizeof(double) * (size_t)(NQB > 0 ? NQB : 1) * Hkv * D);
  if (!kbar) return -1;
  orc_block_mean(sh, K, Hkv, kbar);
  for (int s = 0; s < sh->S; ++s) {
    int L = sh->cu[s + 1] - sh->cu[s], n = nblocks(sh, s);
    int64_t qb0 = qb_offset(sh, s), so = score_offset(sh, s);
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
      int first = i * B, last = (i + 1) * B < L ? (i + 1) * B : L;
      for (int hs = 0; hs < Hs; ++hs)
        for (int j = 0; j < n; ++j) {
          double *dst = &scores[so + ((int64_t)hs * n + i) * n + j];
          if (j >= i) { *dst = -INFINITY; continue; }
          int h0 = sh->mode == 0 ? hs : hs * G, h1 = sh->mode == 0 ? hs + 1 : (hs + 1) * G;
          double group = 0.0;
          for (int h = h0; h < h1; ++h) {
            const double *kb = &kbar[((qb0 + j) * Hkv + h / G) * D];
            double sum_logit = 0.0;
            for (int t = first; t < last; ++t) {
              const float *q = &Q[((int64_t)(sh->cu[s] + t) * Hq + h) * D];
              double logit = 0.0;
              for (int d = 0; d < D; ++d) logit += (double)q[d] * kb[d];
              sum_logit += logit;
            }
            group += sum_logit / (double)(last - first);
          }
          *dst = score_scale * group;
        }
    }
  }
  free(kbar);
  return 0;
}

/* The same scores for ONE row (sequence s, selection head hs, query block i): out[j], j < n_s. */
int orc_block_scores_row(const orc_shape *sh, const float *Q, const float *K, double score_scale, int s, int hs, int i,
                         double *out) {
  int D = sh->D, B = sh->B, Hq = sh->Hq, Hkv = sh->Hkv, G = Hq / Hkv;
  int L = sh->cu[s + 1] - sh->cu[s], n = nblocks(sh, s);
  if (D > 1024) return -2;
  int first = i * B, last = (i + 1) * B < L ? (i + 1) * B : L;
  int h0 = sh->mode == 0 ? hs : hs * G, h1 = sh->mode == 0 ? hs + 1 : (hs + 1) * G;
#pragma omp parallel for schedule(static)
  for (int j = 0; j < n; ++j) {
    if (j >= i) { out[j] = -INFINITY; continue; }
    int jf = j * B, jl = (j + 1) * B < L ? (j + 1) * B : L;
    double group = 0.0, kbar[1024];
    for (int h = h0; h < h1; ++h) {
      for (int d = 0; d < D; ++d) { /* mean of key block j, KV head h/G */
        double acc = 0.0;
        for (int u = jf; u < jl; ++u) acc += (double)K[((int64_t)(sh->cu[s] + u) * Hkv + h / G) * D + d];
        kbar[d] = acc / (double)(jl - jf);
      }
      double sum_logit = 0.0;
      for (int t = first; t < last; ++t) {
        const float *q = &Q[((int64_t)(sh->cu[s] + t) * Hq + h) * D];
        double logit = 0.0;
        for (int d = 0; d < D; ++d) logit += (double)q[d] * kbar[d];
        sum_logit += logit;
      }
      group += sum_logit / (double)(last - first);
    }
    out[j] = score_scale * group;
  }
  return 0;
}

/* Total order used by the selection: higher score first; -0 equals +0; NaN ranks below every
 * number including -infinity; among equals the lower block index first. */
static int ranks_before(float sa, int ja, float sb, int jb) {
  int na = isnan(sa), nb = isnan(sb);
  if (na != nb) return nb;              /* the non-NaN one goes first */
  if (!na && sa != sb) return sa > sb;  /* -0 == +0 compares equal here */
  return ja < jb;
}

/* Number of CSR entries before each row: c(s,i) = min(k_s, i+1), counted directly. */
int orc_sel_rowptr(const orc_shape *sh, const int32_t *topk, int32_t *rowptr) {
  int Hs = sel_heads(sh);
  int64_t NQB = total_qblocks(sh), pos = 0;
  for (int hs = 0; hs < Hs; ++hs)
    for (int s = 0; s < sh->S; ++s) {
      int n = nblocks(sh, s);
      int64_t qb0 = qb_offset(sh, s);
      for (int i = 0; i < n; ++i) {
        rowptr[hs * NQB + qb0 + i] = (int32_t)pos;
        int k = topk[s] < 1 ? 1 : topk[s];
        pos += (k < i + 1) ? k : i + 1;
      }
    }
  rowptr[(int64_t)Hs * NQB] = (int32_t)pos;
  return 0;
}

/* Top-K block selection (section 2.2).  For query block i of sequence s with budget k_s:
 * the diagonal block i is always kept and counts towards the budget; the other
 * c-1 = min(k_s, i+1)-1 blocks are the best of the past blocks j < i under the total order
 * above.  The kept indices are stored ascending.  The decision is taken on the float32
 * scores exactly as given. */
int orc_select_topk(const orc_shape *sh, const float *scores, const int32_t *topk, const int32_t *rowptr,
                    int32_t *idx) {
  int Hs = sel_heads(sh);
  int64_t NQB = total_qblocks(sh);
  for (int s = 0; s < sh->S; ++s) {
    int n = nblocks(sh, s);
    int64_t qb0 = qb_offset(sh, s), so = score_offset(sh, s);
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
    for (int hs = 0; hs < Hs; ++hs)
      for (int i = 0; i < n; ++i) {
        const float *row = &scores[so + ((int64_t)hs * n + i) * n];
        int k = topk[s] < 1 ? 1 : topk[s];
        int c = (k < i + 1) ? k : i + 1;
        int32_t *out = &idx[rowptr[hs * NQB + qb0 + i]];
        char *taken = (char *)calloc((size_t)(i > 0 ? i : 1), 1);
        for (int pick = 0; pick < c - 1; ++pick) { /* repeatedly take the best remaining candidate */
          int best = -1;
          for (int j = 0; j < i; ++j) {
            if (taken[j]) continue;
            if (best < 0 || ranks_before(row[j], j, row[best], best)) best = j;
          }
          taken[best] = 1;
        }
        int m = 0;
        for (int j = 0; j < i; ++j)
          if (taken[j]) out[m++] = j;
        out[m++] = i;
        free(taken);
      }
  }
  return 0;
}

/* ------------------------------------------------------------------------------------- */
/* Attention over the selected keys (Eq. 2).                                              */

typedef struct attn_ctx {
  const orc_shape *sh;
  const float *Q, *K, *V;
  const int32_t *rowptr, *idx;
  double scale;
  int64_t NQB;
  int64_t *qboff; /* [S+1] prefix sums of n_s */
} attn_ctx;

static int ctx_init(attn_ctx *c, const orc_shape *sh, const float *Q, const float *K, const float *V,
                    const int32_t *rowptr, const int32_t *idx, double scale) {
  c->sh = sh; c->Q = Q; c->K = K; c->V = V; c->rowptr = rowptr; c->idx = idx; c->scale = scale;
  c->NQB = total_qblocks(sh);
  c->qboff = (int64_t *)malloc(sizeof(int64_t) * (size_t)(sh->S + 1));
  if (!c->qboff) return -1;
  c->qboff[0] = 0;
  for (int s = 0; s < sh->S; ++s) c->qboff[s + 1] = c->qboff[s] + nblocks(sh, s);
  return 0;
}

/* Key set of query token r (local index in sequence s) for query head h: all tokens of the
 * selected blocks that are not in the future of r.  Past blocks lie wholly before r; the test
 * t <= r only cuts inside the diagonal block.  Returns the count, writes packed token rows. */
static int visible_keys(const attn_ctx *c, int s, int h, int r, int32_t *tok) {
  const orc_shape *sh = c->sh;
  int B = sh->B, L = sh->cu[s + 1] - sh->cu[s], i = r / B, n = 0;
  int64_t row = (int64_t)sel_head_of(sh, h) * c->NQB + c->qboff[s] + i;
  for (int32_t e = c->rowptr[row]; e < c->rowptr[row + 1]; ++e) {
    int j = c->idx[e];
    int first = j * B, last = (j + 1) * B < L ? (j + 1) * B : L;
    for (int t = first; t < last; ++t)
      if (t <= r) tok[n++] = sh->cu[s] + t;
  }
  return n;
}

/* One query row: p = softmax_j(scale * q.k_j) over its key set, o = sum_j p_j v_j,
 * lse = log sum_j exp(scale * q.k_j).  Returns the number of keys. */
static int row_forward(const attn_ctx *c, int s, int h, int r, int32_t *tok, double *p, double *o, double *lse) {
  const orc_shape *sh = c->sh;
  int D = sh->D, g = h / (sh->Hq / sh->Hkv);
  int n = visible_keys(c, s, h, r, tok);
  const float *q = &c->Q[((int64_t)(sh->cu[s] + r) * sh->Hq + h) * D];
  double m = -INFINITY;
  for (int a = 0; a < n; ++a) {
    const float *k = &c->K[((int64_t)tok[a] * sh->Hkv + g) * D];
    double dot = 0.0;
    for (int d = 0; d < D; ++d) dot += (double)q[d] * (double)k[d];
    p[a] = c->scale * dot;
    if (p[a] > m) m = p[a];
  }
  double l = 0.0;
  for (int a = 0; a < n; ++a) { p[a] = exp(p[a] - m); l += p[a]; }
  for (int d = 0; d < D; ++d) o[d] = 0.0;
  for (int a = 0; a < n; ++a) {
    p[a] /= l;
    const float *v = &c->V[((int64_t)tok[a] * sh->Hkv + g) * D];
    for (int d = 0; d < D; ++d) o[d] += p[a] * (double)v[d];
  }
  *lse = m + log(l);
  return n;
}

static int max_seq_len(const orc_shape *sh) {
  int m = 1;
  for (int s = 0; s < sh->S; ++s)
    if (sh->cu[s + 1] - sh->cu[s] > m) m = sh->cu[s + 1] - sh->cu[s];
  return m;
}

/* Forward for every (token, head).  O [T][Hq][D], LSE [Hq][T]. */
int orc_attn_fwd(const orc_shape *sh, const float *Q, const float *K, const float *V, const int32_t *rowptr,
                 const int32_t *idx, double scale, double *O, double *LSE) {
  attn_ctx c;
  if (ctx_init(&c, sh, Q, K, V, rowptr, idx, scale)) return -1;
  int maxL = max_seq_len(sh), D = sh->D;
  for (int s = 0; s < sh->S; ++s) {
    int L = sh->cu[s + 1] - sh->cu[s];
#pragma omp parallel
    {
      int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxL);
      double *p = (double *)malloc(sizeof(double) * (size_t)maxL);
#pragma omp for schedule(dynamic, 8) collapse(2)
      for (int h = 0; h < sh->Hq; ++h)
        for (int r = 0; r < L; ++r) {
          int64_t t = sh->cu[s] + r;
          row_forward(&c, s, h, r, tok, p, &O[(t * sh->Hq + h) * D], &LSE[(int64_t)h * sh->T + t]);
        }
      free(tok);
      free(p);
    }
  }
  free(c.qboff);
  return 0;
}

/* Gradient of one query row's output with respect to q (returned in dq) and to the keys and
 * values of its key set (accumulated into dKacc/dVacc through the caller's addressing):
 *   Dr = dO.o;  dP_j = dO.v_j;  dS_j = p_j (dP_j - Dr);
 *   dq = scale * sum_j dS_j k_j;  dk_j += scale * dS_j q;  dv_j += p_j dO.
 * The selection is held fixed (no gradient flows through the routing). */
typedef void (*kv_sink)(void *user, int32_t key_tok, int g, const double *dk_row, const double *dv_row);

static void row_backward(const attn_ctx *c, int s, int h, int r, const float *dO, int32_t *tok, double *p, double *dq,
                         kv_sink sink, void *user, double *tmpk, double *tmpv) {
  const orc_shape *sh = c->sh;
  int D = sh->D, g = h / (sh->Hq / sh->Hkv);
  double o[1024], lse;
  int n = row_forward(c, s, h, r, tok, p, o, &lse);
  int64_t t = sh->cu[s] + r;
  const float *q = &c->Q[(t * sh->Hq + h) * D];
  const float *go = &dO[(t * sh->Hq + h) * D];
  double Dr = 0.0;
  for (int d = 0; d < D; ++d) Dr += (double)go[d] * o[d];
  for (int d = 0; d < D; ++d) dq[d] = 0.0;
  for (int a = 0; a < n; ++a) {
    const float *k = &c->K[((int64_t)tok[a] * sh->Hkv + g) * D];
    const float *v = &c->V[((int64_t)tok[a] * sh->Hkv + g) * D];
    double dP = 0.0;
    for (int d = 0; d < D; ++d) dP += (double)go[d] * (double)v[d];
    double dS = p[a] * (dP - Dr);
    for (int d = 0; d < D; ++d) {
      dq[d] += c->scale * dS * (double)k[d];
      tmpk[d] = c->scale * dS * (double)q[d];
      tmpv[d] = p[a] * (double)go[d];
    }
    if (sink) sink(user, tok[a], g, tmpk, tmpv);
  }
}

typedef struct full_sink { double *dK, *dV; int Hkv, D; } full_sink;
static void sink_full(void *user, int32_t key_tok, int g, const double *dk, const double *dv) {
  full_sink *f = (full_sink *)user;
  double *a = &f->dK[((int64_t)key_tok * f->Hkv + g) * f->D], *b = &f->dV[((int64_t)key_tok * f->Hkv + g) * f->D];
  for (int d = 0; d < f->D; ++d) { a[d] += dk[d]; b[d] += dv[d]; }
}

/* Backward for everything.  dQ [T][Hq][D], dK/dV [T][Hkv][D]; dK/dV are summed over the query
 * heads of each KV group.  Parallel over (sequence, KV head) so that every thread owns the dK/dV
 * rows it adds to. */
int orc_attn_bwd(const orc_shape *sh, const float *Q, const float *K, const float *V, const float *dO,
                 const int32_t *rowptr, const int32_t *idx, double scale, double *dQ, double *dK, double *dV) {
  if (sh->D > 1024) return -2;
  attn_ctx c;
  if (ctx_init(&c, sh, Q, K, V, rowptr, idx, scale)) return -1;
  int maxL = max_seq_len(sh), D = sh->D, G = sh->Hq / sh->Hkv;
  memset(dK, 0, sizeof(double) * (size_t)sh->T * sh->Hkv * D);
  memset(dV, 0, sizeof(double) * (size_t)sh->T * sh->Hkv * D);
  full_sink fs = {dK, dV, sh->Hkv, D};
#pragma omp parallel
  {
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxL);
    double *p = (double *)malloc(sizeof(double) * (size_t)maxL);
    double *tk = (double *)malloc(sizeof(double) * (size_t)D), *tv = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1) collapse(2)
    for (int s = 0; s < sh->S; ++s)
      for (int g = 0; g < sh->Hkv; ++g) {
        int L = sh->cu[s + 1] - sh->cu[s];
        for (int h = g * G; h < (g + 1) * G; ++h)
          for (int r = 0; r < L; ++r) {
            int64_t t = sh->cu[s] + r;
            row_backward(&c, s, h, r, dO, tok, p, &dQ[(t * sh->Hq + h) * D], sink_full, &fs, tk, tv);
          }
      }
    free(tok); free(p); free(tk); free(tv);
  }
  free(c.qboff);
  return 0;
}

/* Sampled rows: for each sample a (packed token, query head) pair, the row's O, LSE and dQ.
 * O_out, dQ_out [n][D]; LSE_out [n].  dO may be NULL (then dQ_out is untouched). */
int orc_attn_rows(const orc_shape *sh, const float *Q, const float *K, const float *V, const float *dO,
                  const int32_t *rowptr, const int32_t *idx, double scale, int n, const int32_t *tokens,
                  const int32_t *heads, double *O_out, double *LSE_out, double *dQ_out) {
  if (sh->D > 1024) return -2;
  attn_ctx c;
  if (ctx_init(&c, sh, Q, K, V, rowptr, idx, scale)) return -1;
  int maxL = max_seq_len(sh), D = sh->D;
#pragma omp parallel
  {
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxL);
    double *p = (double *)malloc(sizeof(double) * (size_t)maxL);
    double *tk = (double *)malloc(sizeof(double) * (size_t)D), *tv = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
    for (int a = 0; a < n; ++a) {
      int s = 0;
      while (s + 1 < sh->S && tokens[a] >= sh->cu[s + 1]) ++s;
      int r = tokens[a] - sh->cu[s];
      row_forward(&c, s, heads[a], r, tok, p, &O_out[(int64_t)a * D], &LSE_out[a]);
      if (dO) row_backward(&c, s, heads[a], r, dO, tok, p, &dQ_out[(int64_t)a * D], NULL, NULL, tk, tv);
    }
    free(tok); free(p); free(tk); free(tv);
  }
  free(c.qboff);
  return 0;
}

/* dK and dV of ONE key block (sequence s, KV head g, block j): [B][D] each (rows past the
 * sequence end stay zero).  Every query row of the group's heads whose selection contains j
 * contributes; rows are visited per query block in parallel with a private accumulator that is
 * added up in block order afterwards. */
typedef struct blk_sink { double *dK, *dV; int D; int32_t first_tok, last_tok; } blk_sink;
static void sink_block(void *user, int32_t key_tok, int g, const double *dk, const double *dv) {
  (void)g;
  blk_sink *f = (blk_sink *)user;
  if (key_tok < f->first_tok || key_tok >= f->last_tok) return;
  double *a = &f->dK[(int64_t)(key_tok - f->first_tok) * f->D], *b = &f->dV[(int64_t)(key_tok - f->first_tok) * f->D];
  for (int d = 0; d < f->D; ++d) { a[d] += dk[d]; b[d] += dv[d]; }
}

int orc_attn_bwd_kvblock(const orc_shape *sh, const float *Q, const float *K, const float *V, const float *dO,
                         const int32_t *rowptr, const int32_t *idx, double scale, int s, int g, int j,
                         double *dK_out, double *dV_out) {
  if (sh->D > 1024) return -2;
  attn_ctx c;
  if (ctx_init(&c, sh, Q, K, V, rowptr, idx, scale)) return -1;
  int maxL = max_seq_len(sh), D = sh->D, B = sh->B, G = sh->Hq / sh->Hkv;
  int L = sh->cu[s + 1] - sh->cu[s], n = nblocks(sh, s);
  int64_t qb0 = qb_offset(sh, s);
  size_t blk = (size_t)B * D;
  double *part = (double *)calloc((size_t)n * 2 * blk, sizeof(double));
  if (!part) return -1;
#pragma omp parallel
  {
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)maxL);
    double *p = (double *)malloc(sizeof(double) * (size_t)maxL);
    double *tk = (double *)malloc(sizeof(double) * (size_t)D), *tv = (double *)malloc(sizeof(double) * (size_t)D);
    double dq[1024];
#pragma omp for schedule(dynamic, 1)
    for (int i = j; i < n; ++i) {
      blk_sink bs = {&part[(size_t)i * 2 * blk], &part[(size_t)i * 2 * blk + blk], D, sh->cu[s] + j * B,
                     sh->cu[s] + ((j + 1) * B < L ? (j + 1) * B : L)};
      for (int h = g * G; h < (g + 1) * G; ++h) {
        int64_t row = (int64_t)sel_head_of(sh, h) * c.NQB + qb0 + i;
        int has = 0;
        for (int32_t e = rowptr[row]; e < rowptr[row + 1]; ++e) has |= (idx[e] == j);
        if (!has) continue;
        int last = (i + 1) * B < L ? (i + 1) * B : L;
        for (int r = i * B; r < last; ++r) row_backward(&c, s, h, r, dO, tok, p, dq, sink_block, &bs, tk, tv);
      }
    }
    free(tok); free(p); free(tk); free(tv);
  }
  memset(dK_out, 0, sizeof(double) * blk);
  memset(dV_out, 0, sizeof(double) * blk);
  for (int i = j; i < n; ++i)
    for (size_t x = 0; x < blk; ++x) {
      dK_out[x] += part[(size_t)i * 2 * blk + x];
      dV_out[x] += part[(size_t)i * 2 * blk + blk + x];
    }
  free(part);
  free(c.qboff);
  return 0;
}

int orc_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
