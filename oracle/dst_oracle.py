"""CPU checker for the budget controller around the attention path (test infrastructure only):
coverage curves of the routing scores, the profiled latency table, and the dynamic sparsity tuning
rule.  Plain numpy in float64; nothing here is shared with or imported by the GPU library.

What each function follows (SparseBalance paper, arXiv 2604.13847):
  coverage_curves   section 4.1, Eq. 4: routing logits normalised and sorted into importance scores
                    r_1 >= r_2 >= ... with sum 1, C(k) = sum of the k largest.
  perf_predict      section 4.2, Eq. 8 and Eq. 10: look-up in the profiled table M[x, k], with
                    interpolation between neighbouring buckets.
  perf_align        section 4.2, Eq. 9: the largest budget whose predicted latency does not exceed
                    the target.
  dst_budgets       section 4.1, Eq. 3, 5, 7 and Algorithm 1.

Readings taken where the paper is silent (each one is also listed in the design notes):
  * A "micro-batch" is one packed sequence: every sequence carries its own budget.
  * The routing logits of a sequence are its block scores.  For one query block i and one selection
    head the candidates are the strictly earlier blocks j < i (the diagonal block is always kept and
    has no logit); "normalise" is a softmax over the candidates; a budget k keeps the diagonal block
    plus the k-1 best candidates, so the row's coverage is the sum of its min(k-1, i) largest
    normalised scores (1 when that is all of them, also 1 for the first block, which has no
    candidates).  The sequence's curve C(k), k = 1..n, is the mean of the rows' coverages over all
    query blocks and selection heads.
  * FindFeasibleK: when moving from the base budget to the anchor budget would lose more than p of
    coverage, the budget becomes the smallest k with C(k_base) - C(k) <= p (Algorithm 1 passes only
    the curve, the base budget and p to it; the set of Eq. 6 would be empty in that case because C
    is monotone).
  * Budgets are integers in 1..n; the table is interpolated linearly in both the length and the
    budget and clamped at its edges; Perf.align returns 1 when even budget 1 is predicted slower
    than the target.
"""
from __future__ import annotations

import numpy as np


def coverage_curves(nblk, Hs, scores, score_off):
    """scores: flat array, per sequence a dense [Hs][n][n] block at score_off[s] (entries j >= i unused).
    Returns a flat float64 array with C_s(k) at qb_off[s] + k - 1, k = 1..n_s."""
    out = []
    for s, n in enumerate(nblk):
        C = np.zeros(n, dtype=np.float64)
        if n == 0:
            continue
        blk = np.asarray(scores[score_off[s]: score_off[s] + Hs * n * n], dtype=np.float64).reshape(Hs, n, n)
        for hs in range(Hs):
            for i in range(n):
                if i == 0:
                    C += 1.0
                    continue
                cand = blk[hs, i, :i]
                e = np.exp(cand - cand.max())
                r = np.sort(e / e.sum())[::-1]
                pref = np.concatenate([[0.0], np.cumsum(r)])
                pref[i] = 1.0                      # all candidates kept: exactly everything
                k = np.arange(1, n + 1)
                C += pref[np.minimum(k - 1, i)]
        out.append(C / (Hs * n))
    return np.concatenate(out) if out else np.zeros(0)


def _bracket(grid, v):
    """Index a and weight w such that v ~ (1-w)*grid[a] + w*grid[a+1], clamped to the grid."""
    grid = np.asarray(grid, dtype=np.float64)
    if len(grid) == 1 or v <= grid[0]:
        return 0, 0.0
    if v >= grid[-1]:
        return len(grid) - 2, 1.0
    a = int(np.searchsorted(grid, v, side="right") - 1)
    return a, (v - grid[a]) / (grid[a + 1] - grid[a])


def perf_predict(xs, ks, M, x, k):
    """Bilinear interpolation of the table M[len(xs)][len(ks)] at (length x, budget k)."""
    M = np.asarray(M, dtype=np.float64).reshape(len(xs), len(ks))
    a, wa = _bracket(xs, float(x))
    b, wb = _bracket(ks, float(k))
    a2, b2 = min(a + 1, len(xs) - 1), min(b + 1, len(ks) - 1)
    lo = (1.0 - wb) * M[a, b] + wb * M[a, b2]
    hi = (1.0 - wb) * M[a2, b] + wb * M[a2, b2]
    return (1.0 - wa) * lo + wa * hi


def perf_align(xs, ks, M, x, target, kmax):
    """Largest integer budget in 1..kmax whose predicted latency is <= target (1 if none is)."""
    best = 1
    for k in range(1, kmax + 1):
        if perf_predict(xs, ks, M, x, k) <= target:
            best = k
    return best


ANCHOR_MIN, ANCHOR_MEAN, ANCHOR_MAX = 0, 1, 2


def dst_budgets(p, anchor, lens, nblk, k_base, cov, qb_off, xs, ks, M):
    """Algorithm 1 for every sequence of the batch.  Returns (k_final, k_anchor, T_anchor)."""
    S = len(lens)
    kb = [min(max(int(k_base[s]), 1), max(nblk[s], 1)) for s in range(S)]
    live = [s for s in range(S) if nblk[s] > 0]
    T = [perf_predict(xs, ks, M, lens[s], kb[s]) for s in live]
    if not live:
        return np.array(kb, dtype=np.int32), np.array(kb, dtype=np.int32), 0.0
    T_anchor = {ANCHOR_MIN: min(T), ANCHOR_MEAN: sum(T) / len(T), ANCHOR_MAX: max(T)}[anchor]
    k_final, k_anchor = list(kb), list(kb)
    for s in live:
        n = nblk[s]
        C = cov[qb_off[s]: qb_off[s] + n]
        ka = perf_align(xs, ks, M, lens[s], T_anchor, n)
        k_anchor[s] = ka
        kf = ka
        if C[kb[s] - 1] - C[ka - 1] > p:
            kf = next(k for k in range(1, n + 1) if C[kb[s] - 1] - C[k - 1] <= p)
        k_final[s] = kf
    return np.array(k_final, dtype=np.int32), np.array(k_anchor, dtype=np.int32), T_anchor
