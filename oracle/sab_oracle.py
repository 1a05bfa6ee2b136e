"""CPU checker for sparsity-aware batching (test infrastructure only; paper section 4.3, Algorithm 2).
Plain Python/numpy, float64; shares nothing with the library.

  spar_update / spar_predict   the sparsity predictor Spar: per sequence-length bin, an exponential
                               moving average of the final budgets the tuning step produced; before a
                               bin has seen any sample it predicts the base budget.
  sab_weights                  W[i] = Perf.predict(L[i], Spar.predict(L[i]))  (Algorithm 2, first loop)
  balanced_partition           `bin_packing`: the paper only says "a standard balanced partition
                               solver"; reading: longest-processing-time-first greedy - samples in
                               order of decreasing weight (ties: lower index first), each to the bin
                               with the smallest load so far (ties: lower bin first).  Bin sizes are
                               not constrained.
  sab_batches                  the two-level partition: first over the DP ranks, then the rank's
                               samples over its gbs/(mbs*N) micro-batches.
  imbalance                    max / mean of the bin loads (paper Eq. 11).
"""
from __future__ import annotations

import numpy as np

from .dst_oracle import perf_predict


def length_bin(edges, L):
    """Bin b with edges[b] <= L < edges[b+1]; lengths outside fall into the first / last bin."""
    nb = len(edges) - 1
    b = int(np.searchsorted(np.asarray(edges, dtype=np.float64), float(L), side="right") - 1)
    return min(max(b, 0), nb - 1)


def spar_update(ema, seen, edges, decay, lengths, k_final):
    """One calibration step: ema[b] <- decay*ema[b] + (1-decay)*k for every sample, in order; the first
    sample of a bin initialises it."""
    ema, seen = np.array(ema, dtype=np.float64), np.array(seen, dtype=bool)
    for L, k in zip(lengths, k_final):
        b = length_bin(edges, L)
        ema[b] = float(k) if not seen[b] else decay * ema[b] + (1.0 - decay) * float(k)
        seen[b] = True
    return ema, seen


def spar_predict(ema, seen, edges, L, k_base):
    b = length_bin(edges, L)
    return float(ema[b]) if seen[b] else float(k_base)


def sab_weights(xs, ks, M, lengths, k_pred):
    return np.array([perf_predict(xs, ks, M, L, k) for L, k in zip(lengths, k_pred)], dtype=np.float64)


def balanced_partition(w, nbins):
    w = np.asarray(w, dtype=np.float64)
    order = sorted(range(len(w)), key=lambda i: (-w[i], i))
    load = [0.0] * nbins
    bin_of = np.full(len(w), -1, dtype=np.int32)
    for i in order:
        b = min(range(nbins), key=lambda j: (load[j], j))
        bin_of[i] = b
        load[b] += w[i]
    return bin_of


def sab_batches(w, dp_size, dp_rank, num_microbatches):
    """(dp_bin_of[n], mb_bin_of[n]); mb_bin_of is -1 for the samples of other ranks."""
    dp_of = balanced_partition(w, dp_size)
    mine = [i for i in range(len(w)) if dp_of[i] == dp_rank]
    mb_of = np.full(len(w), -1, dtype=np.int32)
    local = balanced_partition([w[i] for i in mine], num_microbatches)
    for j, i in enumerate(mine):
        mb_of[i] = local[j]
    return dp_of, mb_of


def imbalance(w, bin_of, nbins):
    load = np.zeros(nbins)
    for i, b in enumerate(bin_of):
        if b >= 0:
            load[b] += w[i]
    return float(load.max() / load.mean()) if load.mean() > 0 else 1.0
