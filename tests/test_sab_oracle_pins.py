"""Pins of the batching checker (oracle/sab_oracle.py): what a partition must satisfy, the classical
guarantee of the longest-first greedy against the brute-force optimum on tiny inputs, closed forms
of the moving average, and the imbalance measure of Eq. 11.  CPU only."""
import itertools

import numpy as np
import pytest

from oracle import sab_oracle as sab


def _opt_makespan(w, m):
    best = float("inf")
    for assign in itertools.product(range(m), repeat=len(w)):
        load = [0.0] * m
        for x, b in zip(w, assign):
            load[b] += x
        best = min(best, max(load))
    return best


@pytest.mark.parametrize("seed", range(6))
def test_partition_is_valid_and_within_the_greedy_bound(seed):
    rng = np.random.default_rng(seed)
    n, m = int(rng.integers(3, 9)), int(rng.integers(2, 4))
    w = rng.uniform(0.1, 10.0, size=n)
    b = sab.balanced_partition(w, m)
    assert b.shape == (n,) and b.min() >= 0 and b.max() < m        # every sample in exactly one bin
    load = np.bincount(b, weights=w, minlength=m)
    assert load.max() <= (4.0 / 3.0 - 1.0 / (3.0 * m)) * _opt_makespan(w, m) + 1e-12   # Graham's bound for longest-first


def test_partition_closed_forms():
    assert np.bincount(sab.balanced_partition([1.0] * 10, 4), minlength=4).tolist() == [3, 3, 2, 2]   # equal weights: sizes differ by <= 1, low bins first
    assert sab.balanced_partition([5.0, 1.0, 1.0, 1.0, 1.0, 1.0], 2).tolist() == [0, 1, 1, 1, 1, 1]    # the heavy sample alone
    assert sab.balanced_partition([2.0, 7.0, 7.0], 3).tolist() == [2, 0, 1]                            # ties: lower index first, lower bin first
    assert sab.balanced_partition([], 3).shape == (0,)


def test_two_level_partition_and_imbalance():
    rng = np.random.default_rng(1)
    w = rng.uniform(1.0, 50.0, size=64)
    for rank in range(4):
        dp, mb = sab.sab_batches(w, 4, rank, 4)
        assert np.array_equal(dp, sab.balanced_partition(w, 4))
        assert np.all((mb >= 0) == (dp == rank)) and mb.max() < 4
    assert sab.imbalance([1.0, 1.0, 2.0], [0, 1, 2], 3) == pytest.approx(2.0 / (4.0 / 3.0))   # Eq. 11: max over mean
    assert sab.imbalance(w, sab.balanced_partition(w, 4), 4) < 1.05 < sab.imbalance(w, np.arange(64) // 16, 4) + 0.05


def test_moving_average_closed_forms():
    edges = [0, 4096, 16384, 1 << 30]
    ema, seen = sab.spar_update([0, 0, 0], [False] * 3, edges, 0.5, [100, 5000, 6000, 7000], [8, 32, 16, 16])
    assert seen.tolist() == [True, True, False]
    assert ema[0] == 8.0 and ema[1] == 0.5 * (0.5 * 32 + 0.5 * 16) + 0.5 * 16                # first sample initialises, then decays
    assert sab.spar_predict(ema, seen, edges, 20000, 24) == 24.0                             # unseen bin: the base budget
    assert sab.spar_predict(ema, seen, edges, 4096, 24) == ema[1] and sab.length_bin(edges, -5) == 0
    # a constant budget is a fixed point for every decay
    e2, _ = sab.spar_update(ema, seen, edges, 0.9, [100] * 5, [8] * 5)
    assert e2[0] == 8.0
