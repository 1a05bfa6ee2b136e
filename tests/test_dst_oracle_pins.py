"""Pins of the budget-controller checker (oracle/dst_oracle.py) against things other than itself:
the invariants the paper states for the coverage curve (section 4.1, Eq. 4: the importance scores
sum to 1, C is a running sum of sorted scores), closed forms, brute force on tiny inputs, the case
split of Eq. 7 and the definition of Perf.align (section 4.2, Eq. 9).  CPU only."""
import itertools

import numpy as np
import pytest

from oracle import dst_oracle as dst


def flat_scores(blocks):
    """blocks: list of [Hs][n][n] arrays -> (flat, score_off, nblk)"""
    off, flat = [0], []
    for b in blocks:
        flat.append(np.asarray(b, dtype=np.float64).ravel())
        off.append(off[-1] + b.size)
    return np.concatenate(flat), off, [b.shape[1] for b in blocks]


def test_coverage_is_monotone_ends_at_one_and_first_point_is_known():
    rng = np.random.default_rng(0)
    blocks = [rng.normal(size=(3, 7, 7)), rng.normal(size=(3, 1, 1)), rng.normal(size=(3, 12, 12)) * 4.0]
    flat, off, nblk = flat_scores(blocks)
    cov = dst.coverage_curves(nblk, 3, flat, off)
    qb = np.concatenate([[0], np.cumsum(nblk)])
    for s, n in enumerate(nblk):
        C = cov[qb[s]: qb[s] + n]
        assert np.all(np.diff(C) >= -1e-15)
        assert abs(C[-1] - 1.0) < 1e-12           # the importance scores of every row sum to 1
        assert abs(C[0] - 1.0 / n) < 1e-12        # budget 1 keeps the diagonal only: just the first block's row is fully covered


def test_equal_logits_give_the_uniform_closed_form():
    # every candidate equally important: a row with i candidates covers min(k-1, i)/i at budget k
    n, Hs = 9, 2
    flat, off, nblk = flat_scores([np.full((Hs, n, n), 0.37)])
    C = dst.coverage_curves(nblk, Hs, flat, off)
    ref = np.array([(1.0 + sum(min(k - 1, i) / i for i in range(1, n))) / n for k in range(1, n + 1)])
    assert np.allclose(C, ref, atol=1e-13)


def test_one_dominant_block_is_covered_by_budget_two():
    # block 0 carries (almost) all the mass of every row: budget 2 (diagonal + best candidate) covers ~everything
    n, Hs = 8, 1
    b = np.zeros((Hs, n, n)); b[:, :, 0] = 50.0
    flat, off, nblk = flat_scores([b])
    C = dst.coverage_curves(nblk, Hs, flat, off)
    assert C[1] > 1.0 - 1e-12 and C[0] == pytest.approx(1.0 / n)


def test_coverage_against_brute_force_over_subsets():
    # the best coverage any choice of k-1 candidates can reach is the sum of the k-1 largest shares
    rng = np.random.default_rng(3)
    n, Hs = 6, 2
    b = rng.normal(size=(Hs, n, n)) * 2.0
    flat, off, nblk = flat_scores([b])
    C = dst.coverage_curves(nblk, Hs, flat, off)
    for k in range(1, n + 1):
        tot = 0.0
        for hs in range(Hs):
            for i in range(n):
                if i == 0:
                    tot += 1.0
                    continue
                e = np.exp(b[hs, i, :i]); r = e / e.sum()
                m = min(k - 1, i)
                tot += max((sum(r[list(c)]) for c in itertools.combinations(range(i), m)), default=0.0)
        assert C[k - 1] == pytest.approx(tot / (Hs * n), abs=1e-12)


def test_coverage_is_invariant_to_a_shift_of_the_logits_and_to_the_order_of_candidates():
    rng = np.random.default_rng(4)
    n, Hs = 10, 2
    b = rng.normal(size=(Hs, n, n))
    flat, off, nblk = flat_scores([b])
    C = dst.coverage_curves(nblk, Hs, flat, off)
    b2 = b + 3.25
    for i in range(n):
        b2[:, i, :i] = b2[:, i, :i][:, ::-1]
    flat2, _, _ = flat_scores([b2])
    assert np.allclose(C, dst.coverage_curves(nblk, Hs, flat2, off), atol=1e-13)


XS, KS = [1024.0, 4096.0, 16384.0], [4.0, 16.0, 64.0]
TAB = np.array([[1.0, 2.0, 5.0], [3.0, 6.0, 15.0], [10.0, 20.0, 50.0]])


def test_perf_predict_hits_the_table_and_interpolates():
    for a, x in enumerate(XS):
        for b, k in enumerate(KS):
            assert dst.perf_predict(XS, KS, TAB, x, k) == TAB[a, b]
    assert dst.perf_predict(XS, KS, TAB, 2560.0, 4.0) == pytest.approx(2.0)       # halfway between 1 and 3
    assert dst.perf_predict(XS, KS, TAB, 1024.0, 10.0) == pytest.approx(1.5)      # halfway between 1 and 2
    assert dst.perf_predict(XS, KS, TAB, 100.0, 1.0) == 1.0                       # clamped at the edges
    assert dst.perf_predict(XS, KS, TAB, 1e6, 1e3) == 50.0


def test_perf_align_is_the_largest_budget_within_the_target():
    for x, T in ((1024.0, 1.7), (5000.0, 9.0), (16384.0, 9.0), (16384.0, 1e9)):
        k = dst.perf_align(XS, KS, TAB, x, T, 100)
        ok = [kk for kk in range(1, 101) if dst.perf_predict(XS, KS, TAB, x, kk) <= T]
        assert k == (max(ok) if ok else 1)
    assert dst.perf_align(XS, KS, TAB, 16384.0, 9.0, 100) == 1     # nothing fits: budget 1


def _toy(nblk, Hs=2, seed=5):
    rng = np.random.default_rng(seed)
    flat, off, _ = flat_scores([rng.normal(size=(Hs, n, n)) * 3.0 for n in nblk])
    qb = np.concatenate([[0], np.cumsum(nblk)]).astype(int)
    return dst.coverage_curves(nblk, Hs, flat, off), qb


def test_dst_case_split_of_the_final_budget():
    nblk = [16, 64, 256]
    lens = [n * 64 for n in nblk]
    kbase = [8, 16, 32]
    cov, qb = _toy(nblk)
    for anchor in (dst.ANCHOR_MIN, dst.ANCHOR_MEAN, dst.ANCHOR_MAX):
        for p in (0.0, 0.05, 0.3, 1.0):
            kf, ka, Ta = dst.dst_budgets(p, anchor, lens, nblk, kbase, cov, qb, XS, KS, TAB)
            T = [dst.perf_predict(XS, KS, TAB, lens[s], kbase[s]) for s in range(3)]
            assert Ta == pytest.approx({0: min(T), 1: sum(T) / 3, 2: max(T)}[anchor])
            for s in range(3):
                C = cov[qb[s]: qb[s] + nblk[s]]
                assert 1 <= kf[s] <= nblk[s]
                if T[s] <= Ta:                                  # not a bottleneck: the anchor budget, never below the base
                    assert kf[s] == ka[s] >= kbase[s] or ka[s] == nblk[s]
                else:                                           # bottleneck: compressed, but never past the coverage bound
                    assert kf[s] <= kbase[s]
                    assert C[kbase[s] - 1] - C[kf[s] - 1] <= p + 1e-15
                    assert kf[s] >= ka[s]
                    if kf[s] > ka[s]:                           # the bound was binding: one block fewer would break it
                        assert kf[s] == 1 or C[kbase[s] - 1] - C[kf[s] - 2] > p
    # p = 1 never binds: every sequence lands on its anchor budget; the max anchor never compresses
    kf, ka, _ = dst.dst_budgets(1.0, dst.ANCHOR_MEAN, lens, nblk, kbase, cov, qb, XS, KS, TAB)
    assert np.array_equal(kf, ka)
    kf, _, _ = dst.dst_budgets(0.0, dst.ANCHOR_MAX, lens, nblk, kbase, cov, qb, XS, KS, TAB)
    assert np.all(kf >= np.array(kbase))
    # p = 0 with a strictly increasing curve keeps bottlenecks at their base budget
    kf, _, _ = dst.dst_budgets(0.0, dst.ANCHOR_MIN, lens, nblk, kbase, cov, qb, XS, KS, TAB)
    assert kf[2] == kbase[2]
