"""Pins of the CPU checker (oracle/) against things other than itself: a hand-worked instance
of Eq. 2, dense causal attention (Eq. 1), brute-force masked softmax, closed forms, invariants
and finite differences.  CPU only."""
import os

import numpy as np
import pytest

import bruteforce as bf
from oracle import oracle as orc
from paper_2604_13847_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def rnd(seed, tid, shape):
    return synth.normal_f32(seed, tid, int(np.prod(shape))).reshape(shape)


def make(lens, Hq, Hkv, D, B, mode, seed=0):
    cu = synth.cu_from_lengths(lens)
    pb = orc.Problem(cu, Hq, Hkv, D, B, mode)
    T = pb.T
    Q, K, V, dO = (rnd(seed, t, s) for t, s in ((1, (T, Hq, D)), (2, (T, Hkv, D)), (3, (T, Hkv, D)), (4, (T, Hq, D))))
    return pb, Q, K, V, dO


def select(pb, Q, K, topk, score_scale=1.0):
    sc = orc.block_scores(pb, Q, K, score_scale).astype(np.float32)
    return orc.select_topk(pb, sc, topk)


def head_masks(pb, rowptr, idx):
    G = pb.Hq // pb.Hkv
    per_sel = [bf.mask_from_selection(pb.cu, pb.B, pb.NQB, rowptr, idx, hs) for hs in range(pb.Hs)]
    return [per_sel[h if pb.mode == 0 else h // G] for h in range(pb.Hq)]


# ---------------------------------------------------------------- budget rule
def test_keep_ratio_rule_values():
    cu = np.array([0, 640, 640 + 65, 640 + 65 + 1000, 640 + 65 + 1000 + 3], dtype=np.int32)  # n = 10, 2, 16, 1
    k = orc.keep_ratio_to_topk(cu, 64, np.array([0.1, 0.5, 0.26, 0.9], dtype=np.float32))
    assert k.tolist() == [1, 1, 5, 1]          # 0.1f*10 is 1.0000000149 -> 1, not 2; ceil(4.16)=5
    k = orc.keep_ratio_to_topk(cu, 64, np.array([0.0, 1.0, 2.0, 0.0], dtype=np.float32))
    assert k.tolist() == [1, 2, 16, 1]         # clamped to [1, n]
    k = orc.keep_ratio_to_topk(cu, 64, np.array([0.11, 0.51, 0.3125, 1.0], dtype=np.float32))
    assert k.tolist() == [2, 2, 5, 1]


def test_rowptr_counts_closed_form():
    lens = [1000, 64, 130, 5]
    for mode in (0, 1):
        pb = orc.Problem(synth.cu_from_lengths(lens), 4, 2, 8, 64, mode)
        topk = np.array([5, 3, 2, 7], dtype=np.int32)
        rp = orc.sel_rowptr(pb, topk)
        per_head = sum(min(k, n) * n - min(k, n) * (min(k, n) - 1) // 2 for k, n in zip(topk, pb.nblk))
        assert rp[-1] == pb.Hs * per_head
        assert np.all(np.diff(rp) >= 1)


# ---------------------------------------------------------------- scores
@pytest.mark.parametrize("mode", [0, 1])
def test_scores_equal_pooled_dot(mode):
    pb, Q, K, _, _ = make([200, 64, 1, 130, 65], 4, 2, 16, 64, mode, seed=3)
    got = orc.block_scores(pb, Q, K, 0.37)
    want = bf.pooled_scores(pb.cu, pb.B, Q, K, 0.37, mode == 1)
    for s, n in enumerate(pb.nblk):
        g = got[pb.score_off[s]:pb.score_off[s + 1]].reshape(pb.Hs, n, n)
        w = want[s]
        assert np.array_equal(np.isneginf(g), np.isneginf(w))
        fin = np.isfinite(w)
        np.testing.assert_allclose(g[fin], w[fin], rtol=1e-11, atol=1e-12)
        for hs in range(pb.Hs):                      # the single-row entry point agrees
            for i in range(n):
                np.testing.assert_allclose(orc.block_scores_row(pb, Q, K, 0.37, s, hs, i), g[hs, i], rtol=1e-12)


def test_scores_constant_keys_and_tail_divisor():
    # K == const vector c  =>  score = scale * <mean Q, c> for every past block, also for a 1-token tail block
    B, D = 64, 8
    pb, Q, K, _, _ = make([B + 1 + B], 2, 2, D, B, 0, seed=5)      # n = 3, last block has 1 token
    c = np.linspace(-1, 1, D).astype(np.float32)
    K[:] = c
    got = orc.block_scores(pb, Q, K, 2.0).reshape(2, 3, 3)
    for h in range(2):
        for i in range(3):
            rows = slice(i * B, min((i + 1) * B, pb.T))
            want = 2.0 * float(Q[rows, h].astype(np.float64).mean(axis=0) @ c.astype(np.float64))
            for j in range(i):
                assert abs(got[h, i, j] - want) < 1e-12
    # tail divisor: make the 1-token tail KEY block huge; its mean must be the token itself, not token/B
    pb2, Q2, K2, _, _ = make([B + 1 + 2 * B], 1, 1, D, B, 0, seed=6)
    # blocks: [0,64) [64,128) [128,192) [192,193): the tail is block 3 and is never a past block; use block means
    km = orc.block_mean(pb2, K2)
    np.testing.assert_allclose(km[3, 0], K2[192, 0].astype(np.float64), rtol=0, atol=0)
    np.testing.assert_allclose(km[1, 0], K2[64:128, 0].astype(np.float64).mean(axis=0), rtol=1e-13)


# ---------------------------------------------------------------- selection
def test_select_all_equal_scores_takes_lowest_indices():
    pb = orc.Problem(synth.cu_from_lengths([64 * 9]), 1, 1, 4, 64, 0)
    sc = np.full(81, 0.25, dtype=np.float32)
    rp, idx = orc.select_topk(pb, sc, [4])
    for i in range(9):
        c = min(4, i + 1)
        assert idx[rp[i]:rp[i + 1]].tolist() == list(range(c - 1)) + [i]


def test_select_matches_full_sort_with_ties_nan_zero():
    rng = np.random.default_rng(7)
    lens = [64 * 23, 64 * 5 + 3]
    for mode in (0, 1):
        pb = orc.Problem(synth.cu_from_lengths(lens), 4, 2, 4, 64, mode)
        sc = rng.integers(-3, 4, size=int(pb.score_off[-1])).astype(np.float32)   # many exact ties
        sc[rng.random(sc.size) < 0.05] = np.nan
        sc[rng.random(sc.size) < 0.05] = -np.inf
        sc[rng.random(sc.size) < 0.05] = -0.0
        sc[rng.random(sc.size) < 0.05] = 0.0
        sc[rng.random(sc.size) < 0.03] = np.inf
        topk = [6, 2]
        rp, idx = orc.select_topk(pb, sc, topk)
        for s, n in enumerate(pb.nblk):
            blk = sc[pb.score_off[s]:pb.score_off[s + 1]].reshape(pb.Hs, n, n)
            for hs in range(pb.Hs):
                for i in range(n):
                    row = hs * pb.NQB + pb.qb_off[s] + i
                    got = idx[rp[row]:rp[row + 1]].tolist()
                    assert got == bf.sort_select(blk[hs, i], i, min(topk[s], i + 1)), (mode, s, hs, i)
                    assert got[-1] == i and all(a < b for a, b in zip(got, got[1:]))


def test_select_invariant_under_monotone_transform_and_planted_block():
    pb, Q, K, _, _ = make([64 * 12], 2, 1, 16, 64, 0, seed=9)
    # plant: key block 5 = 10 * (mean query direction of head 0, block 9)
    qdir = Q[9 * 64:10 * 64, 0].mean(axis=0)
    K[5 * 64:6 * 64, 0] = 10 * qdir
    sc = orc.block_scores(pb, Q, K, 1.0).astype(np.float32)
    rp, idx = orc.select_topk(pb, sc, [3])
    assert 5 in idx[rp[9]:rp[10]].tolist()
    sc2 = np.where(np.isfinite(sc), np.float32(3.0) * sc + np.float32(1.0), sc)
    sc3 = np.where(np.isfinite(sc), np.exp(sc.astype(np.float64) * 0.1).astype(np.float32), np.float32(-np.inf))
    assert np.unique(sc3[np.isfinite(sc3)]).size == np.unique(sc[np.isfinite(sc)]).size  # transform stayed injective
    for other in (sc2, sc3):
        rp2, idx2 = orc.select_topk(pb, other, [3])
        assert np.array_equal(rp, rp2) and np.array_equal(idx, idx2)


# ---------------------------------------------------------------- forward
def test_hand_worked_instance_of_eq2():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "hand_worked_eq2.txt")) if l.strip() and l[0] != "#"]
    pb = orc.Problem(np.array([0, 4], dtype=np.int32), 1, 1, 1, 2, 0)
    ln3 = np.float32(np.log(3.0))
    Q = np.ones((4, 1, 1), dtype=np.float32)
    K = np.array([0, ln3, 0, ln3], dtype=np.float32).reshape(4, 1, 1)
    V = np.array([1, 5, 2, 10], dtype=np.float32).reshape(4, 1, 1)
    for budget in (1, 2):
        sc = orc.block_scores(pb, Q, K, 1.0).astype(np.float32)
        rp, idx = orc.select_topk(pb, sc, [budget])
        O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, 1.0)
        for b, t, o, lse in rows:
            if int(b) == budget:
                assert abs(O[int(t), 0, 0] - float(o)) < 1e-6 and abs(LSE[0, int(t)] - float(lse)) < 1e-6


@pytest.mark.parametrize("mode", [0, 1])
def test_full_budget_is_dense_causal_attention(mode):
    pb, Q, K, V, dO = make([150, 64, 1, 70], 4, 2, 8, 16, mode, seed=11)
    rp, idx = select(pb, Q, K, pb.nblk)                     # k_s = n_s
    scale = 1.0 / np.sqrt(pb.D)
    dense = [bf.causal_same_sequence_mask(pb.cu)] * pb.Hq    # no selection involved at all
    O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, scale)
    Ow, LSEw, _ = bf.masked_attention(Q, K, V, dense, scale)
    np.testing.assert_allclose(O, Ow, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(LSE, LSEw, rtol=1e-10, atol=1e-12)
    dQ, dK, dV = orc.attn_bwd(pb, Q, K, V, dO, rp, idx, scale)
    dQw, dKw, dVw = bf.masked_attention_grads(Q, K, V, dO, dense, scale)
    for a, b in ((dQ, dQw), (dK, dKw), (dV, dVw)):
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("B,D,lens,Hq,Hkv,mode,topk", [
    (4, 4, [37, 4, 1, 18], 2, 1, 0, [3, 1, 1, 2]),
    (8, 64, [100, 9], 4, 2, 0, [4, 2]),
    (8, 64, [100, 9], 4, 2, 1, [4, 2]),
    (64, 4, [200], 3, 1, 1, [2]),
    (64, 64, [200, 65], 2, 2, 0, [3, 1]),
    (128, 64, [300, 130, 128], 2, 1, 0, [2, 1, 1]),     # selection blocks larger than the kernels' 64-row tiles
    (256, 16, [700, 257], 4, 2, 1, [2, 2]),
])
def test_sparse_matches_bruteforce_mask(B, D, lens, Hq, Hkv, mode, topk):
    pb, Q, K, V, dO = make(lens, Hq, Hkv, D, B, mode, seed=13)
    rp, idx = select(pb, Q, K, topk)
    scale = 0.3
    masks = head_masks(pb, rp, idx)
    O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, scale)
    Ow, LSEw, Ps = bf.masked_attention(Q, K, V, masks, scale)
    np.testing.assert_allclose(O, Ow, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(LSE, LSEw, rtol=1e-10, atol=1e-12)
    # exp(scale*S - LSE) sums to 1 over each row's visible keys (LSE from the checker, S from numpy)
    G = Hq // Hkv
    for h in range(Hq):
        S = scale * (Q[:, h].astype(np.float64) @ K[:, h // G].astype(np.float64).T)
        P = np.where(masks[h], np.exp(S - LSE[h][:, None]), 0.0)
        np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=1e-10)
    dQ, dK, dV = orc.attn_bwd(pb, Q, K, V, dO, rp, idx, scale)
    dQw, dKw, dVw = bf.masked_attention_grads(Q, K, V, dO, masks, scale)
    for a, b in ((dQ, dQw), (dK, dKw), (dV, dVw)):
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)
    # dO == const  =>  dV_j = const * column sums of P
    ones = np.full_like(dO, 0.5)
    _, _, dV1 = orc.attn_bwd(pb, Q, K, V, ones, rp, idx, scale)
    for g in range(Hkv):
        col = sum(Ps[h].sum(axis=0) for h in range(g * G, (g + 1) * G))
        np.testing.assert_allclose(dV1[:, g, :], 0.5 * col[:, None] * np.ones(D), rtol=1e-10, atol=1e-12)


def test_constant_v_gives_constant_o_and_identical_keys_give_mean_v():
    pb, Q, K, V, _ = make([300, 70], 2, 1, 8, 64, 0, seed=17)
    rp, idx = select(pb, Q, K, [2, 2])
    Vc = np.broadcast_to(np.linspace(1, 2, 8).astype(np.float32), V.shape).copy()
    O, _ = orc.attn_fwd(pb, Q, K, Vc, rp, idx, 0.5)
    np.testing.assert_allclose(O, np.broadcast_to(np.linspace(1, 2, 8).astype(np.float32), O.shape), rtol=1e-12)
    Kc = np.broadcast_to(K[0, 0], K.shape).copy()           # all keys identical -> uniform weights
    rp2, idx2 = select(pb, Q, Kc, [2, 2])                   # all-equal scores: lowest indices + diagonal
    O2, LSE2 = orc.attn_fwd(pb, Q, Kc, V, rp2, idx2, 0.5)
    masks = head_masks(pb, rp2, idx2)
    for h in range(2):
        for r in (0, 63, 64, 200, 299, 300, 369):
            vis = masks[h][r]
            np.testing.assert_allclose(O2[r, h], V[vis, 0].astype(np.float64).mean(axis=0), rtol=1e-11, atol=1e-13)
            want_lse = np.log(vis.sum()) + 0.5 * float(Q[r, h].astype(np.float64) @ K[0, 0].astype(np.float64))
            assert abs(LSE2[h, r] - want_lse) < 1e-10


def test_budget_one_is_block_local_causal_attention():
    pb, Q, K, V, _ = make([130, 64], 2, 2, 8, 64, 0, seed=19)
    rp, idx = select(pb, Q, K, [1, 1])
    O, _ = orc.attn_fwd(pb, Q, K, V, rp, idx, 0.7)
    T = pb.T
    blk = np.concatenate([np.arange(130) // 64, 100 + np.arange(64) // 64])
    local = (blk[:, None] == blk[None, :]) & (np.arange(T)[None, :] <= np.arange(T)[:, None])
    Ow, _, _ = bf.masked_attention(Q, K, V, [local, local], 0.7)
    np.testing.assert_allclose(O, Ow, rtol=1e-10, atol=1e-12)


def test_packing_invariance():
    lens = [150, 70, 33]
    pb, Q, K, V, dO = make(lens, 2, 1, 8, 16, 0, seed=23)
    topk = [3, 2, 1]
    rp, idx = select(pb, Q, K, topk)
    O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, 0.4)
    dQ, dK, dV = orc.attn_bwd(pb, Q, K, V, dO, rp, idx, 0.4)
    for s in range(3):
        a, b = pb.cu[s], pb.cu[s + 1]
        p1 = orc.Problem(np.array([0, lens[s]], dtype=np.int32), 2, 1, 8, 16, 0)
        rp1, idx1 = select(p1, Q[a:b], K[a:b], [topk[s]])
        O1, LSE1 = orc.attn_fwd(p1, Q[a:b], K[a:b], V[a:b], rp1, idx1, 0.4)
        dQ1, dK1, dV1 = orc.attn_bwd(p1, Q[a:b], K[a:b], V[a:b], dO[a:b], rp1, idx1, 0.4)
        assert np.array_equal(O[a:b], O1) and np.array_equal(LSE[:, a:b], LSE1)
        assert np.array_equal(dQ[a:b], dQ1) and np.array_equal(dK[a:b], dK1) and np.array_equal(dV[a:b], dV1)


# ---------------------------------------------------------------- backward
def test_finite_differences_fixed_selection():
    pb, Q, K, V, dO = make([40, 9], 4, 2, 4, 8, 0, seed=29)
    rp, idx = select(pb, Q, K, [2, 1])
    scale = 0.6
    Q, K, V, dO = (x.astype(np.float64) for x in (Q, K, V, dO))
    # float32 inputs are required by the checker: use values exactly representable after perturbation
    Q32, K32, V32, dO32 = (x.astype(np.float32) for x in (Q, K, V, dO))
    dQ, dK, dV = orc.attn_bwd(pb, Q32, K32, V32, dO32, rp, idx, scale)

    def loss(q, k, v):
        O, _ = orc.attn_fwd(pb, q, k, v, rp, idx, scale)
        return float((O * dO32.astype(np.float64)).sum())

    eps = 2.0 ** -7                                      # exact in float32 for N(0,1)-sized values
    rng = np.random.default_rng(1)
    for name, X, grad in (("q", Q32, dQ), ("k", K32, dK), ("v", V32, dV)):
        for _ in range(25):
            pos = tuple(rng.integers(0, n) for n in X.shape)
            Xp, Xm = X.copy(), X.copy()
            Xp[pos] += np.float32(eps); Xm[pos] -= np.float32(eps)
            h = (float(Xp[pos]) - float(Xm[pos])) / 2
            args_p = {"q": (Xp, K32, V32), "k": (Q32, Xp, V32), "v": (Q32, K32, Xp)}[name]
            args_m = {"q": (Xm, K32, V32), "k": (Q32, Xm, V32), "v": (Q32, K32, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert abs(fd - grad[pos]) <= 2e-4 * max(1.0, abs(fd)), (name, pos, fd, grad[pos])


@pytest.mark.parametrize("mode", [0, 1])
def test_scale_homogeneity_identity(mode):
    # softmax(scale * (aQ)(K/a)^T) is independent of a  =>  sum_h <Q_h, dQ_h> = <K_g, dK_g> per KV group
    pb, Q, K, V, dO = make([130, 40], 4, 2, 8, 16, mode, seed=31)
    rp, idx = select(pb, Q, K, [3, 2])
    dQ, dK, dV = orc.attn_bwd(pb, Q, K, V, dO, rp, idx, 0.45)
    for s in range(pb.S):
        a, b = pb.cu[s], pb.cu[s + 1]
        for g in range(2):
            lhs = sum(float((Q[a:b, h].astype(np.float64) * dQ[a:b, h]).sum()) for h in (2 * g, 2 * g + 1))
            rhs = float((K[a:b, g].astype(np.float64) * dK[a:b, g]).sum())
            assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(lhs))


def test_gqa_equals_replicated_mha():
    pb, Q, K, V, dO = make([100, 30], 4, 2, 8, 16, 0, seed=37)
    rp, idx = select(pb, Q, K, [3, 1])
    O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, 0.5)
    dQ, dK, dV = orc.attn_bwd(pb, Q, K, V, dO, rp, idx, 0.5)
    pr = orc.Problem(pb.cu, 4, 4, 8, 16, 0)
    Kr, Vr = np.repeat(K, 2, axis=1), np.repeat(V, 2, axis=1)
    Or, LSEr = orc.attn_fwd(pr, Q, Kr, Vr, rp, idx, 0.5)    # same per-query-head selection
    dQr, dKr, dVr = orc.attn_bwd(pr, Q, Kr, Vr, dO, rp, idx, 0.5)
    np.testing.assert_allclose(O, Or, rtol=1e-13); np.testing.assert_allclose(dQ, dQr, rtol=1e-13)
    np.testing.assert_allclose(dK, dKr.reshape(pb.T, 2, 2, 8).sum(axis=2), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dV, dVr.reshape(pb.T, 2, 2, 8).sum(axis=2), rtol=1e-11, atol=1e-13)


def test_sampled_entry_points_agree_with_full():
    for mode in (0, 1):
        pb, Q, K, V, dO = make([300, 70, 5], 4, 2, 8, 64, mode, seed=41)
        rp, idx = select(pb, Q, K, [3, 2, 1])
        O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, 0.5)
        dQ, dK, dV = orc.attn_bwd(pb, Q, K, V, dO, rp, idx, 0.5)
        toks = np.array([0, 63, 64, 299, 300, 369, 370, 374], dtype=np.int32)
        heads = np.array([0, 1, 2, 3, 0, 1, 2, 3], dtype=np.int32)
        Os, LSEs, dQs = orc.attn_rows(pb, Q, K, V, dO, rp, idx, 0.5, toks, heads)
        for a, (t, h) in enumerate(zip(toks, heads)):
            assert np.array_equal(Os[a], O[t, h]) and LSEs[a] == LSE[h, t]
            assert np.array_equal(dQs[a], dQ[t, h])
        for (s, g, j) in ((0, 0, 0), (0, 1, 2), (0, 0, 4), (1, 1, 1), (2, 0, 0)):
            dKb, dVb = orc.attn_bwd_kvblock(pb, Q, K, V, dO, rp, idx, 0.5, s, g, j)
            a = pb.cu[s] + j * 64
            b = min(a + 64, pb.cu[s + 1])
            np.testing.assert_allclose(dKb[: b - a], dK[a:b, g], rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(dVb[: b - a], dV[a:b, g], rtol=1e-11, atol=1e-13)
            assert not dKb[b - a:].any() and not dVb[b - a:].any()


def test_degenerate_shapes():
    # an empty sequence in the middle, a 1-token sequence, budget above n
    pb, Q, K, V, dO = make([5, 0, 1], 2, 1, 4, 4, 0, seed=43)
    assert pb.nblk == [2, 0, 1]
    rp, idx = select(pb, Q, K, [9, 3, 9])
    O, LSE = orc.attn_fwd(pb, Q, K, V, rp, idx, 1.0)
    dense = [bf.causal_same_sequence_mask(pb.cu)] * 2
    Ow, _, _ = bf.masked_attention(Q, K, V, dense, 1.0)
    np.testing.assert_allclose(O, Ow, rtol=1e-12)
    np.testing.assert_allclose(O[5, 0], V[5, 0], rtol=1e-12)       # a lone token attends to itself
