"""CPU-only tests of the C-ABI library: it loads, exports every declared symbol, and its host
logic (validation, closed-form sizes, budget rule, row pointers) agrees with the CPU checker."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sparsebal.h")).read()
    declared = set(re.findall(r"\b(sb_[a-z_0-9]+)\s*\(", hdr))
    assert {"sb_block_scores", "sb_select_topk", "sb_plan_worklist", "sb_sparse_attn_fwd", "sb_sparse_attn_bwd"} <= declared
    lib = sb.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert set(sb.EXPORTS) == declared
    assert "gfx950" in sb.sb_version()


def _ragged_b256(seed):
    return synth.small_ragged(seed, lens=(3000, 64, 1, 700, 0, 257, 5000), B=256, ratio=(0.2, 0.9))


def _ragged_b128(seed):
    return synth.small_ragged(seed, lens=(3000, 64, 1, 700, 0, 257, 5000), B=128, ratio=(0.2, 0.9))


@pytest.mark.parametrize("maker", [synth.config1, synth.config2, synth.config3, synth.config5, synth.small_ragged, _ragged_b128, _ragged_b256])
@pytest.mark.parametrize("mode", [0, 1])
def test_layout_matches_checker_counts(maker, mode):
    w = maker(1)
    topk = w.topk if w.topk is not None else sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
    if w.keep_ratio is not None:
        assert np.array_equal(topk, orc.keep_ratio_to_topk(w.cu, w.B, w.keep_ratio))
    pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, select_mode=mode)
    po = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, mode)
    lay = pb.layout
    assert lay.num_qblocks == po.NQB and lay.sel_heads == po.Hs
    assert lay.scores_elems == int(po.score_off[-1])
    rp = orc.sel_rowptr(po, topk)
    assert np.array_equal(sb.sb_sel_rowptr_host(pb), rp) and lay.sel_nnz == rp[-1] and lay.sel_rows == len(rp) - 1
    # unmasked pairs, counted straight from the definition
    pairs = 0
    for s, n in enumerate(po.nblk):
        L = int(w.cu[s + 1] - w.cu[s])
        k = min(int(topk[s]), n)
        for i in range(n):
            rows = min(w.B, L - i * w.B)
            pairs += (min(k, i + 1) - 1) * rows * w.B + rows * (rows + 1) // 2
    assert lay.attended_pairs_per_head_sum == pairs * w.Hq


def test_keep_ratio_rule():
    cu = np.array([0, 640, 705, 1705, 1708], dtype=np.int32)
    assert sb.sb_keep_ratio_to_topk(cu, 64, [0.1, 0.5, 0.26, 0.9]).tolist() == [1, 1, 5, 1]
    assert sb.sb_keep_ratio_to_topk(cu, 64, [0.0, 1.0, 2.0, 0.0]).tolist() == [1, 2, 16, 1]


def _problem(**kw):
    base = dict(cu_seqlens=[0, 100], topk=[2], Hq=4, Hkv=2, D=64)
    base.update(kw)
    return base


@pytest.mark.parametrize("kw,code", [
    (dict(Hq=3), -1), (dict(D=96), -2), (dict(B=96), -2), (dict(B=512), -2), (dict(topk=[0]), -1), (dict(cu_seqlens=[0, 50, 40]), -1),
    (dict(cu_seqlens=[1, 100]), -1), (dict(dtype=7), -1), (dict(select_mode=3), -1),
    (dict(Hq=18, Hkv=2, select_mode=1), -2), (dict(cu_seqlens=[0, 64 * 16385], topk=[1]), -2),
])
def test_invalid_problems_are_rejected(kw, code):
    args = _problem(**kw)
    if len(args["topk"]) != len(args["cu_seqlens"]) - 1:
        args["topk"] = [1] * (len(args["cu_seqlens"]) - 1)
    with pytest.raises(sb.SparseBalError) as e:
        sb.Problem(**args)
    assert f"error {code}:" in str(e.value) and len(str(e.value)) > 25


def test_empty_problem_layout():
    pb = sb.Problem([0], [], 4, 2, 64)
    assert pb.layout.num_qblocks == 0 and pb.layout.sel_nnz == 0
    pb = sb.Problem([0, 0, 0], [1, 1], 4, 2, 64)
    assert pb.layout.num_qblocks == 0 and pb.layout.sel_nnz == 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(sb, "_lib", None)
    monkeypatch.setattr(sb, "LIB_PATH", "/nonexistent/libsparsebal.so")
    with pytest.raises(sb.SparseBalError):
        sb.sb_version()


# ---------------------------------------------------------------- budget controller, host side
def _random_table(rng, nx, nk):
    xs = np.cumsum(rng.integers(200, 5000, size=nx)).astype(np.float32)
    ks = np.cumsum(rng.integers(1, 12, size=nk)).astype(np.float32)
    lat = (np.outer(xs, ks) * 1e-4 * rng.uniform(0.7, 1.3, size=(nx, nk))).astype(np.float32)
    return xs, ks, lat


def test_latency_table_predict_and_align_match_the_checker():
    from oracle import dst_oracle as dst
    rng = np.random.default_rng(11)
    for nx, nk in ((1, 1), (1, 4), (3, 1), (5, 6)):
        xs, ks, lat = _random_table(rng, nx, nk)
        tab = sb.PerfTable(xs, ks, lat)
        for _ in range(40):
            x = float(rng.uniform(0.5 * xs[0], 1.2 * xs[-1])); k = float(rng.integers(1, int(ks[-1]) + 4))
            assert sb.sb_perf_predict(tab, x, k) == dst.perf_predict(xs, ks, lat, x, k)
            T = float(rng.uniform(0.0, 1.2 * lat.max()))
            assert sb.sb_perf_align(tab, x, T, 40) == dst.perf_align(xs, ks, lat, x, T, 40)
        for a in range(nx):      # exact at the grid points
            for b in range(nk):
                assert sb.sb_perf_predict(tab, float(xs[a]), float(ks[b])) == float(lat[a, b])
    with pytest.raises(sb.SparseBalError):
        sb.sb_perf_predict(sb.PerfTable([2.0, 1.0], [1.0], [[1.0], [2.0]]), 1.0, 1.0)


@pytest.mark.parametrize("anchor", [0, 1, 2])
def test_dst_tune_matches_the_checker(anchor):
    from oracle import dst_oracle as dst
    rng = np.random.default_rng(12 + anchor)
    lens = [700, 64, 0, 5000, 12000, 1, 2300]
    cu = synth.cu_from_lengths(lens)
    nblk = [(L + 63) // 64 for L in lens]
    Hs = 2
    blocks, off = [], [0]
    for n in nblk:
        blocks.append(rng.normal(size=Hs * n * n) * 2.5)
        off.append(off[-1] + Hs * n * n)
    cov = dst.coverage_curves(nblk, Hs, np.concatenate(blocks), off).astype(np.float32)
    qb = np.concatenate([[0], np.cumsum(nblk)]).astype(int)
    xs, ks, lat = _random_table(rng, 4, 5)
    tab = sb.PerfTable(xs, ks, lat)
    kbase = [3, 1, 1, 20, 30, 1, 40]   # the last one is clamped to its 36 blocks
    pb = sb.Problem(cu, kbase, 4, 2, 64)
    for p in (0.0, 0.02, 0.1, 0.3, 1.0):
        kf, ka, ta = sb.sb_dst_tune(pb, cov, tab, anchor, p)
        rf, ra, rt = dst.dst_budgets(p, anchor, lens, nblk, kbase, cov, qb, xs, ks, lat)
        assert np.array_equal(kf, rf) and np.array_equal(ka, ra) and ta == rt


def test_shipped_latency_table_loads_and_aligns():
    tab = sb.PerfTable.from_json(os.path.join(ROOT, "paper_2604_13847_amd", "perf_tables", "mi355x_hq32_hkv8_d128.json"))
    assert np.all(np.diff(tab.lengths) > 0) and np.all(np.diff(tab.budgets) > 0) and np.all(tab.latency > 0)
    # the profiled latency grows with the length at every budget; a longer sequence gets a smaller budget for the same target
    assert np.all(np.diff(tab.latency, axis=0) > 0)
    t = sb.sb_perf_predict(tab, 16384, 32)
    assert sb.sb_perf_align(tab, 16384, t, 256) >= 32 > sb.sb_perf_align(tab, 32768, t, 512)


# ---------------------------------------------------------------- sparsity-aware batching, host side
def test_sab_matches_the_checker_and_balances_the_length_mix():
    from oracle import dst_oracle as dst
    from oracle import sab_oracle as sab
    rng = np.random.default_rng(21)
    tab = sb.PerfTable.from_json(os.path.join(ROOT, "paper_2604_13847_amd", "perf_tables", "mi355x_hq32_hkv8_d128.json"))
    xs, ks, lat = tab.lengths, tab.budgets, tab.latency
    lens = np.array(synth.mixed_lengths(3, 64 * 4096, short=(512, 4096), long=(8192, 32768)), dtype=np.int32)   # the 60/40 length mix
    n = len(lens)
    # sparsity predictor: moving average per length bin, exact against the checker
    edges = [0, 2048, 8192, 16384, 1 << 30]
    spar = sb.SparsityPredictor(edges, decay=0.8)
    ema, seen = np.zeros(4), np.zeros(4, dtype=bool)
    for step in range(3):
        kfin = rng.integers(1, 64, size=n)
        spar.update(lens, kfin)
        ema, seen = sab.spar_update(ema, seen, edges, 0.8, lens, kfin)       # the checker keeps its state in float64
    # The library keeps the running value in float32 (one step is computed in double and rounded once): every update
    # adds at most half an ulp of a value below 64, and earlier errors decay by 0.8 per update, so the two states differ
    # by at most 2^-24 * 64 / (1 - 0.8) = 1.9e-5.
    assert np.array_equal(spar.seen.astype(bool), seen)
    assert np.abs(spar.ema.astype(np.float64) - ema).max() <= 2.0 ** -24 * 64 / 0.2
    kpred = np.array([spar.predict(int(L), 16.0) for L in lens])
    kref = np.array([sab.spar_predict(ema, seen, edges, L, 16.0) for L in lens])
    assert np.abs(kpred - kref).max() <= 2.0 ** -24 * 64 / 0.2
    # the predictions are exactly the stored state of the bin
    assert np.array_equal(kpred, np.array([sab.spar_predict(spar.ema.astype(np.float64), seen, edges, L, 16.0) for L in lens]))
    assert sb.SparsityPredictor(edges).predict(5000, 12.0) == 12.0
    # weights and the two-level partition, exact
    for rank in range(4):
        w, dp, mb = sb.sb_sab_batches(tab, lens, kpred, 4, rank, 2)
        wr = sab.sab_weights(xs, ks, lat, lens, kpred)
        rdp, rmb = sab.sab_batches(wr, 4, rank, 2)
        assert np.array_equal(w, wr) and np.array_equal(dp, rdp) and np.array_equal(mb, rmb)
    assert np.array_equal(sb.sb_balanced_partition(wr, 7), sab.balanced_partition(wr, 7))
    # Eq. 11 on the synthetic mix: latency-weighted bins are better balanced (in predicted latency) than length-weighted ones
    by_len = sab.balanced_partition(lens.astype(np.float64), 4)
    assert sab.imbalance(wr, dp, 4) <= sab.imbalance(wr, by_len, 4) + 1e-12
