"""GPU parity of the budget controller: coverage curves of the routing scores (paper section 4.1,
Eq. 4) against the float64 checker, element by element, and the tuning rule (Algorithm 1) end to end
on the GPU's own curves."""
import numpy as np
import pytest
import torch

from helpers import DEV, to_dev
from oracle import dst_oracle as dst
from oracle import oracle as orc
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth

pytestmark = pytest.mark.gpu

# fp32 softmax, sort and running sums against float64: shares are <= 1 and a curve value is a mean of row sums
TOL = 2e-6


def _curves(w, mode, scores_override=None):
    topk = w.topk if w.topk is not None else sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
    dt = sb.SB_BF16 if w.dtype == "bf16" else sb.SB_F32
    pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, dtype=dt, select_mode=mode, device=DEV)
    po = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, mode)
    if scores_override is None:
        t = w.tensors()
        scores = sb.sb_block_scores(pb, to_dev(t["q"], w.dtype), to_dev(t["k"], w.dtype))
    else:
        scores = torch.from_numpy(scores_override.astype(np.float32)).to(DEV)
    cov = sb.sb_score_coverage(pb, scores)
    torch.cuda.synchronize()
    sc_h = scores.cpu().numpy()[: pb.layout.scores_elems]
    ref = dst.coverage_curves(po.nblk, po.Hs, sc_h, po.score_off)
    return pb, po, cov.cpu().numpy()[: po.NQB], ref, topk


@pytest.mark.parametrize("mode", [0, 1])
def test_coverage_small_ragged(mode):
    w = synth.small_ragged(seed=3, lens=(200, 64, 1, 0, 130, 1100, 77), Hq=4, Hkv=2, D=64)
    pb, po, got, ref, _ = _curves(w, mode)
    assert got.shape == ref.shape and np.abs(got - ref).max() <= TOL
    for s, n in enumerate(po.nblk):   # what the definition fixes at the ends of every curve
        if n:
            C = got[po.qb_off[s]: po.qb_off[s] + n]
            assert abs(C[0] - 1.0 / n) <= 1e-7 and abs(C[-1] - 1.0) <= 1e-7 and np.all(np.diff(C) >= -1e-7)


def test_coverage_benchmark_workload_and_determinism():
    w = synth.config2(0)
    pb, po, got, ref, _ = _curves(w, 0)
    assert np.abs(got - ref).max() <= TOL
    # a second run gives the same bits (fixed summation order)
    t = w.tensors()
    scores = sb.sb_block_scores(pb, to_dev(t["q"], "bf16"), to_dev(t["k"], "bf16"))
    again = sb.sb_score_coverage(pb, scores).cpu().numpy()[: po.NQB]
    assert np.array_equal(again, got)


def test_coverage_ties_wide_range_and_long_rows():
    # one sequence of 700 blocks (rows longer than the 256 threads of a workgroup, not a power of two),
    # scores with exact ties and a wide dynamic range
    n, Hs = 700, 2
    w = synth.Workload("long", [n * 64 - 5], Hs, Hs, 64, topk=[8])
    rng = np.random.default_rng(9)
    sc = np.round(rng.normal(size=(Hs, n, n)) * 6.0) * 0.5
    sc[0, :, 3] = 40.0
    pb, po, got, ref, _ = _curves(w, 0, scores_override=sc.ravel())
    assert np.abs(got - ref).max() <= TOL


def test_coverage_rows_on_both_sides_of_the_register_sort():
    """Rows of up to 2048 candidates are sorted in registers, longer ones in LDS: sequences of 2100 and 2050 blocks have
    rows of both kinds, the 3-head group leaves a wavefront of the register kernel without a head, and the short
    sequences use every register count (1 .. 32 keys per lane)."""
    w = synth.Workload("both", [2100 * 64 - 3, 2050 * 64, 65 * 64, 130 * 64, 300 * 64, 600 * 64, 1100 * 64], 3, 3, 64, topk=[16] * 7, seed=12)
    pb, po, got, ref, _ = _curves(w, 0)
    assert np.abs(got - ref).max() <= TOL
    for s, n in enumerate(po.nblk):
        C = got[po.qb_off[s]: po.qb_off[s] + n]
        assert abs(C[0] - 1.0 / n) <= 1e-7 and abs(C[-1] - 1.0) <= 1e-7 and np.all(np.diff(C) >= -1e-7)


@pytest.mark.parametrize("anchor", [0, 1, 2])
def test_tuned_budgets_end_to_end(anchor):
    # budgets from the GPU's curves drive the attention path: the tuned problem runs and matches the checker's decision
    w = synth.small_ragged(seed=5, lens=(900, 3000, 260, 5000), Hq=4, Hkv=2, D=64, ratio=(0.2, 0.5))
    pb, po, cov, _, kbase = _curves(w, 0)
    xs = np.array([256, 1024, 4096, 8192], dtype=np.float32)
    ks = np.array([1, 8, 32, 128], dtype=np.float32)
    lat = (np.outer(xs, np.minimum(ks, 128)) * 1e-5 + 0.02).astype(np.float32)
    tab = sb.PerfTable(xs, ks, lat)
    for p in (0.02, 0.3):
        kf, ka, ta = sb.sb_dst_tune(pb, cov, tab, anchor, p)
        rf, ra, rt = dst.dst_budgets(p, anchor, w.lens, po.nblk, kbase, cov, po.qb_off, xs, ks, lat)
        assert np.array_equal(kf, rf) and np.array_equal(ka, ra) and ta == rt
        pb2 = sb.Problem(w.cu, kf, w.Hq, w.Hkv, w.D, w.B, device=DEV)
        assert pb2.layout.sel_nnz == sum(w.Hq * (min(k, n) * n - min(k, n) * (min(k, n) - 1) // 2) for k, n in zip(kf, po.nblk))
