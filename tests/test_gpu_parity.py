"""GPU parity: every call of the C-ABI library against the CPU checker on the same seeded inputs.

Scores within float32 tolerance; selection bit-exact given identical scores; plan properties;
O / LSE / dQ / dK / dV within max-abs 2e-2 and mean-abs 2e-3 of the float64 checker run on the same
selection (the GPU's)."""
import numpy as np
import pytest
import torch

from helpers import DEV, MEAN_ABS, Run, check_bwd_items, check_close, check_lse, err_stats, to_dev, to_host_f32
from oracle import oracle as orc
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth

pytestmark = pytest.mark.gpu


def check_scores(r: Run):
    got = r.scores.cpu().numpy()[: r.pb.layout.scores_elems]
    q, k, _, _ = (r.host[n] for n in ("q", "k", "v", "do"))     # scores are computed from the stored values
    ref = orc.block_scores(r.opb, q, k, r.scale)
    assert np.array_equal(np.isneginf(got), np.isneginf(ref))
    fin = np.isfinite(ref)
    if fin.any():
        scale = max(1e-3, float(np.abs(ref[fin]).max()))
        assert np.abs(got[fin] - ref[fin]).max() <= 2e-5 * scale, np.abs(got[fin] - ref[fin]).max() / scale
    return got


def check_selection(r: Run, got_scores):
    rp, idx = orc.select_topk(r.opb, got_scores, r.topk)       # decision on the GPU's own float32 scores
    assert np.array_equal(r.rowptr_h, rp)
    assert np.array_equal(r.idx_h, idx)


def check_plan(r: Run):
    pv = sb.plan_views(r.pb, r.plan)
    lay, po = r.pb.layout, r.opb
    NQB, Hs, Hkv, G = lay.num_qblocks, lay.sel_heads, r.w.Hkv, r.w.Hq // r.w.Hkv
    assert np.array_equal(pv["qb_off"], po.qb_off.astype(np.int32))
    wf = pv["work_fwd"]
    assert np.array_equal(np.sort(wf), np.arange(Hs * NQB))                  # every item exactly once
    cost = np.diff(r.rowptr_h)
    assert np.all(np.diff(cost[wf]) <= 0)                                    # longest first
    # bitmap is the exact transpose of the CSR
    colcost = np.zeros(Hkv * NQB, dtype=np.int64)
    bm = pv["bitmap"]
    for s, n in enumerate(po.nblk):
        w = (n + 31) // 32
        for hs in range(Hs):
            dense = np.zeros((n, n), dtype=bool)                             # dense[j, i]
            for i in range(n):
                row = hs * NQB + po.qb_off[s] + i
                js = r.idx_h[r.rowptr_h[row]:r.rowptr_h[row + 1]]
                dense[js, i] = True
                g = hs // G if r.mode == 0 else hs
                colcost[g * NQB + po.qb_off[s] + js] += 1 if r.mode == 0 else G
            words = bm[Hs * pv["bm_off"][s] + hs * n * w: Hs * pv["bm_off"][s] + (hs + 1) * n * w].reshape(n, w)
            bits = ((words[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool).reshape(n, w * 32)[:, :n]
            assert np.array_equal(bits, dense), (s, hs)
    assert np.array_equal(pv["colcost"], colcost)
    assert colcost.sum() == cost.sum() * (1 if r.mode == 0 else G)
    check_bwd_items(pv, colcost, po.nblk, po.qb_off, NQB, Hkv)


def check_attention(r: Run, bwd=True):
    q, k, v, do = r.oracle_inputs()
    O, LSE = orc.attn_fwd(r.opb, q, k, v, r.rowptr_h, r.idx_h, r.scale)
    stats = {"O": check_close("O", to_host_f32(r.o), O)}
    stats["LSE"] = check_lse(r.lse.cpu().numpy(), LSE)
    if bwd:
        dQ, dK, dV = orc.attn_bwd(r.opb, q, k, v, do, r.rowptr_h, r.idx_h, r.scale)
        stats["dQ"] = check_close("dQ", to_host_f32(r.dq), dQ)
        stats["dK"] = check_close("dK", to_host_f32(r.dk), dK)
        stats["dV"] = check_close("dV", to_host_f32(r.dv), dV)
    return stats


def full_check(w, mode, **kw):
    r = Run(w, mode, **kw)
    sc = check_scores(r)
    check_selection(r, sc)
    if w.B == 64:          # (for larger selection blocks the plan is laid out for 64-token tiles)
        check_plan(r)
    print(w, "mode", mode, check_attention(r), flush=True)
    return r


def test_config1_fp32_inputs():
    for seed in (0, 1, 2):
        r = full_check(synth.config1(seed), sb.SB_SELECT_PER_QHEAD)
        # The kernels round float32 inputs to bf16 on entry and the check above gives the checker the same rounded values.
        # Against the checker on the raw float32 values the input rounding shows as well (2^-9 relative on every
        # operand of a 64-long dot product): reported, and held to twice the bound.
        t = r.host
        O, LSE = orc.attn_fwd(r.opb, t["q"], t["k"], t["v"], r.rowptr_h, r.idx_h, r.scale)
        dQ, dK, dV = orc.attn_bwd(r.opb, t["q"], t["k"], t["v"], t["do"], r.rowptr_h, r.idx_h, r.scale)
        for name, got, ref in (("O", r.o, O), ("dQ", r.dq, dQ), ("dK", r.dk, dK), ("dV", r.dv, dV)):
            frac, mn, mx = err_stats(to_host_f32(got), ref)
            print(f"seed {seed} {name} against the checker on the unrounded float32 inputs: max-abs {mx:.4g} mean-abs {mn:.4g}", flush=True)
            assert frac <= 2.0 and mn <= 2 * MEAN_ABS


def test_pooled_keys_against_block_means():
    """kbar_out of sb_block_scores is the mean of K over the valid tokens of every block (tail blocks divide by their
    own count)."""
    for w in (synth.small_ragged(seed=41, lens=(200, 64, 1, 130, 0, 77, 450), Hq=4, Hkv=2, D=128, ratio=(0.3, 0.9)),
              synth.small_ragged(seed=42, lens=(700, 257, 1), Hq=6, Hkv=3, D=64, B=256, ratio=(0.3, 0.9)),
              synth.config1(0)):
        t = w.tensors()
        topk = w.topk if w.topk is not None else sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
        pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, dtype=sb.SB_BF16 if w.dtype == "bf16" else sb.SB_F32, device=DEV)
        _, kbar = sb.sb_block_scores(pb, to_dev(t["q"], w.dtype), to_dev(t["k"], w.dtype), want_kbar=True)
        torch.cuda.synchronize()
        po = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, 0)
        ref = orc.block_mean(po, t["k"])
        got = kbar.cpu().numpy()[: ref.size].reshape(ref.shape)
        assert np.abs(got - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max()), np.abs(got - ref).max()


# Workloads of a randomised sweep whose dQ / dK missed max-abs 2e-2 by a hair while Dr = rowsum(dO * O) was taken from the
# stored bf16 O on rows with one or two visible keys (the second token of a sequence, or of a block that keeps only
# itself).
@pytest.mark.parametrize("case", [
    dict(seed=1009, lens=[513, 1000, 786, 157], Hq=16, Hkv=2, D=128, B=256, ratio=(0.1, 0.3), mode=0),
    dict(seed=1021, lens=[63, 65], Hq=12, Hkv=3, D=64, B=256, ratio=(1.0, 1.0), mode=1),
    dict(seed=1019, lens=[1673, 1480, 65], Hq=8, Hkv=2, D=128, B=64, ratio=(0.0, 0.6), mode=0),
])
def test_rows_with_one_or_two_visible_keys_sweep_cases(case):
    mode = case.pop("mode")
    full_check(synth.small_ragged(**case), mode)


def test_one_token_sequences_many_heads_per_kv_head():
    """A batch of one-token sequences, 5 and 8 query heads per KV head (a case a randomised sweep turned up): O = V, dQ = dK
    = 0 and dV is the sum of the group's dO rows, so every dV element is large (1.8 or 2.3 on average) and the bf16 store
    alone moves the mean error past 2e-3; the mean bound's store term (helpers.py) is what this case needs, nothing else:
    the literal max-abs stays far inside its bound."""
    for G, lens in ((5, (1,)), (8, (1, 1, 1, 2))):
        w = synth.small_ragged(seed=90 + G, lens=lens, Hq=2 * G, Hkv=2, D=128, ratio=(0.3, 0.6))
        r = full_check(w, sb.SB_SELECT_PER_QHEAD)
        q, k, v, do = r.oracle_inputs()
        first = np.asarray(w.cu[:-1])                                   # the first token of every sequence sees only itself
        assert np.array_equal(to_host_f32(r.o)[first], np.repeat(v[first], G, axis=1))   # O = V exactly (the softmax weight is 1)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("D", [64, 128])
def test_rows_that_keep_only_their_own_block(mode, D):
    """Budget 1 everywhere and many very short sequences: every row sees at most its own block, the first rows of each
    sequence one, two, three keys."""
    lens = [2, 3, 1, 2, 65, 2, 130, 4, 2, 64, 2, 5] * 6
    w = synth.small_ragged(seed=51 + D, lens=lens, Hq=8, Hkv=2, D=D, ratio=(0.0, 0.0))
    r = full_check(w, mode)
    assert np.all(r.topk == 1)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("D", [64, 128])
def test_small_ragged_batches(mode, D):
    # several tiles per sequence, ragged tails, a 1-token sequence, an empty sequence, a <1-block sequence
    w = synth.small_ragged(seed=3, lens=(200, 64, 1, 130, 0, 77, 450), Hq=4, Hkv=2, D=D, ratio=(0.3, 0.9))
    full_check(w, mode)


@pytest.mark.parametrize("G", [1, 2, 3, 7, 8])
def test_group_sizes_per_kvgroup(G):
    w = synth.small_ragged(seed=4, lens=(300, 65), Hq=G, Hkv=1, D=128, ratio=(0.4, 0.8))
    full_check(w, sb.SB_SELECT_PER_KVGROUP)
    w = synth.small_ragged(seed=5, lens=(130, 190), Hq=2 * G, Hkv=2, D=64, ratio=(0.4, 0.8))
    full_check(w, sb.SB_SELECT_PER_QHEAD)


def test_full_budget_equals_dense_causal():
    w = synth.small_ragged(seed=6, lens=(333, 100), Hq=4, Hkv=2, D=128, ratio=(1.0, 1.0))
    r = full_check(w, 0)
    assert np.array_equal(r.topk, r.opb.nblk)


def test_budget_one_and_long_row():
    w = synth.small_ragged(seed=7, lens=(64 * 40 + 5,), Hq=2, Hkv=1, D=64, ratio=(0.0, 0.0))     # k = 1
    full_check(w, 0)
    w = synth.small_ragged(seed=8, lens=(64 * 300 + 17,), Hq=2, Hkv=2, D=64, ratio=(0.05, 0.05))  # 301 blocks, k = 16
    r = Run(w, 0, do_bwd=False)
    check_selection(r, check_scores(r))
    check_plan(r)


def test_selection_ties_nan_and_zero_bit_exact():
    # hand the selector adversarial scores: many exact ties, NaN, +-0, +-inf
    w = synth.small_ragged(seed=9, lens=(64 * 70, 64 * 9 + 1), Hq=4, Hkv=2, D=64)
    for mode in (0, 1):
        topk = np.array([9, 3], dtype=np.int32)
        pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, select_mode=mode, device=DEV)
        po = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, 64, mode)
        rng = np.random.default_rng(3)
        sc = rng.integers(-3, 4, size=pb.layout.scores_elems).astype(np.float32)
        for val, p in ((np.nan, .05), (-np.inf, .05), (-0.0, .05), (0.0, .05), (np.inf, .03)):
            sc[rng.random(sc.size) < p] = val
        rowptr, idx = sb.sb_select_topk(pb, torch.from_numpy(sc).to(DEV))
        rp, ix = orc.select_topk(po, sc, topk)
        assert np.array_equal(rowptr.cpu().numpy(), rp)
        assert np.array_equal(idx.cpu().numpy()[: rp[-1]], ix)


@pytest.mark.parametrize("mode,Hq,D", [(0, 4, 128), (1, 8, 64), (1, 8, 128), (1, 6, 64)])
def test_caller_supplied_selection_and_determinism(mode, Hq, D):
    # any valid selection is accepted: use the checker's selection from its own float64 scores
    w = synth.small_ragged(seed=10, lens=(5000, 129), Hq=Hq, Hkv=2, D=D, ratio=(0.3, 0.5))
    topk = sb.sb_keep_ratio_to_topk(w.cu, 64, w.keep_ratio)
    po = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, 64, mode)
    t = w.tensors()
    sel = orc.select_topk(po, orc.block_scores(po, t["q"], t["k"], 1 / np.sqrt(D)).astype(np.float32), topk)
    r1 = Run(w, mode, sel_override=sel)
    check_attention(r1)
    r2 = Run(w, mode, sel_override=sel)
    for a, b in ((r1.o, r2.o), (r1.lse, r2.lse), (r1.dq, r2.dq), (r1.dk, r2.dk), (r1.dv, r2.dv)):
        assert torch.equal(a, b)                       # run-to-run bitwise identical


@pytest.mark.parametrize("mode,B,D", [(0, 64, 64), (1, 64, 64), (0, 128, 128)])
def test_attention_sink_selection_splits_heavy_columns(mode, B, D):
    """A caller-supplied selection in which every query block keeps block 0 plus the blocks right before it (the shape
    real attention maps have): block 0 of the long sequence is kept by 701 query blocks of four heads, more than the
    split weight, so its column is cut into parts whose fp32 partial dK/dV are reduced in a fixed order."""
    nlong = 700 if B == 64 else 300   # (with 128-token blocks the plan works on two 64-token tiles per block: both tile columns of block 0 are split)
    w = synth.Workload("sink", [B * nlong + 9, 300, B * 40], 8, 2, D, B=B, topk=[4, 3, 5], seed=71)
    Hs = 8 if mode == 0 else 2
    sel = synth.sink_selection(w.cu, B, w.topk, Hs)
    r1 = Run(w, mode, sel_override=sel)
    if B == 64:
        check_plan(r1)
    pv = sb.plan_views(r1.pb, r1.plan)
    assert len(pv["split_cols"]) >= 2 and pv["slots_used"] >= 6, (pv["split_cols"], pv["slots_used"])
    # dK/dV of a split column add up the bf16-rounded P and dS of ~180 000 query rows (2^-9 relative each): a random walk
    # whose size follows the column's magnitude, not the element's, and which the bound 2e-2 + 2^-8 |ref| of an element
    # that happens to be small cannot see (a float64 model of exactly that rounding gives 0.025-0.032 before the output
    # rounding).  The token rows of split columns are therefore held to 2e-2 + 2^-8 max|ref of the key block|, every
    # other row to the usual bound.
    q, k, v, do = r1.oracle_inputs()
    O, LSE = orc.attn_fwd(r1.opb, q, k, v, r1.rowptr_h, r1.idx_h, r1.scale)
    dQ, dK, dV = orc.attn_bwd(r1.opb, q, k, v, do, r1.rowptr_h, r1.idx_h, r1.scale)
    stats = {"O": check_close("O", to_host_f32(r1.o), O), "LSE": check_lse(r1.lse.cpu().numpy(), LSE),
             "dQ": check_close("dQ", to_host_f32(r1.dq), dQ)}
    NQB = len(pv["qb_seq"])                                   # columns are 64-token tiles
    tile_off = np.asarray(pv["qb_off"], dtype=np.int64)
    heavy = np.zeros((w.T, w.Hkv), dtype=bool)
    for col, _, _ in pv["split_cols"]:
        g, qb = divmod(int(col), NQB)
        s = int(np.searchsorted(tile_off, qb, side="right") - 1)
        a = int(w.cu[s]) + 64 * (qb - int(tile_off[s]))
        b = min(a + 64, int(w.cu[s + 1]))
        heavy[a:b, g] = True
        for name, got, ref in (("dK", r1.dk, dK), ("dV", r1.dv, dV)):
            x, y = to_host_f32(got[a:b, g]).astype(np.float64), ref[a:b, g]
            err = np.abs(x - y).max()
            assert err <= 2e-2 + 2.0 ** -8 * np.abs(y).max(), (name, col, err, np.abs(y).max())
            stats[f"{name}[split {int(col)}]"] = (round(float(err), 5), round(float(np.abs(y).max()), 2))
    for name, got, ref in (("dK", r1.dk, dK), ("dV", r1.dv, dV)):
        stats[name] = check_close(name, to_host_f32(got)[~heavy], ref[~heavy])
        assert np.abs(to_host_f32(got) - ref).mean() <= MEAN_ABS
    print(w, "mode", mode, "split columns", pv["split_cols"].tolist(), stats, flush=True)
    r2 = Run(w, mode, sel_override=sel)
    for a, b in ((r1.dk, r2.dk), (r1.dv, r2.dv), (r1.dq, r2.dq)):
        assert torch.equal(a, b)                       # run-to-run bitwise identical, split columns included


def test_empty_problem_is_a_noop():
    pb = sb.Problem([0, 0], [1], 4, 2, 64, device=DEV)
    z = torch.zeros(8, dtype=torch.bfloat16, device=DEV)
    sc = sb.sb_block_scores(pb, z, z)
    rowptr, idx = sb.sb_select_topk(pb, sc)
    plan = sb.sb_plan_worklist(pb, rowptr, idx)
    o, lse = sb.sb_sparse_attn_fwd(pb, z, z, z, rowptr, idx, plan)
    sb.sb_sparse_attn_bwd(pb, z, z, z, o, lse, z, rowptr, idx, plan)
    torch.cuda.synchronize()
    assert rowptr.cpu().numpy()[0] == 0


@pytest.mark.parametrize("B", [128, 256])
@pytest.mark.parametrize("mode", [0, 1])
def test_selection_blocks_larger_than_a_tile(B, mode):
    """Selection blocks of 128 / 256 tokens (the block size of the paper's own runs is 256): scores, selection and
    attention against the checker run with the same block size, element by element."""
    w = synth.small_ragged(seed=4 + B, lens=(1500, B, 1, 0, B + 1, 2 * B - 1, 2300, 64), Hq=6, Hkv=2, D=128, B=B, ratio=(0.25, 0.8))
    r = Run(w, mode)
    q, k, v, do = r.oracle_inputs()
    ref_sc = orc.block_scores(r.opb, q, k, r.scale)
    got_sc = r.scores.cpu().numpy()[: r.pb.layout.scores_elems]
    fin = np.isfinite(ref_sc)
    assert np.array_equal(np.isneginf(got_sc), np.isneginf(ref_sc))
    assert np.abs(got_sc[fin] - ref_sc[fin]).max() <= 2e-5 * max(1e-3, np.abs(ref_sc[fin]).max())
    rp, idx = orc.select_topk(r.opb, got_sc, r.topk)
    assert np.array_equal(rp, r.rowptr_h) and np.array_equal(idx, r.idx_h)
    O, LSE = orc.attn_fwd(r.opb, q, k, v, r.rowptr_h, r.idx_h, r.scale)
    dQ, dK, dV = orc.attn_bwd(r.opb, q, k, v, do, r.rowptr_h, r.idx_h, r.scale)
    for name, got, ref in (("O", r.o, O), ("dQ", r.dq, dQ), ("dK", r.dk, dK), ("dV", r.dv, dV)):
        print(name, check_close(name, to_host_f32(got), ref))
    print("LSE", check_lse(r.lse.cpu().numpy(), LSE))


def test_block_256_full_budget_is_dense_causal():
    w = synth.small_ragged(seed=9, lens=(1000, 300), Hq=2, Hkv=1, D=64, B=256, ratio=(1.0, 1.0))
    r = Run(w, 0)
    dense = synth.Workload("dense64", w.lens, 2, 1, 64, B=64, keep_ratio=[1.0, 1.0], seed=9)   # same tokens, 64-token blocks, everything kept
    r64 = Run(dense, 0)
    for a, b in ((r.o, r64.o), (r.dq, r64.dq), (r.dk, r64.dk), (r.dv, r64.dv)):
        assert np.abs(to_host_f32(a) - to_host_f32(b)).max() <= 2e-2


def test_sixteen_query_heads_on_one_kv_head_per_qhead():
    """More than eight selection heads per KV head: the key-major kernel walks them in groups of eight."""
    w = synth.small_ragged(seed=13, lens=(700, 130, 65), Hq=16, Hkv=1, D=64, ratio=(0.3, 0.7))
    r = Run(w, 0)
    q, k, v, do = r.oracle_inputs()
    O, LSE = orc.attn_fwd(r.opb, q, k, v, r.rowptr_h, r.idx_h, r.scale)
    dQ, dK, dV = orc.attn_bwd(r.opb, q, k, v, do, r.rowptr_h, r.idx_h, r.scale)
    for name, got, ref in (("O", r.o, O), ("dQ", r.dq, dQ), ("dK", r.dk, dK), ("dV", r.dv, dV)):
        print(name, check_close(name, to_host_f32(got), ref))


@pytest.mark.parametrize("mode", [0, 1])
def test_head_dim_64_seven_heads_per_kv_head_block_256(mode):
    """The head shape of the smaller model of the paper's runs (section 5: 14 query heads on 2 KV heads, head_dim 64)
    with the block size of those runs."""
    w = synth.small_ragged(seed=21, lens=(1100, 257, 700), Hq=14, Hkv=2, D=64, B=256, ratio=(0.3, 0.8))
    r = Run(w, mode)
    check_selection(r, check_scores(r))
    print(w, "mode", mode, check_attention(r), flush=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("D", [64, 128])
def test_four_heads_per_kv_group_share_tiles(D, dtype):
    """Per-KV-group selection with four query heads per KV head: the forward kernel that shares the K/V tiles of an item
    between the group's heads (ragged tails, a 1-token and an empty sequence, more than one tile per row)."""
    w = synth.small_ragged(seed=17, lens=(330, 64, 1, 0, 129, 500), Hq=8, Hkv=2, D=D, ratio=(0.3, 0.9), dtype=dtype)
    full_check(w, sb.SB_SELECT_PER_KVGROUP)


def test_more_than_1024_sequences():
    """More sequences than one pass of the geometry scan holds (1024): offsets carry over between passes."""
    lens = [1 + (37 * s + 11 * (s // 7)) % 150 for s in range(1100)]
    w = synth.small_ragged(seed=23, lens=lens, Hq=2, Hkv=1, D=64, ratio=(0.3, 1.0))
    full_check(w, sb.SB_SELECT_PER_QHEAD)


@pytest.mark.parametrize("mode", [0, 1])
def test_score_select_in_one_call(mode):
    """sb_score_select = sb_block_scores + sb_select_topk: same bits as the two calls, and the selection is the checker's
    on the scores it returned."""
    w = synth.small_ragged(seed=31, lens=(700, 64, 1, 0, 130, 1500), Hq=8, Hkv=2, D=128, ratio=(0.2, 0.9))
    r = Run(w, mode, do_bwd=False)
    scores, rowptr, idx = sb.sb_score_select(r.pb, r.q, r.k)
    torch.cuda.synchronize()
    n = r.pb.layout.scores_elems
    assert torch.equal(scores[:n].view(torch.int32), r.scores[:n].view(torch.int32))
    assert torch.equal(rowptr, r.rowptr) and torch.equal(idx[: int(r.rowptr_h[-1])], r.idx[: int(r.rowptr_h[-1])])
    rp, ix = orc.select_topk(r.opb, scores.cpu().numpy()[:n], r.topk)
    assert np.array_equal(rp, rowptr.cpu().numpy()) and np.array_equal(ix, idx.cpu().numpy()[: int(rp[-1])])


@pytest.mark.parametrize("mode,Hq,Hkv,lens", [(0, 8, 2, (64 * 300, 64 * 250 + 5)), (1, 8, 4, (64 * 560 - 3, 64 * 470))])
def test_ticketed_launches_elementwise(mode, Hq, Hkv, lens):
    """More than 4096 query-major items: the forward and dQ launches hand one item in sixteen out through a ticket
    counter at the end of the launch.  Every output element is compared, so an item that no workgroup took, or that two
    took, would show; per-query-head selection with one head per workgroup, and per-KV-group selection with the group's
    two heads in one workgroup."""
    w = synth.small_ragged(seed=81 + mode, lens=lens, Hq=Hq, Hkv=Hkv, D=64, ratio=(0.02, 0.04))
    r = Run(w, mode)
    assert r.pb.layout.sel_rows >= 4096
    print(w, "mode", mode, check_attention(r), flush=True)
    o2, lse2 = sb.sb_sparse_attn_fwd(r.pb, r.q, r.k, r.v, r.rowptr, r.idx, r.plan)       # same bits whoever draws which ticket
    dq2, dk2, dv2 = sb.sb_sparse_attn_bwd(r.pb, r.q, r.k, r.v, r.o, r.lse, r.do, r.rowptr, r.idx, r.plan)
    torch.cuda.synchronize()
    for a, b in ((o2, r.o), (dq2, r.dq), (dk2, r.dk), (dv2, r.dv)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(lse2, r.lse)


def fused_selection_matches(r: Run):
    """sb_score_select without a score buffer (one kernel, scores stay on chip) against the two calls of `r`."""
    _, rowptr, idx = sb.sb_score_select(r.pb, r.q, r.k, want_scores=False)
    torch.cuda.synchronize()
    nnz = int(r.rowptr_h[-1])
    assert torch.equal(rowptr, r.rowptr), "row pointers differ"
    assert torch.equal(idx[:nnz], r.idx[:nnz]), "selected blocks differ"


@pytest.mark.parametrize("mode", [0, 1])
def test_fused_score_select_same_bits(mode):
    """The single-kernel form selects the same blocks as sb_block_scores + sb_select_topk, bit for bit: ragged
    sequences, sequences inside one group of 16 rows, both head widths, larger selection blocks, budgets from 1 block
    to everything."""
    cases = [synth.small_ragged(seed=71, lens=(700, 64, 1, 0, 130, 1500, 64 * 40 + 3), Hq=8, Hkv=2, D=128, ratio=(0.05, 0.9)),
             synth.small_ragged(seed=72, lens=[1 + (53 * s) % 400 for s in range(60)], Hq=4, Hkv=2, D=64, ratio=(0.1, 1.0)),
             synth.small_ragged(seed=73, lens=(256 * 37 + 9, 300, 256 * 18), Hq=6, Hkv=3, D=64, B=256, ratio=(0.1, 0.5)),
             synth.small_ragged(seed=78, lens=(64 * 30 + 1, 300), Hq=16, Hkv=4, D=64, ratio=(0.1, 0.5)),   # 16 selection heads: permuted over the XCDs
             synth.Workload("budget1", [64 * 50, 64 * 20], 4, 1, 128, topk=[1, 2], seed=74),
             synth.Workload("budget_all", [64 * 50 + 1, 64 * 20], 4, 4, 128, topk=[51, 19], seed=75)]
    for w in cases:
        r = Run(w, mode, do_bwd=False)
        fused_selection_matches(r)
        print(w, "mode", mode, "fused selection identical", flush=True)


def test_fused_score_select_ties_and_long_rows():
    """All-equal scores (zero queries): ties go to the lower block index in both forms.  A sequence of 2600 blocks: fewer
    rows per workgroup in the fused kernel (its LDS holds 8 rows of that length, not 16)."""
    w = synth.small_ragged(seed=76, lens=(64 * 300 + 5, 900), Hq=4, Hkv=2, D=128, ratio=(0.1, 0.3))
    r = Run(w, sb.SB_SELECT_PER_QHEAD, do_bwd=False)
    r.q.zero_()
    r.scores = sb.sb_block_scores(r.pb, r.q, r.k)
    r.rowptr, r.idx = sb.sb_select_topk(r.pb, r.scores)
    torch.cuda.synchronize()
    r.rowptr_h = r.rowptr.cpu().numpy()
    idx_h = r.idx.cpu().numpy()
    k0, n0 = int(min(r.topk[0], 301)), 301
    row = n0 - 1                                             # last row of the first sequence, head 0
    assert list(idx_h[r.rowptr_h[row]:r.rowptr_h[row + 1]]) == list(range(k0 - 1)) + [n0 - 1]
    fused_selection_matches(r)
    w = synth.Workload("long2600", [64 * 2600 - 7, 64 * 33], 2, 1, 64, keep_ratio=[0.01, 0.5], seed=77)
    for mode in (0, 1):
        r = Run(w, mode, do_bwd=False)
        sc = check_scores(r)
        check_selection(r, sc)
        fused_selection_matches(r)


@pytest.mark.parametrize("nblk", [8200, 12500])
def test_more_than_8192_blocks_in_one_sequence(nblk):
    """A sequence of 8200 blocks (524 800 tokens): more columns than one pass of the plan's transpose holds, one row per
    workgroup in the selection, 129 row tiles in the score kernel.  With 12500 blocks the selection's LDS region also
    exceeds the default dynamic limit of 48 KiB."""
    w = synth.Workload("long1", [64 * (nblk - 1) + 5, 70], 1, 1, 64, keep_ratio=[0.0002, 1.0], seed=29)   # k = 2 or 3, and 2
    r = Run(w, sb.SB_SELECT_PER_QHEAD)
    sc = check_scores(r)
    check_selection(r, sc)
    fused_selection_matches(r)
    check_plan(r)
    print(w, check_attention(r), flush=True)
