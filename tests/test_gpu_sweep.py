"""A small seeded sweep over random shapes (selection block, head_dim, head counts, selection mode, input type, ragged
lengths, keep ratios): every call of the library against the checker, plus the one-kernel selection against the two-kernel
one.  The wider sweeps that turned up the special cases committed in test_gpu_parity.py draw from the same recipe."""
import numpy as np
import pytest

from helpers import Run
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth
from test_gpu_parity import check_attention, check_plan, check_scores, check_selection, fused_selection_matches

pytestmark = pytest.mark.gpu


def draw_case(rng, c):
    B = int(rng.choice([64, 64, 64, 128, 256]))
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 3, 4, 5, 7, 8]))
    mode = int(rng.choice([0, 1]))
    S = int(rng.integers(1, 6))
    lens = [int(rng.choice([0, 1, 63, 64, 65, 200, 513, 1000, 1537, 2300])) if rng.random() < 0.5 else int(rng.integers(1, 2500))
            for _ in range(S)]
    if sum(lens) == 0:
        lens[0] = 77
    lo = float(rng.choice([0.0, 0.1, 0.3, 1.0]))
    hi = max(lo, float(rng.choice([0.3, 0.6, 1.0])))
    dtype = "f32" if rng.random() < 0.15 else "bf16"
    return synth.small_ragged(seed=2000 + c, lens=lens, Hq=G * Hkv, Hkv=Hkv, D=D, B=B, ratio=(lo, hi), dtype=dtype), mode


@pytest.mark.parametrize("seed", [41, 42])
def test_random_shapes(seed):
    rng = np.random.default_rng(seed)
    for c in range(8):
        w, mode = draw_case(rng, 100 * seed + c)
        r = Run(w, mode)
        check_selection(r, check_scores(r))
        if w.B == 64:
            check_plan(r)
        fused_selection_matches(r)
        print(w, "lens", w.lens, "mode", mode, check_attention(r), flush=True)


def adversarial_scores(rng, kind, n):
    x = rng.normal(size=n)
    if kind == 1:
        x = np.round(x * 2) / 2                            # heavy ties
    elif kind == 2:
        x = np.exp(x * 10)                                 # forty octaves
    elif kind == 3:
        x = -np.exp(x * 10)                                # all negative, wide
    elif kind == 4:
        x = np.where(rng.random(n) < 0.9, 1.5, x)          # mostly one value
    elif kind == 5:                                        # special values sprinkled in
        x = x.astype(np.float32)
        m = rng.random(n)
        x[m < 0.02] = np.nan
        x[(m >= 0.02) & (m < 0.04)] = np.inf
        x[(m >= 0.04) & (m < 0.06)] = -np.inf
        x[(m >= 0.06) & (m < 0.10)] = 0.0
        x[(m >= 0.10) & (m < 0.14)] = -0.0
        x[(m >= 0.14) & (m < 0.16)] = 1e-40
    elif kind == 6:
        x = 1.0 + x * 1e-6                                 # the whole row within one bin of the threshold search
    elif kind == 7:
        x = np.floor(x * 64) * 2.0 ** -20 + 3.0            # ties within one bin
    return x.astype(np.float32)


@pytest.mark.parametrize("seed", [7])
def test_selection_on_adversarial_scores(seed):
    """sb_select_topk on score matrices it is handed directly (ties, forty octaves of range, NaN, infinities, signed zeros,
    denormals, rows that fall into one bin of the threshold search), budgets from 1 to all with values on both sides of
    the quarter-of-the-row switch between the two threshold searches: bit-exact against the checker's total order."""
    import torch
    from helpers import DEV
    from oracle import oracle as orc
    rng = np.random.default_rng(seed)
    for c in range(48):
        Hs, S = int(rng.choice([1, 2, 3])), int(rng.integers(1, 4))
        lens = [int(rng.choice([1, 64 * 5, 64 * 64 + 1, 64 * 65, 64 * 300, 64 * 1100, 64 * 2049])) if rng.random() < 0.5
                else int(rng.integers(1, 64 * 700)) for _ in range(S)]
        nb = [(l + 63) // 64 for l in lens]
        topk = [int(max(1, rng.choice([1, 2, 3, 8, 17, 64, n // 8 + 1, n // 4, n // 4 + 1, n // 2 + 1, max(n - 1, 1), n]))) for n in nb]
        w = synth.Workload("sel", lens, Hs, Hs, 64, topk=topk, seed=c)
        pb = sb.Problem(w.cu, w.topk, w.Hq, w.Hkv, w.D, w.B, dtype=sb.SB_BF16, select_mode=0, device=DEV)
        po = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, 0)
        sc = adversarial_scores(rng, c % 8, int(pb.layout.scores_elems))
        rp, ix = sb.sb_select_topk(pb, torch.from_numpy(sc).to(DEV))
        torch.cuda.synchronize()
        rp_h = rp.cpu().numpy()
        rr, ii = orc.select_topk(po, sc, np.asarray(topk, dtype=np.int32))
        assert np.array_equal(rr, rp_h) and np.array_equal(ii, ix.cpu().numpy()[: int(rp_h[-1])]), (c, c % 8, nb, topk)
