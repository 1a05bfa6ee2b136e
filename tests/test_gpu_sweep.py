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
