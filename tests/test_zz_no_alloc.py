"""The selection entry point that allocates nothing (sb_select_topk_static) against sb_select_topk: same bits, on two
calls in a row on the same GPU, the second with a smaller input (the built-in scratch keeps the first call's tables)."""
import ctypes as C

import numpy as np
import pytest
import torch

from helpers import DEV, to_dev
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth

pytestmark = pytest.mark.gpu


def _both(w, mode):
    t = w.tensors()
    topk = sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
    pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, select_mode=mode, device=DEV)
    lay = pb.layout
    assert lay.select_ws_bytes <= (1 << 20)
    scores = sb.sb_block_scores(pb, to_dev(t["q"], "bf16"), to_dev(t["k"], "bf16"))
    rowptr, idx = sb.sb_select_topk(pb, scores)                       # the existing entry point, caller's workspace
    # the new one, straight through the C ABI: no workspace, outputs pre-filled with a pattern
    rp2 = torch.full((lay.sel_rows + 1,), -7, dtype=torch.int32, device=DEV)
    ix2 = torch.full((max(lay.sel_nnz, 1),), -7, dtype=torch.int32, device=DEV)
    before = torch.cuda.memory_allocated()
    rc = sb.lib().sb_select_topk_static(pb.ref(), C.c_void_p(scores.data_ptr()), C.c_void_p(rp2.data_ptr()),
                                        C.c_void_p(ix2.data_ptr()), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, sb.lib().sb_last_error().decode()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    nnz = int(rowptr[-1].item())
    assert nnz == lay.sel_nnz
    assert torch.equal(rp2, rowptr), "row pointers differ"
    assert torch.equal(ix2[:nnz], idx[:nnz]), "selected blocks differ"


@pytest.mark.parametrize("mode", [0, 1])
def test_two_calls_in_a_row_second_one_smaller(mode):
    big = synth.small_ragged(seed=61, lens=(64 * 90 + 7, 700, 64, 1, 0, 130, 2500), Hq=8, Hkv=2, D=128, ratio=(0.1, 0.6))
    small = synth.small_ragged(seed=62, lens=(300, 65), Hq=4, Hkv=2, D=64, ratio=(0.3, 0.9))
    _both(big, mode)
    _both(small, mode)
    _both(big, mode)


def test_empty_problem_and_oversized_problem():
    pb = sb.Problem([0, 0], [1], 4, 2, 64, device=DEV)
    rp = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    rc = sb.lib().sb_select_topk_static(pb.ref(), None, C.c_void_p(rp.data_ptr()), None, None)
    torch.cuda.synchronize()
    assert rc == 0 and int(rp[0].item()) == 0
    # 300 000 one-token sequences: the block -> sequence table alone exceeds the built-in scratch
    S = 300000
    pb = sb.Problem(np.arange(S + 1), np.ones(S), 2, 1, 64, device=DEV)
    assert pb.layout.select_ws_bytes > (1 << 20)
    x = torch.zeros(4, dtype=torch.int32, device=DEV)
    rc = sb.lib().sb_select_topk_static(pb.ref(), C.c_void_p(x.data_ptr()), C.c_void_p(x.data_ptr()), C.c_void_p(x.data_ptr()), None)
    assert rc == -3 and "built-in scratch" in sb.lib().sb_last_error().decode()
