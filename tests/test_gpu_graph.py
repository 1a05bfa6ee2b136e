"""The whole path recorded into a HIP graph (through torch's stream capture) and replayed: the library
allocates nothing, never synchronises and clears its buffers with kernels, so a captured step must
give the eager result on every replay."""
import numpy as np
import pytest
import torch

from helpers import DEV, to_dev
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", ["small", "ticketed"])
def test_captured_step_replays_bitwise(case):
    """"ticketed": more than 4096 query-major items, so the forward and dQ launches hand the tail of their work list out
    through a ticket counter that a fill kernel clears in every step; this step also scores and selects in one kernel."""
    if case == "small":
        w = synth.small_ragged(seed=2, lens=(700, 64, 1, 2100, 333), Hq=8, Hkv=2, D=128, ratio=(0.2, 0.6))
    else:
        w = synth.small_ragged(seed=4, lens=(64 * 520 - 9, 700, 1), Hq=8, Hkv=2, D=64, ratio=(0.03, 0.08))
    topk = sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
    pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, device=DEV)
    lay = pb.layout
    t = w.tensors()
    q, k, v, do = (to_dev(t[n], "bf16") for n in ("q", "k", "v", "do"))
    raw = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=DEV)
    ws = [raw(lay.scores_ws_bytes), raw(lay.select_ws_bytes), raw(lay.fwd_ws_bytes), raw(lay.bwd_ws_bytes)]
    plan = raw(lay.plan_bytes)
    bufs = dict(o=torch.empty_like(q), lse=torch.empty((w.Hq, w.T), dtype=torch.float32, device=DEV),
                dq=torch.empty_like(q), dk=torch.empty_like(k), dv=torch.empty_like(v))
    scores = torch.empty(lay.scores_elems, dtype=torch.float32, device=DEV)
    rowptr = torch.empty(lay.sel_rows + 1, dtype=torch.int32, device=DEV)
    idx = torch.empty(lay.sel_nnz, dtype=torch.int32, device=DEV)
    import ctypes as C
    L = sb.lib()
    P = lambda x: C.c_void_p(x.data_ptr())

    def step():
        st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        if case == "small":
            rc = L.sb_block_scores(pb.ref(), P(q), P(k), None, P(scores), P(ws[0]), st)
            rc |= L.sb_select_topk(pb.ref(), P(scores), P(rowptr), P(idx), P(ws[1]), st)
        else:
            rc = L.sb_score_select(pb.ref(), P(q), P(k), None, None, P(rowptr), P(idx), P(ws[0]), st)
        rc |= L.sb_plan_worklist(pb.ref(), P(rowptr), P(idx), P(plan), st)
        rc |= L.sb_sparse_attn_fwd(pb.ref(), P(q), P(k), P(v), P(rowptr), P(idx), P(plan), P(bufs["o"]), P(bufs["lse"]), P(ws[2]), st)
        rc |= L.sb_sparse_attn_bwd(pb.ref(), P(q), P(k), P(v), P(bufs["o"]), P(bufs["lse"]), P(do), P(rowptr), P(idx), P(plan),
                                   P(bufs["dq"]), P(bufs["dk"]), P(bufs["dv"]), P(ws[3]), st)
        assert rc == 0, L.sb_last_error().decode()

    step()
    torch.cuda.synchronize()
    eager = {n: b.clone() for n, b in bufs.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for replay in range(3):
        for b in bufs.values():
            b.zero_()                           # eager work between the replays
        plan.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, b in bufs.items():
            assert torch.equal(b.view(torch.int16) if b.dtype == torch.bfloat16 else b, eager[n].view(torch.int16) if b.dtype == torch.bfloat16 else eager[n]), (n, replay)
