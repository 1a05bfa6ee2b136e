"""Thin ctypes binding of libsparsebal (include/sparsebal.h): argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels; torch is used here for device
memory and the current stream.  There is no CPU fallback: if the shared library is missing the
import of `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsparsebal.so")

SB_OK = 0
SB_BF16, SB_F32 = 0, 1
SB_SELECT_PER_QHEAD, SB_SELECT_PER_KVGROUP = 0, 1
SB_CU_SLOTS = 512

EXPORTS = ["sb_get_layout", "sb_keep_ratio_to_topk", "sb_sel_rowptr_host", "sb_block_scores", "sb_select_topk", "sb_select_topk_static", "sb_score_select",
           "sb_plan_worklist", "sb_plan_sections", "sb_sparse_attn_fwd", "sb_sparse_attn_bwd", "sb_score_coverage", "sb_perf_predict", "sb_perf_align", "sb_dst_tune",
           "sb_spar_update", "sb_spar_predict", "sb_balanced_partition", "sb_sab_batches",
           "sb_set_instrumentation", "sb_read_cu_busy", "sb_read_kernel_times",
           "sb_last_error", "sb_version"]


class sb_problem(C.Structure):
    _fields_ = [("total_tokens", C.c_int32), ("num_seqs", C.c_int32), ("num_q_heads", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("block_size", C.c_int32), ("dtype", C.c_int32),
                ("select_mode", C.c_int32), ("softmax_scale", C.c_float), ("score_scale", C.c_float),
                ("cu_seqlens_host", C.c_void_p), ("cu_seqlens_dev", C.c_void_p), ("topk_host", C.c_void_p),
                ("topk_dev", C.c_void_p)]


class sb_layout(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("num_qblocks", "sel_heads", "scores_elems", "pooled_elems", "sel_rows", "sel_nnz",
                                         "plan_bytes", "scores_ws_bytes", "select_ws_bytes", "fwd_ws_bytes", "bwd_ws_bytes",
                                         "attended_pairs_per_head_sum", "coverage_ws_bytes")]


class sb_perf_table(C.Structure):
    _fields_ = [("num_lengths", C.c_int32), ("num_budgets", C.c_int32), ("lengths", C.c_void_p), ("budgets", C.c_void_p),
                ("latency", C.c_void_p)]


_lib = None


class SparseBalError(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SparseBalError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        _lib = C.CDLL(LIB_PATH)
        _lib.sb_last_error.restype = C.c_char_p
        _lib.sb_version.restype = C.c_char_p
    return _lib


def _check(rc):
    if rc != SB_OK:
        raise SparseBalError(f"libsparsebal error {rc}: {lib().sb_last_error().decode()}")


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return C.c_void_p(t.data_ptr())
    return t.ctypes.data_as(C.c_void_p)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Problem:
    """Holds sb_problem plus the host/device arrays it points to."""

    def __init__(self, cu_seqlens, topk, Hq, Hkv, D, B=64, dtype=SB_BF16, select_mode=SB_SELECT_PER_QHEAD,
                 softmax_scale=0.0, score_scale=0.0, device=None):
        self.cu_host = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        self.topk_host = np.ascontiguousarray(topk, dtype=np.int32)
        self.S, self.T = len(self.cu_host) - 1, int(self.cu_host[-1]) if len(self.cu_host) else 0
        self.device = device
        if device is not None:
            self.cu_dev = torch.from_numpy(self.cu_host).to(device)
            self.topk_dev = torch.from_numpy(self.topk_host).to(device) if self.S else torch.zeros(1, dtype=torch.int32, device=device)
        else:
            self.cu_dev = self.topk_dev = None
        self.c = sb_problem(self.T, self.S, Hq, Hkv, D, B, dtype, select_mode, softmax_scale, score_scale,
                            self.cu_host.ctypes.data, self.cu_dev.data_ptr() if device is not None else None,
                            self.topk_host.ctypes.data if self.S else None,
                            self.topk_dev.data_ptr() if device is not None else None)
        self.Hq, self.Hkv, self.D, self.B, self.dtype, self.select_mode = Hq, Hkv, D, B, dtype, select_mode
        self.layout = sb_get_layout(self)

    def ref(self):
        return C.byref(self.c)


def sb_get_layout(pb: Problem) -> sb_layout:
    out = sb_layout()
    _check(lib().sb_get_layout(pb.ref(), C.byref(out)))
    return out


def sb_keep_ratio_to_topk(cu_seqlens, block_size, keep_ratio) -> np.ndarray:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    rho = np.ascontiguousarray(keep_ratio, dtype=np.float32)
    out = np.zeros(len(rho), dtype=np.int32)
    _check(lib().sb_keep_ratio_to_topk(_ptr(cu), len(rho), block_size, _ptr(rho), _ptr(out)))
    return out


def sb_sel_rowptr_host(pb: Problem) -> np.ndarray:
    out = np.zeros(pb.layout.sel_rows + 1, dtype=np.int32)
    _check(lib().sb_sel_rowptr_host(pb.ref(), _ptr(out)))
    return out


def _bytes(n, device):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


def sb_block_scores(pb: Problem, q, k, want_kbar=False, ws=None):
    lay = pb.layout
    scores = torch.empty(max(lay.scores_elems, 1), dtype=torch.float32, device=q.device)
    kbar = torch.empty(max(lay.pooled_elems, 1), dtype=torch.float32, device=q.device) if want_kbar else None
    ws = ws if ws is not None else _bytes(lay.scores_ws_bytes, q.device)
    _check(lib().sb_block_scores(pb.ref(), _ptr(q), _ptr(k), _ptr(kbar), _ptr(scores), _ptr(ws), _stream()))
    return (scores, kbar) if want_kbar else scores


def sb_select_topk(pb: Problem, scores, ws=None):
    lay = pb.layout
    rowptr = torch.empty(lay.sel_rows + 1, dtype=torch.int32, device=scores.device)
    idx = torch.empty(max(lay.sel_nnz, 1), dtype=torch.int32, device=scores.device)
    ws = ws if ws is not None else _bytes(lay.select_ws_bytes, scores.device)
    _check(lib().sb_select_topk(pb.ref(), _ptr(scores), _ptr(rowptr), _ptr(idx), _ptr(ws), _stream()))
    return rowptr, idx


def sb_select_topk_static(pb: Problem, scores, rowptr=None, idx=None):
    """sb_select_topk without a workspace argument (the library's built-in scratch); outputs may be passed in."""
    lay = pb.layout
    rowptr = rowptr if rowptr is not None else torch.empty(lay.sel_rows + 1, dtype=torch.int32, device=scores.device)
    idx = idx if idx is not None else torch.empty(max(lay.sel_nnz, 1), dtype=torch.int32, device=scores.device)
    _check(lib().sb_select_topk_static(pb.ref(), _ptr(scores), _ptr(rowptr), _ptr(idx), _stream()))
    return rowptr, idx


def sb_score_select(pb: Problem, q, k, ws=None, want_scores=True):
    """Scores and selection in one call; returns (scores, sel_rowptr, sel_idx); scores is None with want_scores=False
    (the single-kernel form that keeps the scores on chip)."""
    lay = pb.layout
    scores = torch.empty(max(lay.scores_elems, 1), dtype=torch.float32, device=q.device) if want_scores else None
    rowptr = torch.empty(lay.sel_rows + 1, dtype=torch.int32, device=q.device)
    idx = torch.empty(max(lay.sel_nnz, 1), dtype=torch.int32, device=q.device)
    ws = ws if ws is not None else _bytes(lay.scores_ws_bytes, q.device)
    _check(lib().sb_score_select(pb.ref(), _ptr(q), _ptr(k), None, _ptr(scores), _ptr(rowptr), _ptr(idx), _ptr(ws), _stream()))
    return scores, rowptr, idx


def sb_plan_worklist(pb: Problem, sel_rowptr, sel_idx, plan=None):
    plan = plan if plan is not None else _bytes(pb.layout.plan_bytes, sel_rowptr.device)
    _check(lib().sb_plan_worklist(pb.ref(), _ptr(sel_rowptr), _ptr(sel_idx), _ptr(plan), _stream()))
    return plan


def sb_sparse_attn_fwd(pb: Problem, q, k, v, sel_rowptr, sel_idx, plan, o=None, lse=None, ws=None):
    o = o if o is not None else torch.empty_like(q)
    lse = lse if lse is not None else torch.empty((pb.Hq, pb.T), dtype=torch.float32, device=q.device)
    ws = ws if ws is not None else _bytes(pb.layout.fwd_ws_bytes, q.device)
    _check(lib().sb_sparse_attn_fwd(pb.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(sel_rowptr), _ptr(sel_idx), _ptr(plan),
                                    _ptr(o), _ptr(lse), _ptr(ws), _stream()))
    return o, lse


def sb_sparse_attn_bwd(pb: Problem, q, k, v, o, lse, d_o, sel_rowptr, sel_idx, plan, dq=None, dk=None, dv=None, ws=None):
    dq = dq if dq is not None else torch.empty_like(q)
    dk = dk if dk is not None else torch.empty_like(k)
    dv = dv if dv is not None else torch.empty_like(v)
    ws = ws if ws is not None else _bytes(pb.layout.bwd_ws_bytes, q.device)
    _check(lib().sb_sparse_attn_bwd(pb.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(sel_rowptr),
                                    _ptr(sel_idx), _ptr(plan), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), _stream()))
    return dq, dk, dv


SB_ANCHOR_MIN, SB_ANCHOR_MEAN, SB_ANCHOR_MAX = 0, 1, 2


def sb_score_coverage(pb: Problem, scores, ws=None):
    """Coverage curves C_s(k) of the routing scores: NQB floats on the device."""
    cov = torch.empty(max(pb.layout.num_qblocks, 1), dtype=torch.float32, device=scores.device)
    ws = ws if ws is not None else _bytes(pb.layout.coverage_ws_bytes, scores.device)
    _check(lib().sb_score_coverage(pb.ref(), _ptr(scores), _ptr(cov), _ptr(ws), _stream()))
    return cov


class PerfTable:
    """Holds sb_perf_table plus the host arrays it points to."""

    def __init__(self, lengths, budgets, latency):
        self.lengths = np.ascontiguousarray(lengths, dtype=np.float32)
        self.budgets = np.ascontiguousarray(budgets, dtype=np.float32)
        self.latency = np.ascontiguousarray(latency, dtype=np.float32).reshape(len(self.lengths), len(self.budgets))
        self.c = sb_perf_table(len(self.lengths), len(self.budgets), self.lengths.ctypes.data, self.budgets.ctypes.data,
                               self.latency.ctypes.data)

    def ref(self):
        return C.byref(self.c)

    @classmethod
    def from_json(cls, path):
        """A table written by paper_2604_13847_amd/profile_latency.py."""
        import json
        with open(path) as f:
            j = json.load(f)
        return cls(j["lengths"], j["budgets"], j["latency_ms"])


def sb_perf_predict(tab: PerfTable, length, budget) -> float:
    out = C.c_double()
    _check(lib().sb_perf_predict(tab.ref(), C.c_double(length), C.c_double(budget), C.byref(out)))
    return out.value


def sb_perf_align(tab: PerfTable, length, target, max_budget) -> int:
    out = C.c_int32()
    _check(lib().sb_perf_align(tab.ref(), C.c_double(length), C.c_double(target), int(max_budget), C.byref(out)))
    return out.value


def sb_dst_tune(pb: Problem, coverage_host, tab: PerfTable, anchor, threshold_p):
    """Algorithm 1 for every sequence; pb's topk are the base budgets.  Returns (k_final, k_anchor, T_anchor)."""
    cov = np.ascontiguousarray(coverage_host, dtype=np.float32)
    kf, ka = np.zeros(max(pb.S, 1), dtype=np.int32), np.zeros(max(pb.S, 1), dtype=np.int32)
    ta = C.c_double()
    _check(lib().sb_dst_tune(pb.ref(), _ptr(cov), tab.ref(), int(anchor), C.c_double(threshold_p), _ptr(kf), _ptr(ka), C.byref(ta)))
    return kf[: pb.S], ka[: pb.S], ta.value


class SparsityPredictor:
    """Spar of Algorithm 2: per length bin, a moving average of the budgets the tuning step produced."""

    def __init__(self, bin_edges, decay=0.9):
        self.edges = np.ascontiguousarray(bin_edges, dtype=np.float32)
        self.nb = len(self.edges) - 1
        self.ema = np.zeros(self.nb, dtype=np.float32)
        self.seen = np.zeros(self.nb, dtype=np.uint8)
        self.decay = float(decay)

    def update(self, lengths, k_final):
        L, k = np.ascontiguousarray(lengths, dtype=np.int32), np.ascontiguousarray(k_final, dtype=np.int32)
        _check(lib().sb_spar_update(_ptr(self.ema), _ptr(self.seen), _ptr(self.edges), self.nb, C.c_double(self.decay), _ptr(L), _ptr(k), len(L)))

    def predict(self, length, k_base) -> float:
        out = C.c_double()
        _check(lib().sb_spar_predict(_ptr(self.ema), _ptr(self.seen), _ptr(self.edges), self.nb, int(length), C.c_double(k_base), C.byref(out)))
        return out.value


def sb_balanced_partition(weights, num_bins) -> np.ndarray:
    w = np.ascontiguousarray(weights, dtype=np.float64)
    out = np.zeros(max(len(w), 1), dtype=np.int32)
    _check(lib().sb_balanced_partition(_ptr(w), len(w), int(num_bins), _ptr(out)))
    return out[: len(w)]


def sb_sab_batches(tab: PerfTable, lengths, k_pred, dp_size, dp_rank, num_microbatches):
    """Algorithm 2.  Returns (weights, dp_bin_of, mb_bin_of)."""
    L, k = np.ascontiguousarray(lengths, dtype=np.int32), np.ascontiguousarray(k_pred, dtype=np.float64)
    n = len(L)
    w, dp, mb = np.zeros(max(n, 1)), np.zeros(max(n, 1), dtype=np.int32), np.zeros(max(n, 1), dtype=np.int32)
    _check(lib().sb_sab_batches(tab.ref(), _ptr(L), _ptr(k), n, int(dp_size), int(dp_rank), int(num_microbatches), _ptr(w), _ptr(dp), _ptr(mb)))
    return w[:n], dp[:n], mb[:n]


SB_INSTR_CU_BUSY, SB_INSTR_KERNEL_EVENTS = 1, 2
KERNEL_NAMES = ["pool", "score", "topk", "plan", "fwd", "bwd_prep", "bwd_dq", "bwd_dkv", "coverage", "score_select"]


def sb_set_instrumentation(flag: int):
    _check(lib().sb_set_instrumentation(int(flag)))


def sb_read_kernel_times():
    """{kernel: (total_ms, launches)} since the last call."""
    ms = np.zeros(len(KERNEL_NAMES), dtype=np.float64)
    cnt = np.zeros(len(KERNEL_NAMES), dtype=np.int64)
    _check(lib().sb_read_kernel_times(_ptr(ms), _ptr(cnt)))
    return {n: (float(ms[i]), int(cnt[i])) for i, n in enumerate(KERNEL_NAMES)}


def sb_read_cu_busy(ws) -> np.ndarray:
    out = np.zeros(SB_CU_SLOTS, dtype=np.uint64)
    _check(lib().sb_read_cu_busy(_ptr(ws), _ptr(out), _stream()))
    return out


def sb_version() -> str:
    return lib().sb_version().decode()


# ------------------------------------------------------------------ plan inspection (tests only)
_PLAN_KEYS = ["qb_off", "bm_off", "qb_seq", "work_fwd", "colcost", "bitmap", "bwd_items", "counters", "split_cols",
              "bwd_items_count", "split_weight", "split_max"]


def plan_views(pb: Problem, plan: torch.Tensor):
    """Decode the opaque plan for property tests, from the section offsets the library reports.  Everything is at the
    granularity of 64-token tiles (NT of them), whatever the selection block size."""
    sec = np.zeros(len(_PLAN_KEYS), dtype=np.int64)
    _check(lib().sb_plan_sections(pb.ref(), _ptr(sec)))
    o = dict(zip(_PLAN_KEYS, (int(x) for x in sec)))
    S, Hkv = pb.S, pb.Hkv
    raw = plan.cpu().numpy()

    def view(start, count, dt):
        return raw[start:start + count * np.dtype(dt).itemsize].view(dt)

    qb_off = view(o["qb_off"], S + 1, np.int32)
    NT = int(qb_off[-1])
    Hs = pb.layout.sel_heads
    counters = view(o["counters"], 2, np.int32)
    return {
        "qb_off": qb_off, "bm_off": view(o["bm_off"], S + 1, np.int64), "qb_seq": view(o["qb_seq"], NT, np.int32),
        "work_fwd": view(o["work_fwd"], Hs * NT, np.int32), "colcost": view(o["colcost"], Hkv * NT, np.int32),
        "bitmap": raw[o["bitmap"]:o["bwd_items"]].view(np.uint32),
        "bwd_items": view(o["bwd_items"], 4 * o["bwd_items_count"], np.int32).reshape(-1, 4),
        "slots_used": int(counters[0]), "split_cols": view(o["split_cols"], 3 * int(counters[1]), np.int32).reshape(-1, 3),
        "split_weight": o["split_weight"], "split_max": o["split_max"],
    }
