"""ctypes front end of the C checker in sparsebal_oracle.c (test infrastructure only).

Every function takes float32 numpy arrays (already rounded to the storage type under test)
and returns float64 results.  See the C file for the definitions and their citations.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build_oracle

MODE_PER_QHEAD, MODE_PER_KVGROUP = 0, 1


class _Shape(C.Structure):
    _fields_ = [("T", C.c_int32), ("S", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("B", C.c_int32), ("mode", C.c_int32), ("cu", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_oracle())
        _lib.orc_num_qblocks.restype = C.c_int64
        _lib.orc_scores_elems.restype = C.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Problem:
    """Shape + cu_seqlens holder; keeps the arrays alive for the C calls."""

    def __init__(self, cu, Hq, Hkv, D, B=64, mode=MODE_PER_QHEAD):
        self.cu = _i32(cu)
        self.S, self.T = len(self.cu) - 1, int(self.cu[-1])
        self.Hq, self.Hkv, self.D, self.B, self.mode = Hq, Hkv, D, B, mode
        self.Hs = Hq if mode == MODE_PER_QHEAD else Hkv
        self.sh = _Shape(self.T, self.S, Hq, Hkv, D, B, mode, self.cu.ctypes.data)
        self.nblk = [(int(self.cu[s + 1] - self.cu[s]) + B - 1) // B for s in range(self.S)]
        self.NQB = int(sum(self.nblk))
        self.qb_off = np.concatenate([[0], np.cumsum(self.nblk)]).astype(np.int64)
        self.score_off = (np.concatenate([[0], np.cumsum([n * n for n in self.nblk])]) * self.Hs).astype(np.int64)

    def ref(self):
        return C.byref(self.sh)


def keep_ratio_to_topk(cu, B, rho):
    cu, rho = _i32(cu), _f32(rho)
    out = np.zeros(len(rho), dtype=np.int32)
    lib().orc_keep_ratio_to_topk(_p(cu), len(rho), B, _p(rho), _p(out))
    return out


def block_mean(pb: Problem, X):
    X = _f32(X)
    H = X.shape[1]
    out = np.zeros((pb.NQB, H, pb.D), dtype=np.float64)
    assert lib().orc_block_mean(pb.ref(), _p(X), H, _p(out)) == 0
    return out


def block_scores(pb: Problem, Q, K, score_scale):
    Q, K = _f32(Q), _f32(K)
    out = np.zeros(int(pb.score_off[-1]), dtype=np.float64)
    assert lib().orc_block_scores(pb.ref(), _p(Q), _p(K), C.c_double(score_scale), _p(out)) == 0
    return out


def block_scores_row(pb: Problem, Q, K, score_scale, s, hs, i):
    Q, K = _f32(Q), _f32(K)
    out = np.zeros(pb.nblk[s], dtype=np.float64)
    assert lib().orc_block_scores_row(pb.ref(), _p(Q), _p(K), C.c_double(score_scale), s, hs, i, _p(out)) == 0
    return out


def sel_rowptr(pb: Problem, topk):
    topk = _i32(topk)
    out = np.zeros(pb.Hs * pb.NQB + 1, dtype=np.int32)
    assert lib().orc_sel_rowptr(pb.ref(), _p(topk), _p(out)) == 0
    return out


def select_topk(pb: Problem, scores_f32, topk):
    """scores_f32: the float32 score array the decision is taken on.  Returns (rowptr, idx)."""
    scores, topk = _f32(scores_f32), _i32(topk)
    rowptr = sel_rowptr(pb, topk)
    idx = np.zeros(max(int(rowptr[-1]), 1), dtype=np.int32)
    assert lib().orc_select_topk(pb.ref(), _p(scores), _p(topk), _p(rowptr), _p(idx)) == 0
    return rowptr, idx[: int(rowptr[-1])]


def attn_fwd(pb: Problem, Q, K, V, rowptr, idx, scale):
    Q, K, V, rowptr, idx = _f32(Q), _f32(K), _f32(V), _i32(rowptr), _i32(idx)
    O = np.zeros((pb.T, pb.Hq, pb.D), dtype=np.float64)
    LSE = np.zeros((pb.Hq, pb.T), dtype=np.float64)
    assert lib().orc_attn_fwd(pb.ref(), _p(Q), _p(K), _p(V), _p(rowptr), _p(idx), C.c_double(scale), _p(O), _p(LSE)) == 0
    return O, LSE


def attn_bwd(pb: Problem, Q, K, V, dO, rowptr, idx, scale):
    Q, K, V, dO, rowptr, idx = _f32(Q), _f32(K), _f32(V), _f32(dO), _i32(rowptr), _i32(idx)
    dQ = np.zeros((pb.T, pb.Hq, pb.D), dtype=np.float64)
    dK = np.zeros((pb.T, pb.Hkv, pb.D), dtype=np.float64)
    dV = np.zeros((pb.T, pb.Hkv, pb.D), dtype=np.float64)
    assert lib().orc_attn_bwd(pb.ref(), _p(Q), _p(K), _p(V), _p(dO), _p(rowptr), _p(idx), C.c_double(scale),
                              _p(dQ), _p(dK), _p(dV)) == 0
    return dQ, dK, dV


def attn_rows(pb: Problem, Q, K, V, dO, rowptr, idx, scale, tokens, heads):
    """O, LSE and (if dO is given) dQ of the sampled (packed token, query head) rows."""
    Q, K, V, rowptr, idx = _f32(Q), _f32(K), _f32(V), _i32(rowptr), _i32(idx)
    dO = None if dO is None else _f32(dO)
    tokens, heads = _i32(tokens), _i32(heads)
    n = len(tokens)
    O = np.zeros((n, pb.D), dtype=np.float64)
    LSE = np.zeros(n, dtype=np.float64)
    dQ = np.zeros((n, pb.D), dtype=np.float64)
    assert lib().orc_attn_rows(pb.ref(), _p(Q), _p(K), _p(V), _p(dO), _p(rowptr), _p(idx), C.c_double(scale), n,
                               _p(tokens), _p(heads), _p(O), _p(LSE), _p(dQ)) == 0
    return O, LSE, (dQ if dO is not None else None)


def attn_bwd_kvblock(pb: Problem, Q, K, V, dO, rowptr, idx, scale, s, g, j):
    """dK, dV ([B][D] each) of key block j of sequence s, KV head g."""
    Q, K, V, dO, rowptr, idx = _f32(Q), _f32(K), _f32(V), _f32(dO), _i32(rowptr), _i32(idx)
    dK = np.zeros((pb.B, pb.D), dtype=np.float64)
    dV = np.zeros((pb.B, pb.D), dtype=np.float64)
    assert lib().orc_attn_bwd_kvblock(pb.ref(), _p(Q), _p(K), _p(V), _p(dO), _p(rowptr), _p(idx), C.c_double(scale),
                                      s, g, j, _p(dK), _p(dV)) == 0
    return dK, dV


def num_threads():
    return int(lib().orc_num_threads())
