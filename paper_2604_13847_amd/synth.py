"""Seeded synthetic inputs for block-sparse attention workloads.

This module draws numbers and nothing else: it holds no arithmetic of the
attention method (no pooling, scoring, selection, softmax, budget rule).  Both
the GPU tests and the CPU checker take their inputs from here so that the two
sides see identical bits.

Generator: a counter-based hash.  Element `i` of tensor `tid` under `seed` is a
function of (seed, tid, i) only, so any slice can be regenerated without state
and the draw does not depend on torch's or numpy's RNG.
  z = mix64(seed * C0 + tid * C1 + i)            (the splitmix64 finaliser)
  u1 = (top 24 bits + 0.5) / 2^24, u2 = (low 24 bits + 0.5) / 2^24
  n  = sqrt(-2 ln u1) * cos(2 pi u2)              (Box-Muller, one normal per counter)

Workload shapes stand in for the paper's long-context data mixes (60 % short /
40 % long packed sequences, bimodal and long-tailed length histograms; paper
sections 1 and 3.1); the datasets themselves are not used.
"""
from __future__ import annotations

import numpy as np

_C0 = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xD1B54A32D192ED03)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# tensor ids
TID_Q, TID_K, TID_V, TID_DO, TID_LEN, TID_RATIO, TID_MISC = 1, 2, 3, 4, 5, 6, 7


def _mix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
        x = x ^ (x >> np.uint64(31))
    return x


def raw_u64(seed: int, tid: int, start: int, count: int) -> np.ndarray:
    """64 hashed bits for counters start .. start+count-1 of stream (seed, tid)."""
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * _C0 + np.uint64(tid) * _C1
        ctr = np.arange(start, start + count, dtype=np.uint64) + base
    return _mix64(ctr)


def uniform01(seed: int, tid: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in (0,1) with 53-bit resolution from the top bits."""
    z = raw_u64(seed, tid, start, count)
    return ((z >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal_chunk(args):
    seed, tid, s, n, out, to_bf16 = args
    inv = 1.0 / 16777216.0
    z = raw_u64(seed, tid, s, n)
    u1 = ((z >> np.uint64(40)).astype(np.float64) + 0.5) * inv
    u2 = ((z & np.uint64(0xFFFFFF)).astype(np.float64) + 0.5) * inv
    x = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    out[s:s + n] = round_to_bf16(x) if to_bf16 else x


def normal_f32(seed: int, tid: int, count: int, chunk: int = 1 << 18, to_bf16: bool = False) -> np.ndarray:
    """`count` i.i.d. N(0,1) values as float32 (computed in float64, then rounded; with `to_bf16`
    rounded once more to the nearest bfloat16 value).  Chunks are independent (counter-based), so
    they are filled by a small thread pool, each chunk small enough to stay in cache."""
    out = np.empty(count, dtype=np.float32)
    jobs = [(seed, tid, s, min(chunk, count - s), out, to_bf16) for s in range(0, count, chunk)]
    if len(jobs) <= 1:
        for j in jobs:
            _normal_chunk(j)
        return out
    from concurrent.futures import ThreadPoolExecutor
    import os
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(_normal_chunk, jobs))
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returns float32 holding bf16 values."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        y = (b + r) & np.uint32(0xFFFF0000)
    nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    y = np.where(nan, b | np.uint32(0x00400000), y).astype(np.uint32)
    return y.view(np.float32).reshape(x.shape)


def bf16_bits(x_bf16_valued: np.ndarray) -> np.ndarray:
    """The 16-bit patterns (as int16) of a float32 array that already holds bf16 values."""
    b = np.ascontiguousarray(x_bf16_valued, dtype=np.float32).view(np.uint32)
    return (b >> np.uint32(16)).astype(np.uint16).view(np.int16).reshape(x_bf16_valued.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Inverse of bf16_bits: int16/uint16 patterns -> float32 values."""
    u = np.ascontiguousarray(bits).view(np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).reshape(bits.shape)


def _randint(seed: int, tid: int, ctr: int, lo: int, hi: int) -> int:
    """Uniform integer in [lo, hi] from counter ctr."""
    u = float(uniform01(seed, tid, ctr, 1)[0])
    return lo + min(int(u * (hi - lo + 1)), hi - lo)


def mixed_lengths(seed: int, total: int, short=(512, 4096), long=(8192, 16384), p_short=0.6):
    """Sequence lengths drawn until `total` tokens are filled; the last draw is truncated."""
    lens, filled, c = [], 0, 0
    while filled < total:
        pick = float(uniform01(seed, TID_LEN, c, 1)[0]); c += 1
        lo, hi = short if pick < p_short else long
        L = _randint(seed, TID_LEN, c, lo, hi); c += 1
        L = min(L, total - filled)
        lens.append(L); filled += L
    return lens


def cu_from_lengths(lens) -> np.ndarray:
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return cu


class Workload:
    """Shape of one problem instance.  Exactly one of `keep_ratio` / `topk` is set."""

    def __init__(self, name, lens, Hq, Hkv, D, B=64, keep_ratio=None, topk=None, dtype="bf16", seed=0):
        self.name, self.seed = name, seed
        self.lens = list(lens)
        self.cu = cu_from_lengths(self.lens)
        self.T, self.S = int(self.cu[-1]), len(self.lens)
        self.Hq, self.Hkv, self.D, self.B = Hq, Hkv, D, B
        self.keep_ratio = None if keep_ratio is None else np.asarray(keep_ratio, dtype=np.float32)
        self.topk = None if topk is None else np.asarray(topk, dtype=np.int32)
        self.dtype = dtype

    def tensors(self):
        """Q, K, V, dO as float32 arrays; values are bf16-representable when dtype == 'bf16'."""
        shp_q, shp_k = (self.T, self.Hq, self.D), (self.T, self.Hkv, self.D)
        out = {}
        for name, tid, shp in (("q", TID_Q, shp_q), ("k", TID_K, shp_k), ("v", TID_V, shp_k), ("do", TID_DO, shp_q)):
            out[name] = normal_f32(self.seed, tid, int(np.prod(shp)), to_bf16=self.dtype == "bf16").reshape(shp)
        return out

    def __repr__(self):
        return (f"Workload({self.name}, S={self.S}, T={self.T}, Hq={self.Hq}, Hkv={self.Hkv}, "
                f"D={self.D}, B={self.B}, dtype={self.dtype}, seed={self.seed})")


def _ratios(seed, S, lo, hi, first_ctr=0):
    u = uniform01(seed, TID_RATIO, first_ctr, S)
    return (lo + (hi - lo) * u).astype(np.float32)


def config1(seed=0):
    """Single sequence L=1024, 1/1 heads, D=64, fp32 inputs, top-k 4."""
    return Workload("cfg1", [1024], 1, 1, 64, topk=[4], dtype="f32", seed=seed)


def config2(seed=0, total=32768):
    """Packed varlen 60/40 short/long mix, 32/8 heads, D=128, keep ratio U[0.1,0.5]."""
    lens = mixed_lengths(seed, total)
    return Workload("cfg2", lens, 32, 8, 128, keep_ratio=_ratios(seed, len(lens), 0.1, 0.5), seed=seed)


def config3(seed=0, total=65536):
    """As config2 with length ranges doubled, 28/4 heads, keep ratio U[0.05,0.3]."""
    lens = mixed_lengths(seed, total, short=(1024, 8192), long=(16384, 32768))
    return Workload("cfg3", lens, 28, 4, 128, keep_ratio=_ratios(seed, len(lens), 0.05, 0.3), seed=seed)


def config4(seed=0, L=131072):
    """Single long sequence, 32/8 heads, fixed top-k 32."""
    return Workload("cfg4", [L], 32, 8, 128, topk=[32], seed=seed)


def config5(seed=0, total=262144, long_len=131072, long_first=True):
    """One long sequence (keep 0.05) plus short sequences U{256..2048} (keep U[0.5,1.0])."""
    lens, filled, c = [], long_len, 0
    while filled < total:
        L = min(_randint(seed, TID_LEN, c, 256, 2048), total - filled); c += 1
        lens.append(L); filled += L
    rs = _ratios(seed, len(lens), 0.5, 1.0)
    if long_first:
        lens, ratios = [long_len] + lens, np.concatenate([[np.float32(0.05)], rs])
    else:
        lens, ratios = lens + [long_len], np.concatenate([rs, [np.float32(0.05)]])
    return Workload("cfg5", lens, 32, 8, 128, keep_ratio=ratios.astype(np.float32), seed=seed)


def config_block256(seed=0, total=65536):
    """The block size and budget of the paper's own runs (section 5: MoBA with block 256, top-k 32) on the 60/40
    length mix of config3, with the head shape of Qwen2.5-3B (16 query heads on 2 KV heads, head_dim 128)."""
    lens = mixed_lengths(seed, total, short=(1024, 8192), long=(16384, 32768))
    return Workload("blk256", lens, 16, 2, 128, B=256, topk=[32] * len(lens), seed=seed)


def config_d64(seed=0, total=65536):
    """As config_block256 with the head shape of Qwen2.5-0.5B, the smaller model of the paper's runs (section 5):
    14 query heads on 2 KV heads, head_dim 64."""
    lens = mixed_lengths(seed, total, short=(1024, 8192), long=(16384, 32768))
    return Workload("d64", lens, 14, 2, 64, B=256, topk=[32] * len(lens), seed=seed)


def small_ragged(seed=0, lens=(200, 64, 1, 130, 77), Hq=4, Hkv=2, D=64, B=64, ratio=(0.3, 1.0), dtype="bf16"):
    """A small packed batch with ragged tails, several tiles per sequence; for element-wise parity."""
    return Workload("small", list(lens), Hq, Hkv, D, B=B,
                    keep_ratio=_ratios(seed, len(lens), ratio[0], ratio[1]), dtype=dtype, seed=seed)


def sink_selection(cu, B, topk, Hs):
    """A caller-supplied selection with the shape real attention maps have (an "attention sink" plus a local window):
    query block i of a sequence with budget k keeps block 0, the diagonal block and the blocks right before it, c =
    min(k, i + 1) blocks in all.  Every selection head gets the same rows.  Returns (rowptr [Hs*NQB+1], idx) in the CSR
    layout of the library (rows ordered by selection head, then sequence, then query block; entries ascending).  Block 0
    of a long sequence is then kept by every query block: the heaviest possible key-major column."""
    cu = np.asarray(cu, dtype=np.int64)
    rows_c, rows_i = [], []
    for s in range(len(cu) - 1):
        n = int((cu[s + 1] - cu[s] + B - 1) // B)
        i = np.arange(n, dtype=np.int64)
        rows_i.append(i)
        rows_c.append(np.minimum(int(min(max(int(topk[s]), 1), max(n, 1))), i + 1))
    c = np.concatenate(rows_c) if rows_c else np.zeros(0, dtype=np.int64)
    i = np.concatenate(rows_i) if rows_i else np.zeros(0, dtype=np.int64)
    start = np.concatenate([[0], np.cumsum(c)])
    nnz = int(start[-1])
    row_of = np.repeat(np.arange(len(c)), c)
    pos = np.arange(nnz) - start[row_of]                       # position inside the row
    ci, ii = c[row_of], i[row_of]
    idx1 = np.where(pos == 0, np.where(ci == ii + 1, 0, np.where(ci == 1, ii, 0)), ii - (ci - 1) + pos)
    rowptr = np.concatenate([(start[:-1][None, :] + nnz * np.arange(Hs)[:, None]).reshape(-1), [nnz * Hs]])
    return rowptr.astype(np.int32), np.tile(idx1, Hs).astype(np.int32)
