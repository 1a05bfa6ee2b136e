#!/usr/bin/env python3
"""Benchmark of the block-sparse attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic packed batch: routing scores -> top-k
selection -> work plan -> sparse attention forward -> backward, through the C-ABI library.
Prints ONE JSON line: effective TFLOP/s over the selected blocks (14*D*pairs*Hq per step, the
diagonal block counted as its causal triangle), the roofline of the dominant kernel measured with
HIP events on the launch stream, and the CPU checker timed on a bounded sample of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
# HBM bytes per launch of the attention kernels on cfg2 / per_qhead from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# (scaled as described in profiles/attn_kernels_cfg2_per_qhead_hbm_traffic.txt); None for other workloads.
MEASURED_TRAFFIC_BYTES = {("cfg2", "per_qhead"): {"fwd": 1.003e9 + 0.273e9, "bwd_dq": 1.982e9 + 0.277e9, "bwd_dkv": 8.940e9 + 0.135e9}}


def make_workload(name, seed):
    from paper_2604_13847_amd import synth
    return {"cfg1": synth.config1, "cfg2": synth.config2, "cfg3": synth.config3, "cfg4": synth.config4,
            "cfg5": synth.config5, "blk256": synth.config_block256, "d64": synth.config_d64}[name](seed)


def cpu_baseline(w, host, opb, topk, rowptr_h, idx_h, scale, budget_s=15.0):
    """The CPU checker, as it stands, on a bounded random sample of query rows (forward + the row's
    full backward arithmetic); throughput in the same effective-flop unit."""
    from oracle import oracle as orc
    rng = np.random.default_rng(0)
    G = w.Hq // w.Hkv
    cu = w.cu
    # per-row pair counts from the selection
    def sample(n):
        toks = rng.integers(0, w.T, size=n).astype(np.int32)
        heads = rng.integers(0, w.Hq, size=n).astype(np.int32)
        return toks, heads
    def pairs_of(toks, heads):
        tot = 0
        seq = np.searchsorted(cu, toks, side="right") - 1
        for t, h, s in zip(toks, heads, seq):
            r = int(t - cu[s]); i = r // w.B
            hs = h if opb.mode == 0 else h // G
            row = hs * opb.NQB + int(opb.qb_off[s]) + i
            c = int(rowptr_h[row + 1] - rowptr_h[row])
            tot += (c - 1) * w.B + (r - i * w.B + 1)
        return tot
    q, k, v, do = host
    toks, heads = sample(64)
    t0 = time.perf_counter()
    orc.attn_rows(opb, q, k, v, do, rowptr_h, idx_h, scale, toks, heads)
    dt = time.perf_counter() - t0
    n = int(min(max(64, 64 * budget_s / max(dt, 1e-4)), 200000))
    toks, heads = sample(n)
    t0 = time.perf_counter()
    orc.attn_rows(opb, q, k, v, do, rowptr_h, idx_h, scale, toks, heads)
    dt = time.perf_counter() - t0
    flops = 14.0 * w.D * pairs_of(toks, heads)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{n} random (token, head) query rows of the same batch, forward + row backward, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--mode", default="per_qhead", choices=["per_qhead", "per_kvgroup"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cu-busy", action="store_true", help="(default) also report the per-CU busy-time spread")
    ap.add_argument("--no-cu-busy", action="store_true", help="skip the two instrumented launches that measure the per-CU busy-time spread")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_13847_amd import binding as sb
    from paper_2604_13847_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = make_workload(args.workload, args.seed)
    mode = sb.SB_SELECT_PER_QHEAD if args.mode == "per_qhead" else sb.SB_SELECT_PER_KVGROUP
    topk = w.topk if w.topk is not None else sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
    dt_code = sb.SB_BF16 if w.dtype == "bf16" else sb.SB_F32
    pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, dtype=dt_code, select_mode=mode, device=dev)
    lay = pb.layout
    t = w.tensors()

    def up(x):
        if w.dtype == "bf16":
            return torch.from_numpy(synth.bf16_bits(x)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)
    q, k, v, do = (up(t[n]) for n in ("q", "k", "v", "do"))

    # every buffer is allocated once, outside the timed region
    def raw(nbytes):
        return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)
    ws_scores, ws_fwd, ws_bwd = raw(lay.scores_ws_bytes), raw(lay.fwd_ws_bytes), raw(lay.bwd_ws_bytes)
    plan = raw(lay.plan_bytes)
    o, lse = torch.empty_like(q), torch.empty((w.Hq, w.T), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    L = sb.lib()
    import ctypes as C
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    scores = torch.empty(max(lay.scores_elems, 1), dtype=torch.float32, device=dev)
    rowptr = torch.empty(lay.sel_rows + 1, dtype=torch.int32, device=dev)
    idx = torch.empty(max(lay.sel_nnz, 1), dtype=torch.int32, device=dev)
    P = lambda x: C.c_void_p(x.data_ptr())

    def step():
        rc = L.sb_score_select(pb.ref(), P(q), P(k), None, P(scores), P(rowptr), P(idx), P(ws_scores), st)
        rc |= L.sb_plan_worklist(pb.ref(), P(rowptr), P(idx), P(plan), st)
        rc |= L.sb_sparse_attn_fwd(pb.ref(), P(q), P(k), P(v), P(rowptr), P(idx), P(plan), P(o), P(lse), P(ws_fwd), st)
        rc |= L.sb_sparse_attn_bwd(pb.ref(), P(q), P(k), P(v), P(o), P(lse), P(do), P(rowptr), P(idx), P(plan),
                                   P(dq), P(dk), P(dv), P(ws_bwd), st)
        if rc != 0:
            raise RuntimeError(L.sb_last_error().decode())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    sb.sb_set_instrumentation(sb.SB_INSTR_KERNEL_EVENTS)
    sb.sb_read_kernel_times()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ktimes = sb.sb_read_kernel_times()
    sb.sb_set_instrumentation(0)

    pairs = lay.attended_pairs_per_head_sum                 # summed over query heads
    flops_step = 14.0 * w.D * pairs
    ms_step = elapsed / args.steps * 1e3
    value = flops_step / (ms_step * 1e-3) / 1e12
    kavg = {n: (ms / c if c else 0.0) for n, (ms, c) in ktimes.items()}
    # contractions each attention kernel cannot avoid, in units of 2*D*pairs flops
    contractions = {"fwd": 2, "bwd_dq": 3, "bwd_dkv": 4}
    dom = max(contractions, key=lambda n: kavg[n])
    dom_flops = contractions[dom] * 2.0 * w.D * pairs
    achieved = dom_flops / (kavg[dom] * 1e-3) / 1e12
    attn_ms = kavg["fwd"] + kavg["bwd_prep"] + kavg["bwd_dq"] + kavg["bwd_dkv"]

    out = {
        "metric": "sparse-attn fwd+bwd effective TFLOP/s (selected blocks) + % bf16 MFMA peak",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: packed varlen T={w.T} S={w.S} Hq={w.Hq} Hkv={w.Hkv} D={w.D} block={w.B} "
                               f"causal, per-sequence budgets {topk.tolist() if len(topk) <= 16 else str(topk[:8].tolist()) + '...'}",
                   "select_mode": args.mode, "seed": args.seed, "pairs_per_step": int(pairs),
                   "flops_per_step": flops_step, "selected_tiles": int(lay.sel_nnz)},
        "pct_of_bf16_mfma_peak": round(100.0 * value / BF16_MFMA_PEAK_TFLOPS, 3),
        "attention_only": {"ms": round(attn_ms, 4), "tflops": round(flops_step / (attn_ms * 1e-3) / 1e12, 3)},
        "kernel_ms": {n: round(x, 4) for n, x in kavg.items()},
        "roofline": {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 3), "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 5),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, args.mode), {}).get(dom),
                     "flops_per_launch": dom_flops, "avg_launch_ms": round(kavg[dom], 4)},
    }

    if not args.no_cu_busy:  # outside the timed region: one instrumented forward and one instrumented backward
        spreads = {}
        for name, call in (("fwd", lambda: L.sb_sparse_attn_fwd(pb.ref(), P(q), P(k), P(v), P(rowptr), P(idx), P(plan), P(o), P(lse), P(ws_fwd), st)),
                           ("bwd", lambda: L.sb_sparse_attn_bwd(pb.ref(), P(q), P(k), P(v), P(o), P(lse), P(do), P(rowptr), P(idx), P(plan), P(dq), P(dk), P(dv), P(ws_bwd), st))):
            sb.sb_set_instrumentation(sb.SB_INSTR_CU_BUSY)
            call()
            busy = sb.sb_read_cu_busy(ws_fwd if name == "fwd" else ws_bwd).astype(np.float64)
            sb.sb_set_instrumentation(0)
            busy = busy[busy > 0]
            spreads[name] = {"cus": int(busy.size), "spread_max_minus_min_over_mean": round(float((busy.max() - busy.min()) / busy.mean()), 4),
                             "max_over_mean": round(float(busy.max() / busy.mean()), 4)}
        out["cu_busy"] = spreads

    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        opb = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, mode)
        host = tuple(t[n] if w.dtype == "bf16" else synth.round_to_bf16(t[n]) for n in ("q", "k", "v", "do"))
        rp_h = rowptr.cpu().numpy()
        out["cpu_baseline"] = cpu_baseline(w, host, opb, topk, rp_h, idx.cpu().numpy()[: int(rp_h[-1])], 1.0 / np.sqrt(w.D))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
