#!/usr/bin/env python3
"""Benchmark of the block-sparse attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic packed batch: routing scores -> top-k
selection -> work plan -> sparse attention forward -> backward, through the C-ABI library, with
every input resident in HBM.  Prints ONE JSON line:
  value            effective TFLOP/s over the selected blocks (14*D*pairs*Hq per step, the diagonal
                   block counted as its causal triangle) on the default workload, the largest
                   single-GPU configuration (262144-token skewed batch, per-query-head selection)
  roofline         the dominant kernel against the bf16 matrix peak, its launch duration measured with
                   HIP events on the launch stream inside the timed region
  hbm              achieved GB/s of the pooling / scoring / selection kernels (HBM-bound steps)
  cu_busy          per-CU busy-time spread of the forward and the backward (Eq. 11 of the paper per CU)
  cpu_baseline     the CPU checker timed on a bounded sample of the same batch
  also             the same path on the 32768-token batch and in per-KV-group selection mode
"""
import argparse
import ctypes as C
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HBM_PEAK_GBPS = 8000.0


def make_workload(name, seed):
    from paper_2604_13847_amd import synth
    return {"cfg1": synth.config1, "cfg2": synth.config2, "cfg3": synth.config3, "cfg4": synth.config4,
            "cfg5": synth.config5, "blk256": synth.config_block256, "d64": synth.config_d64}[name](seed)


def measured_traffic(workload, mode, selection, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload, or None.  The
    summary holds lines `traffic_bytes_per_launch <kernel> <bytes>` written from FETCH_SIZE and WRITE_SIZE."""
    sel = "" if selection == "topk" else "_" + selection
    path = os.path.join(ROOT, "profiles", f"attn_kernels_{workload}_{mode}{sel}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"traffic_bytes_per_launch\s+(\S+)\s+([0-9.eE+]+)", line.strip())
        if m and m.group(1) == kernel:
            return float(m.group(2))
    return None


def cpu_baseline(w, host, opb, rowptr_h, idx_h, scale, budget_s=15.0):
    """The CPU checker, as it stands, on a bounded random sample of query rows (forward + the row's
    full backward arithmetic); throughput in the same effective-flop unit."""
    from oracle import oracle as orc
    rng = np.random.default_rng(0)
    G = w.Hq // w.Hkv
    cu = w.cu

    def sample(n):
        toks = rng.integers(0, w.T, size=n).astype(np.int32)
        heads = rng.integers(0, w.Hq, size=n).astype(np.int32)
        return toks, heads

    def pairs_of(toks, heads):  # per-row pair counts from the selection
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


def run(workload, mode_name, seed, steps, warmup, selection="topk", cu_busy=True, cpu=False, brief=False):
    import torch
    from paper_2604_13847_amd import binding as sb
    from paper_2604_13847_amd import synth

    dev = "cuda:0"
    w = make_workload(workload, seed)
    mode = sb.SB_SELECT_PER_QHEAD if mode_name == "per_qhead" else sb.SB_SELECT_PER_KVGROUP
    topk = w.topk if w.topk is not None else sb.sb_keep_ratio_to_topk(w.cu, w.B, w.keep_ratio)
    dt_code = sb.SB_BF16 if w.dtype == "bf16" else sb.SB_F32
    pb = sb.Problem(w.cu, topk, w.Hq, w.Hkv, w.D, w.B, dtype=dt_code, select_mode=mode, device=dev)
    lay = pb.layout
    key = (workload, seed)
    if run.cache.get("key") != key:          # the same values serve both selection modes
        run.cache.clear()
        run.cache.update(key=key, host=w.tensors())
    t = run.cache["host"]

    def up(x):
        if w.dtype == "bf16":
            return torch.from_numpy(synth.bf16_bits(x)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(x).to(dev)
    q, k, v, do = (up(t[n]) for n in ("q", "k", "v", "do"))

    def raw(nbytes):  # every buffer is allocated once, outside the timed region
        return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)
    ws_scores, ws_fwd, ws_bwd = raw(lay.scores_ws_bytes), raw(lay.fwd_ws_bytes), raw(lay.bwd_ws_bytes)
    plan = raw(lay.plan_bytes)
    o, lse = torch.empty_like(q), torch.empty((w.Hq, w.T), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    L = sb.lib()
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    scores = torch.empty(max(lay.scores_elems, 1), dtype=torch.float32, device=dev)
    rowptr = torch.empty(lay.sel_rows + 1, dtype=torch.int32, device=dev)
    idx = torch.empty(max(lay.sel_nnz, 1), dtype=torch.int32, device=dev)
    if selection == "sink":  # a caller-supplied selection: the scoring and selection calls are not part of the step
        rp_h, ix_h = synth.sink_selection(w.cu, w.B, topk, int(lay.sel_heads))
        assert len(ix_h) == lay.sel_nnz
        rowptr.copy_(torch.from_numpy(rp_h)); idx[: len(ix_h)].copy_(torch.from_numpy(ix_h))
    P = lambda x: C.c_void_p(x.data_ptr())

    def fwd():
        return L.sb_sparse_attn_fwd(pb.ref(), P(q), P(k), P(v), P(rowptr), P(idx), P(plan), P(o), P(lse), P(ws_fwd), st)

    def bwd():
        return L.sb_sparse_attn_bwd(pb.ref(), P(q), P(k), P(v), P(o), P(lse), P(do), P(rowptr), P(idx), P(plan),
                                    P(dq), P(dk), P(dv), P(ws_bwd), st)

    def step():
        rc = 0
        if selection == "topk":
            rc = L.sb_score_select(pb.ref(), P(q), P(k), None, P(scores), P(rowptr), P(idx), P(ws_scores), st)
        rc |= L.sb_plan_worklist(pb.ref(), P(rowptr), P(idx), P(plan), st)
        rc |= fwd()
        rc |= bwd()
        if rc != 0:
            raise RuntimeError(L.sb_last_error().decode())

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly `steps` steps, the library's per-kernel HIP events on (they come from a pool,
    # nothing is created in the loop), one torch event per step boundary for the median / min
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    sb.sb_set_instrumentation(sb.SB_INSTR_KERNEL_EVENTS)
    sb.sb_read_kernel_times()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ktimes = sb.sb_read_kernel_times()
    sb.sb_set_instrumentation(0)
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))

    pairs = lay.attended_pairs_per_head_sum                 # summed over query heads
    flops_step = 14.0 * w.D * pairs
    ms_step = elapsed / steps * 1e3
    value = flops_step / (ms_step * 1e-3) / 1e12
    k_step = {n: ms / steps for n, (ms, c) in ktimes.items()}                 # per step, all launches of the slot
    k_launch = {n: (ms / c if c else 0.0) for n, (ms, c) in ktimes.items()}   # per launch
    attn_ms = k_step["fwd"] + k_step["bwd_prep"] + k_step["bwd_dq"] + k_step["bwd_dkv"]
    res = {"workload": workload, "select_mode": mode_name, "value": round(value, 3), "ms_per_step": round(ms_step, 4),
           "ms_per_step_median": round(per_step[len(per_step) // 2], 4), "ms_per_step_min": round(per_step[0], 4),
           "pct_of_bf16_mfma_peak": round(100.0 * value / BF16_MFMA_PEAK_TFLOPS, 3),
           "kernel_ms": {n: round(x, 4) for n, x in k_step.items()}}
    if brief:
        return res
    # contractions each attention kernel cannot avoid in its role, in units of 2*D*pairs flops
    contractions = {"fwd": 2, "bwd_dq": 3, "bwd_dkv": 4}
    dom = max(contractions, key=lambda n: k_launch[n])
    dom_flops = contractions[dom] * 2.0 * w.D * pairs
    achieved = dom_flops / (k_launch[dom] * 1e-3) / 1e12
    res.update({
        "config": {"workload": f"{w.name}: packed varlen T={w.T} S={w.S} Hq={w.Hq} Hkv={w.Hkv} D={w.D} block={w.B} "
                               f"causal, per-sequence budgets {topk.tolist() if len(topk) <= 16 else str(topk[:8].tolist()) + '...'}",
                   "select_mode": mode_name, "selection": selection, "seed": seed, "pairs_per_step": int(pairs),
                   "flops_per_step": flops_step, "selected_tiles": int(lay.sel_nnz)},
        "attention_only": {"ms": round(attn_ms, 4), "tflops": round(flops_step / (attn_ms * 1e-3) / 1e12, 3)},
        "kernel_tflops": {n: round(contractions[n] * 2.0 * w.D * pairs / (k_launch[n] * 1e-3) / 1e12, 2) for n in contractions},
        "roofline": {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 3), "peak": BF16_MFMA_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 5),
                     "traffic": measured_traffic(workload, mode_name, selection, dom),
                     "flops_per_launch": dom_flops, "avg_launch_ms": round(k_launch[dom], 4)},
    })
    # HBM-bound steps: algorithmic bytes (every tensor once) over the measured kernel time
    esz = 2 if w.dtype == "bf16" else 4
    pooled = 4 * lay.num_qblocks * (w.Hq + w.Hkv) * w.D
    hbm = {"pool": w.T * (w.Hq + w.Hkv) * w.D * esz + pooled,
           "score": pooled + 4 * lay.scores_elems,
           "topk": 4 * lay.scores_elems + 4 * lay.sel_nnz + 4 * (lay.sel_rows + 1)}
    res["hbm"] = {n: {"bytes": int(b), "ms": round(k_step[n], 4), "gbps": round(b / (k_step[n] * 1e-3) / 1e9, 1) if k_step[n] > 0 else None,
                      "frac_of_8TBps": round(b / (k_step[n] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) if k_step[n] > 0 else None}
                  for n, b in hbm.items()}

    if selection == "topk":
        # outside the timed region: the same scoring + selection as one kernel that keeps the scores on chip
        # (sb_score_select without a score buffer); the step above uses the two-kernel form, whose HBM rates are asked for
        rp2, ix2 = torch.empty_like(rowptr), torch.empty_like(idx)
        sb.sb_set_instrumentation(sb.SB_INSTR_KERNEL_EVENTS)
        sb.sb_read_kernel_times()
        for _ in range(5):
            if L.sb_score_select(pb.ref(), P(q), P(k), None, None, P(rp2), P(ix2), P(ws_scores), st) != 0:
                raise RuntimeError(L.sb_last_error().decode())
        torch.cuda.synchronize()
        kt = sb.sb_read_kernel_times()
        sb.sb_set_instrumentation(0)
        nnz = int(lay.sel_nnz)
        # likewise outside the step: the coverage curves of the budget controller (Eq. 4) from the scores of the last step
        ws_cov = raw(lay.coverage_ws_bytes)
        sb.sb_score_coverage(pb, scores, ws=ws_cov)
        torch.cuda.synchronize()
        sb.sb_set_instrumentation(sb.SB_INSTR_KERNEL_EVENTS)
        for _ in range(3):
            sb.sb_score_coverage(pb, scores, ws=ws_cov)
        torch.cuda.synchronize()
        kc = sb.sb_read_kernel_times()
        sb.sb_set_instrumentation(0)
        del ws_cov
        res["score_coverage_ms"] = round(kc["coverage"][0] / 3, 4)
        res["fused_score_select"] = {"kernel_ms": round(kt["score_select"][0] / 5, 4),
                                     "two_kernel_ms": round(k_step["score"] + k_step["topk"], 4),
                                     "identical_selection": bool(torch.equal(rp2, rowptr) and torch.equal(ix2[:nnz], idx[:nnz]))}

    # cold caches (outside the timed region): five more steps, each after 1 GiB of unrelated writes has gone through the
    # L2 and the memory-side cache (256 MB); the figure above is the warm, steady-state one a training loop sees
    flush = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    cold = []
    for _ in range(5):
        flush.zero_()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); step(); b.record()
        torch.cuda.synchronize()
        cold.append(a.elapsed_time(b))
    del flush
    res["cold_cache"] = {"ms_per_step_median": round(sorted(cold)[2], 4), "ms_per_step_min": round(min(cold), 4),
                         "flush": "1 GiB written before every step"}

    if cu_busy:  # outside the timed region: one instrumented forward and one instrumented backward
        ncu = torch.cuda.get_device_properties(0).multi_processor_count
        spreads = {}
        for name, call, wsb in (("fwd", fwd, ws_fwd), ("bwd", bwd, ws_bwd)):
            sb.sb_set_instrumentation(sb.SB_INSTR_CU_BUSY)
            call()
            busy = np.sort(sb.sb_read_cu_busy(wsb).astype(np.float64))[::-1]
            sb.sb_set_instrumentation(0)
            busy = busy[:ncu]                       # the device's CUs, idle ones included
            spreads[name] = {"cus": int(ncu), "cus_with_work": int((busy > 0).sum()),
                             "spread_max_minus_min_over_mean": round(float((busy.max() - busy.min()) / busy.mean()), 4),
                             "max_over_mean": round(float(busy.max() / busy.mean()), 4)}
        res["cu_busy"] = spreads

    if cpu:
        from oracle import oracle as orc
        opb = orc.Problem(w.cu, w.Hq, w.Hkv, w.D, w.B, mode)
        host = tuple(t[n] if w.dtype == "bf16" else synth.round_to_bf16(t[n]) for n in ("q", "k", "v", "do"))
        rp_h = rowptr.cpu().numpy()
        res["cpu_baseline"] = cpu_baseline(w, host, opb, rp_h, idx.cpu().numpy()[: int(rp_h[-1])], 1.0 / np.sqrt(w.D))
    return res


run.cache = {}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", help="cfg1..cfg5 are BASELINE.json's configs[0..4]; blk256, d64")
    ap.add_argument("--mode", default="per_qhead", choices=["per_qhead", "per_kvgroup"])
    ap.add_argument("--selection", default="topk", choices=["topk", "sink"],
                    help="sink: a caller-supplied selection (block 0 + the most recent blocks) instead of the top-k of the scores")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cu-busy", action="store_true", help="skip the two instrumented launches that measure the per-CU busy-time spread")
    ap.add_argument("--no-also", action="store_true", help="skip the secondary runs (per-KV-group mode, the 32768-token batch)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    r = run(args.workload, args.mode, args.seed, args.steps, args.warmup, selection=args.selection,
            cu_busy=not args.no_cu_busy, cpu=not args.no_cpu_baseline)
    out = {
        "metric": "sparse-attn fwd+bwd effective TFLOP/s (selected blocks) + % bf16 MFMA peak",
        "value": r["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "config": r["config"],
        "ms_per_step_median": r["ms_per_step_median"], "ms_per_step_min": r["ms_per_step_min"],
        "pct_of_bf16_mfma_peak": r["pct_of_bf16_mfma_peak"], "attention_only": r["attention_only"],
        "kernel_ms": r["kernel_ms"], "kernel_tflops": r["kernel_tflops"], "roofline": r["roofline"], "hbm": r["hbm"],
        "cold_cache": r["cold_cache"],
    }
    for key in ("fused_score_select", "score_coverage_ms", "cu_busy", "cpu_baseline"):
        if key in r:
            out[key] = r[key]
    if not args.no_also and args.selection == "topk":
        also = []
        other = "per_kvgroup" if args.mode == "per_qhead" else "per_qhead"
        also.append(run(args.workload, other, args.seed, args.steps, args.warmup, brief=True))     # same values, other selection mode
        if args.workload != "cfg2":
            also.append(run("cfg2", args.mode, args.seed, args.steps, args.warmup, brief=True))    # configs[1]
        out["also"] = also
    print(json.dumps(out))


if __name__ == "__main__":
    main()
