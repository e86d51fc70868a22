#!/usr/bin/env python3
"""Benchmark: one step = slimattn_fwd + slimattn_bwd over every unit of one synthetic pack.

Prints ONE JSON line (see --help).  The workload is the Llama-3-8B-shaped 32K-token pack
(lognormal lengths, slices of 4096, 32 query / 8 KV heads, head_dim 128, bf16); the timed steps
cycle over the packs drawn from the four fixed seeds, all resident in HBM before timing starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
HBM_PEAK_GBS = 8000.0


def _pack(w, seed):
    import workloads as W
    rng = np.random.default_rng(seed)
    L = W.draw_lengths(w, rng)
    q, k, v, dO = W.draw_values(w, int(L.sum()), rng)
    return L, q, k, v, dO


def _cpu_baseline(w, packs, budget_s=12.0):
    """The fp64 oracle (forward + backward, unsliced definition) timed on host cores over a bounded
    sample: (sample, query head) items of the first pack, longest samples first, until the budget
    is used.  Throughput counts causal-effective flops, like the GPU figure."""
    from oracle import attention as A
    L, q, k, v, dO = packs[0]
    cu = np.concatenate([[0], np.cumsum(L)])
    g = w.n_q_heads // w.n_kv_heads
    scale = w.head_dim ** -0.5
    order = np.argsort(-L, kind="stable")
    flops, items, t0 = 0, 0, time.perf_counter()
    done = False
    for h in range(w.n_q_heads):
        for s in order:
            a, b = int(cu[s]), int(cu[s + 1])
            qq, kk, vv, dd = q[a:b, h:h + 1], k[a:b, h // g:h // g + 1], v[a:b, h // g:h // g + 1], dO[a:b, h:h + 1]
            o, lse = A.fwd_sample(qq, kk, vv, scale)
            A.bwd_sample(qq, kk, vv, o, lse, dd, scale)
            n = b - a
            flops += 14 * w.head_dim * (n * (n + 1) // 2)
            items += 1
            if time.perf_counter() - t0 > budget_s:
                done = True
                break
        if done:
            break
    dt = time.perf_counter() - t0
    cores = len(os.sched_getaffinity(0))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{items} (sample, query-head) items of the seed-{1} pack, longest samples first, fwd+bwd fp64, "
                      f"{dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg1_llama8b_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-unit", action="store_true", help="one launch per unit instead of one fused launch")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2509_26246_amd as S
    import workloads as W
    from paper_2509_26246_amd import harness as H

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    S.load_library()                      # fails loudly if the HIP library is missing
    w = W.WORKLOADS[args.workload]
    packs = [_pack(w, seed) for seed in W.SEEDS]
    probs, pairs = [], []
    for L, q, k, v, dO in packs:
        cu, sl = S.build_slices(L, w.slice_size)
        fu = S.build_units(cu, sl, w.fwd_policy[0], **w.fwd_policy[1])
        bu = S.build_units(cu, sl, w.bwd_policy[0], **w.bwd_policy[1])
        probs.append(H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=(w.dtype == "bf16")))
        pairs.append(int(sum(S.slice_pairs(r) for r in sl)))
    flags = S.FLAG_PER_UNIT_LAUNCH if args.per_unit else 0
    d, hq = w.head_dim, w.n_q_heads

    def step(i):
        p = probs[i % len(probs)]
        p.forward(flags=flags)
        p.backward(flags=flags)

    # A plain device copy of known size (256 MiB read + 256 MiB written) before anything else: under
    # `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` it calibrates the counters' units for roofline.traffic.
    cal = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
    cal2 = torch.empty_like(cal)
    cal2.copy_(cal)
    del cal, cal2
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    S.profile_enable(64 * max(args.steps, 1) if args.per_unit else 8 * max(args.steps, 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = S.profile_read()
    S.profile_enable(0)

    step_pairs = [pairs[i % len(probs)] for i in range(args.steps)]
    tot_pairs = sum(step_pairs)
    fwd_flops = S.flops_fwd(tot_pairs, d, hq)
    bwd_flops = S.flops_bwd(tot_pairs, d, hq)
    wall = t1 - t0
    fwd_ms = prof["fwd"][0]
    bwd_ms = sum(prof[c][0] for c in ("delta", "dq", "dkdv", "finalize", "fill"))
    value = (fwd_flops + bwd_flops) / wall / 1e12
    fwd_tf = fwd_flops / (fwd_ms * 1e-3) / 1e12 if fwd_ms > 0 else 0.0
    bwd_tf = bwd_flops / (bwd_ms * 1e-3) / 1e12 if bwd_ms > 0 else 0.0

    # Roofline of the dominant kernel (largest share of kernel time).  The five counted tile products
    # of the backward pass (scores, dP, dV, dK, dQ; 2*d*Hq flops per pair each) are split between its
    # two kernels so that they add up to the counted total: dK/dV kernel 3 (dK, dV and half of the two
    # recomputed products), dQ kernel 2; the forward kernel has 2.
    share = {"fwd": 2, "dq": 2, "dkdv": 3}
    dom = max(share, key=lambda c: prof[c][0])
    dom_ms, dom_n = prof[dom]
    dom_flops = share[dom] * 2 * d * hq * tot_pairs
    achieved = dom_flops / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{dom}_{args.workload}.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / BF16_MFMA_PEAK_TFLOPS, "traffic": traffic,
                "avg_launch_ms": dom_ms / max(dom_n, 1), "launches": dom_n,
                "algorithmic_flops_per_launch": dom_flops / max(dom_n, 1)}

    out = {
        "metric": "causal-effective attention TFLOP/s fwd & bwd (sliced varlen) + % bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / max(args.steps, 1), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "total_tokens": w.total_tokens, "n_q_heads": hq,
                   "n_kv_heads": w.n_kv_heads, "head_dim": d, "slice_size": w.slice_size, "seeds": list(W.SEEDS),
                   "launch": "per-unit" if args.per_unit else "fused", "fwd_policy": w.fwd_policy[0],
                   "bwd_policy": w.bwd_policy[0]},
        "fwd_tflops": fwd_tf, "bwd_tflops": bwd_tf,
        "fwd_pct_bf16_peak": 100 * fwd_tf / BF16_MFMA_PEAK_TFLOPS, "bwd_pct_bf16_peak": 100 * bwd_tf / BF16_MFMA_PEAK_TFLOPS,
        "kernel_ms_per_step": {c: prof[c][0] / max(args.steps, 1) for c in prof},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(w, packs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
