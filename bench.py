#!/usr/bin/env python3
"""Benchmark: one step = slimattn_fwd + slimattn_bwd over every unit of one synthetic pack.

Prints ONE JSON line.  The default workload is the Llama-3-8B-shaped 32K-token pack (lognormal lengths,
slices of 4096, 32 query / 8 KV heads, head_dim 128, bf16); the timed steps cycle over the packs drawn from
the four fixed seeds, all resident in HBM before timing starts.

`value` is the fused launch (one launch per kernel over the whole unit list: the result does not depend on
the grouping, so the unit lists then only decide validation).  The same line also carries `per_unit`: the
same packs run one launch per unit in list order, which is how a pipeline runtime that receives one
MicroPack at a time calls the library and the mode in which the forward and backward unit lists matter,
with the spread of per-unit times.  `--per-unit` makes that mode the main measurement (and `value`).
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
HBM_PEAK_GBS = 8000.0
# The five counted tile products of the backward pass (scores, dP, dV, dK, dQ; 2*d*Hq flops per pair each)
# are split between its two kernels so that they add up to the counted total: dK/dV kernel 3 (dK, dV and
# half of the two recomputed products), dQ kernel 2; the forward kernel has 2.  What the kernels execute:
# forward 2, dQ 3, dK/dV 4 products per tile, on whole tiles.
CREDITED = {"fwd": 2, "dq": 2, "dkdv": 3}
EXECUTED = {"fwd": 2, "dq": 3, "dkdv": 4}


def _pack(w, seed):
    import workloads as W
    rng = np.random.default_rng(seed)
    L = W.draw_lengths(w, rng)
    q, k, v, dO = W.draw_values(w, int(L.sum()), rng)
    return L, q, k, v, dO


def _cpu_baseline(w, packs, seed, budget_s=12.0):
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
            if b - a > 16384:                     # one such item alone would outlast the budget many times
                continue
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
            "sample": f"{items} (sample, query-head) items of the seed-{seed} pack (samples up to 16384 rows), longest "
                      f"first, fwd+bwd fp64, {dt:.1f} s"}


def _runs_of_scope(sl, ids):
    """Slices of one launch scope -> runs of query rows (adjacent slices of a sample merged): (q_lo, q_hi, kv_start)."""
    rec = sorted((int(sl[t][2]), int(sl[t][2] + sl[t][3]), int(sl[t][4]), int(sl[t][0])) for t in ids)
    runs = []
    for a, b, ks, smp in rec:
        if runs and runs[-1][3] == smp and runs[-1][1] == a:
            runs[-1][1] = b
        else:
            runs.append([a, b, ks, smp])
    return runs


def _executed_pairs(runs, q_tile=128, k_tile_fwd=64, kv_tile=256, q_step=32):
    """(query, key) pairs per query head the kernels run products on, whole tiles included: the forward's blocks
    (128 rows, every wave walks all 64-key tiles of the block), the dQ kernel's waves (32 rows, tiles up to the
    wave's diagonal), the dK/dV kernel's blocks (256 keys against steps of 32 query rows at or after them)."""
    fwd = dq = dkdv = 0
    by_sample = {}
    for a, b, ks, smp in runs:
        by_sample.setdefault(smp, []).append((a, b, ks))
        for r0 in range(a, b, q_tile):
            q_end = min(b, r0 + q_tile)
            n_tiles = (q_end - ks + k_tile_fwd - 1) // k_tile_fwd
            fwd += n_tiles * q_tile * k_tile_fwd
            for wv in range(4):
                q0w = r0 + 32 * wv
                dq += min(n_tiles, (q0w + 31 - ks) // k_tile_fwd + 1) * 32 * k_tile_fwd
    for rs in by_sample.values():
        ks, kv_end = rs[0][2], rs[-1][1]
        for k0 in range(ks, kv_end, kv_tile):
            steps = sum((b - max(a, k0) + q_step - 1) // q_step for a, b, _ in rs if b > k0)
            dkdv += steps * q_step * kv_tile
    return {"fwd": fwd, "dq": dq, "dkdv": dkdv}


def _algorithmic_bytes(T, hq, hkv, d, e=2):
    """HBM bytes one fused launch of each kernel has to move at least (every tensor once)."""
    return {"fwd": e * (2 * T * hq * d + 2 * T * hkv * d) + 4 * T * hq,
            "dq": e * (4 * T * hq * d + 2 * T * hkv * d) + 20 * T * hq,
            "dkdv": e * (2 * T * hq * d + 4 * T * hkv * d) + 16 * T * hq}


def _spread(xs):
    xs = [float(x) for x in xs]
    if not xs:
        return None
    mean = sum(xs) / len(xs)
    sd = (sum((x - mean) ** 2 for x in xs) / len(xs)) ** 0.5
    return {"n_units": len(xs), "min_ms": min(xs), "median_ms": statistics.median(xs), "max_ms": max(xs), "mean_ms": mean,
            "cv": sd / mean if mean > 0 else 0.0}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg1_llama8b_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-unit", action="store_true", help="main measurement: one launch per unit instead of one fused launch")
    ap.add_argument("--seeds", default="", help="comma-separated subset of the workload's seeds (default: all four)")
    ap.add_argument("--brief", action="store_true", help="the main measurement only: no per-seed values, no secondary per-unit records, no graph replay, no search")
    ap.add_argument("--granule", type=int, default=0,
                    help="solver partition: cuts on multiples of this many rows (default: the rows whose forward work "
                         "items fill the chip once, 256 blocks x 128 rows / head pairs, at least 256)")
    ap.add_argument("--partition", choices=["policy", "solver"], default="policy",
                    help="slice table and unit lists of the main measurement: the workload's greedy policies on fixed-size "
                         "slices, or the exact min-max partition solver (same unit counts, cuts on 256-row granules)")
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
    seeds = [int(x) for x in args.seeds.split(",")] if args.seeds else list(W.SEEDS)
    packs = [_pack(w, seed) for seed in seeds]
    d, hq, hkv = w.head_dim, w.n_q_heads, w.n_kv_heads
    def policy_tables(L):
        cu, sl = S.build_slices(L, w.slice_size)
        return cu, sl, S.build_units(cu, sl, w.fwd_policy[0], **w.fwd_policy[1]), S.build_units(cu, sl, w.bwd_policy[0], **w.bwd_policy[1])

    def solver_tables(L):
        """The exact partition for the same numbers of units the policies produce and the same cost weights; slices no
        longer than the workload's slice size."""
        _, _, fu, bu = policy_tables(L)
        wq_f, wl_f = w.fwd_policy[1].get("w_quad", 2), w.fwd_policy[1].get("w_lin", 0)
        wq_b, wl_b = w.bwd_policy[1].get("w_quad", 5), w.bwd_policy[1].get("w_lin", 0)
        # Cuts on multiples of the rows that fill the chip once with forward work items (a query tile of 128 rows and a
        # pair of heads per block, 256 blocks): a unit a little over such a multiple would leave a second round of
        # blocks almost empty, and on long samples one round takes milliseconds.
        granule = args.granule or max(256, 256 * 128 // max(1, w.n_q_heads // 2))
        r = S.solve_partition(L, m_fwd=len(fu[0]) - 1, m_bwd=len(bu[0]) - 1, w_quad_fwd=wq_f, w_lin_fwd=wl_f, w_quad_bwd=wq_b,
                              w_lin_bwd=wl_b, granule=granule, max_slice=max(w.slice_size, granule))
        return r["cu"], r["slices"], r["fwd"], r["bwd"]

    def make_problems(table_fn):
        probs, pairs, tabs, build_ms = [], [], [], {"slices_and_units": [], "derive_and_upload": [], "derive_and_queue_upload": []}
        for L, q, k, v, dO in packs:
            t0 = time.perf_counter()
            cu, sl, fu, bu = table_fn(L)
            t1 = time.perf_counter()
            torch.cuda.set_device(0)
            tmp = S.tables_create(cu, sl, fu[0], fu[1], bu[0], bu[1])      # timed on its own: derived work-lists + one upload
            t2 = time.perf_counter()
            tmp.destroy()
            t3 = time.perf_counter()
            tmp = S.tables_create(cu, sl, fu[0], fu[1], bu[0], bu[1], stream=torch.cuda.current_stream().cuda_stream)
            t4 = time.perf_counter()                                       # host time when the upload is queued on the stream
            torch.cuda.synchronize()
            tmp.destroy()
            build_ms["slices_and_units"].append((t1 - t0) * 1e3)
            build_ms["derive_and_upload"].append((t2 - t1) * 1e3)
            build_ms["derive_and_queue_upload"].append((t4 - t3) * 1e3)
            probs.append(H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=(w.dtype == "bf16")))
            pairs.append(int(sum(S.slice_pairs(r) for r in sl)))
            tabs.append((cu, sl, fu, bu))
        return probs, pairs, tabs, build_ms

    probs, pairs, tabs, build_ms = make_problems(solver_tables if args.partition == "solver" else policy_tables)
    n_packs = len(probs)

    # A plain device copy of known size (256 MiB read + 256 MiB written) before anything else: under
    # `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` it calibrates the counters' units for roofline.traffic.
    cal = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
    cal2 = torch.empty_like(cal)
    cal2.copy_(cal)
    del cal, cal2

    def launches_per_step(p):
        return p.tables.n_fwd_units + 5 * p.tables.n_bwd_units + 10

    def measure(flags, steps, warmup, which=None):
        """Runs warmup + steps over the packs `which` (default: all, cycling); returns wall seconds, pairs done and
        the per-launch records (class, pass, unit, ms)."""
        idx = list(range(n_packs)) if which is None else list(which)
        # The warm-up runs timed like the steps and nothing but a synchronisation separates the two; its records are
        # cut off afterwards.  The interpreter's cyclic garbage collector stays off meanwhile: a full collection
        # (tens of milliseconds with torch loaded) inside the first calls of the timed loop, when the GPU has
        # little queued, left the GPU idle for as long.
        gc.collect()
        gc.disable()
        n_warm = sum(launches_per_step(probs[idx[i % len(idx)]]) for i in range(warmup))
        S.profile_enable(n_warm + sum(launches_per_step(probs[idx[i % len(idx)]]) for i in range(steps)) + 16)
        for i in range(warmup):
            p = probs[idx[i % len(idx)]]
            p.forward(flags=flags); p.backward(flags=flags)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            p = probs[idx[i % len(idx)]]
            p.forward(flags=flags); p.backward(flags=flags)
        measure.host_enqueue_s = time.perf_counter() - t0    # all launches queued; the GPU is still working
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        gc.enable()
        cls, ps, un, ms = S.profile_read_launches()
        S.profile_enable(0)
        # the warm-up's records: everything before the record of the (warmup + 1)-th forward call (a call's own
        # record precedes those of its kernels)
        first = int(np.flatnonzero(cls == S.KERNEL_CLASSES.index("fwd_call"))[warmup]) if warmup > 0 else 0
        return t1 - t0, sum(pairs[idx[i % len(idx)]] for i in range(steps)), (cls[first:], ps[first:], un[first:], ms[first:])

    def measure_graph(flags, steps, warmup):
        """The same step replayed from a HIP graph per pack (forward + backward recorded once by stream capture):
        what is left of the gaps between a step's launches when the host does not issue them one by one.  No
        per-kernel events (they are not part of a capture): wall time only."""
        graphs = [p.capture_step(flags) for p in probs]
        gc.collect()
        gc.disable()
        for i in range(warmup):
            graphs[i % n_packs].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i % n_packs].replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        gc.enable()
        tot = sum(pairs[i % n_packs] for i in range(steps))
        del graphs
        return {"value": (S.flops_fwd(tot, d, hq) + S.flops_bwd(tot, d, hq)) / (t1 - t0) / 1e12, "ms_per_step": (t1 - t0) * 1e3 / max(steps, 1)}

    def summarise(wall, tot_pairs, rec, steps):
        cls, ps, un, ms = rec
        per = {c: (float(ms[cls == i].sum()), int((cls == i).sum())) for i, c in enumerate(S.KERNEL_CLASSES)}
        fwd_flops, bwd_flops = S.flops_fwd(tot_pairs, d, hq), S.flops_bwd(tot_pairs, d, hq)
        # whole calls, first launch to last on the caller's stream (gaps between a call's launches included)
        fwd_ms, bwd_ms = per["fwd_call"][0], per["bwd_call"][0]
        out = {"value": (fwd_flops + bwd_flops) / wall / 1e12, "ms_per_step": wall * 1e3 / max(steps, 1),
               "fwd_tflops": fwd_flops / (fwd_ms * 1e-3) / 1e12 if fwd_ms > 0 else 0.0,
               "bwd_tflops": bwd_flops / (bwd_ms * 1e-3) / 1e12 if bwd_ms > 0 else 0.0,
               "kernel_ms_per_step": {c: per[c][0] / max(steps, 1) for c in per if not c.endswith("_call") and c != "unused"},
               "call_ms_per_step": {"fwd": fwd_ms / max(steps, 1), "bwd": bwd_ms / max(steps, 1)}}
        out["fwd_pct_bf16_peak"] = 100 * out["fwd_tflops"] / BF16_MFMA_PEAK_TFLOPS
        out["bwd_pct_bf16_peak"] = 100 * out["bwd_tflops"] / BF16_MFMA_PEAK_TFLOPS
        return out, per

    def unit_times(rec):
        """{(pass, pack, unit): mean ms over the steps in which that pack ran} from per-launch records."""
        cls, ps, un, ms = rec
        step, prev_pass, acc = 0, 0, {}
        for p_, u, m in zip(ps, un, ms):                # launches come in step order: forward, then backward
            if p_ == 0 and prev_pass == 1:
                step += 1
            prev_pass = p_
            if u >= 0:
                key = (int(p_), step % n_packs, int(u))
                tot, cnt = acc.get(key, (0.0, set()))
                cnt.add(step)
                acc[key] = (tot + float(m), cnt)
        return {k_: tot / len(cnt) for k_, (tot, cnt) in acc.items()}

    def pipeline_sim(rec):
        """The measured per-unit times through the DAG simulator: makespan and idle share of a 1F1B pipeline whose
        every stage holds one such attention layer, per number of stages (mean over the packs)."""
        ut = unit_times(rec)
        out = {}
        # what one attention layer keeps per token between its tasks: K and V (bf16) as the cache, the fp32 rows
        # dK and dV are accumulated in until their release, and q, o (bf16) and lse from forward to backward
        kv_b, grad_b, act_b = 2 * hkv * d * 2, 2 * hkv * d * 4, 2 * hq * d * 2 + hq * 4
        for stages in (1, 2, 4, 8):
            tot, busy = 0.0, 0.0
            mem = {"kv_state_per_slice": 0.0, "kv_state_per_sample": 0.0, "with_activations_per_slice": 0.0, "with_activations_per_sample": 0.0}
            for i, (cu, sl, fu, bu) in enumerate(tabs):
                fc = [int(round(ut[(0, i, u)] * 1e6)) for u in range(len(fu[0]) - 1)]      # ns
                bc = [int(round(ut[(1, i, u)] * 1e6)) for u in range(len(bu[0]) - 1)]
                g = S.dag_build_1f1b(sl, fu, bu, stages, fc, bc)
                start, finish, t_total = S.dag_timeline(g["weight"], g["edge_from"], g["edge_to"])
                tot += t_total * 1e-6
                busy += (sum(fc) + sum(bc)) * 1e-6
                for key, act, per_slice in (("kv_state_per_slice", 0, True), ("kv_state_per_sample", 0, False),
                                            ("with_activations_per_slice", act_b, True), ("with_activations_per_sample", act_b, False)):
                    peak, _ = S.dag_memory(start, finish, S.dag_buffers_1f1b(sl, fu, bu, stages, act, kv_b, grad_b, per_slice), stages)
                    mem[key] += float(peak.max()) / 2 ** 20
            out[str(stages)] = {"makespan_ms": tot / n_packs, "idle_share": 1.0 - busy / tot if tot > 0 else 0.0,
                                "peak_mib_worst_stage": {k_: round(v_ / n_packs, 1) for k_, v_ in mem.items()}}
        return out

    def unit_count_search(rec, stages=4, m_max=64):
        """The paper's outer loop on this GPU's own timings: task time = fixed + cost x rate per pass, fitted by least
        squares to the measured per-unit times of `rec` (cost = the workload's weights on pairs and rows); then, per
        pack, every candidate unit count (multiples of the pipeline width on the logarithmic grid) is partitioned by the
        exact solver, priced, and run through the 1F1B simulator with its memory footprint.  Mean over the packs."""
        ut = unit_times(rec)
        wts = {0: (w.fwd_policy[1].get("w_quad", 2), w.fwd_policy[1].get("w_lin", 0)),
               1: (w.bwd_policy[1].get("w_quad", 5), w.bwd_policy[1].get("w_lin", 0))}
        rates = {}
        for pss in (0, 1):
            xs, ys = [], []
            for i, (cu, sl, fu, bu) in enumerate(tabs):
                ptr, flat = (fu, bu)[pss]
                for u in range(len(ptr) - 1):
                    cost = sum(wts[pss][0] * S.slice_pairs(sl[t]) + wts[pss][1] * int(sl[t][3]) for t in flat[ptr[u]:ptr[u + 1]])
                    xs.append(float(cost)); ys.append(ut[(pss, i, u)] * 1e6)             # ns
            slope, icpt = np.polyfit(np.array(xs), np.array(ys), 1) if len(xs) > 1 else (ys[0] / max(xs[0], 1.0), 0.0)
            rates[pss] = (max(0, int(round(icpt))), max(1, int(round(slope * 2 ** 30))), 2 ** 30)
        cands = S.candidate_unit_counts(stages, m_max)
        granule = args.granule or max(256, 256 * 128 // max(1, w.n_q_heads // 2))
        solver = dict(w_quad_fwd=wts[0][0], w_lin_fwd=wts[0][1], w_quad_bwd=wts[1][0], w_lin_bwd=wts[1][1], granule=granule,
                      max_slice=max(w.slice_size, granule))
        kv_b, grad_b, act_b = 2 * hkv * d * 2, 2 * hkv * d * 4, 2 * hq * d * 2 + hq * 4
        t_sum, pk_sum, chosen = np.zeros(len(cands)), np.zeros(len(cands)), []
        t0 = time.perf_counter()
        for L, *_ in packs:
            t, pk, best = S.search_unit_count(L, cands, solver, stages, rates[0], rates[1], act_b, kv_b, grad_b, n_threads=8)
            t_sum += t * 1e-6
            pk_sum += pk / 2 ** 20
            chosen.append(int(cands[best]) if best >= 0 else -1)
        search_ms = (time.perf_counter() - t0) * 1e3 / n_packs
        return {"stages": stages, "fit_ns": {"fwd_fixed_ns": rates[0][0], "fwd_ns_per_1e9_cost": rates[0][1] / 2 ** 30 * 1e9,
                                             "bwd_fixed_ns": rates[1][0], "bwd_ns_per_1e9_cost": rates[1][1] / 2 ** 30 * 1e9},
                "candidates": [int(m) for m in cands], "predicted_ms": [round(x / n_packs, 3) for x in t_sum],
                "peak_mib_worst_stage": [round(x / n_packs, 1) for x in pk_sum], "chosen_per_pack": chosen,
                "search_ms_per_pack": round(search_ms, 3)}

    def unit_spread(rec, steps):
        """Time of each scheduling unit (all kernels launched for it, averaged over the steps in which its pack ran):
        spread over the units of all packs together, and the coefficient of variation inside each pack (the packs
        differ in total work, so only that says how even one pack's units are)."""
        ut = unit_times(rec)
        out = {}
        for name, pss in (("fwd", 0), ("bwd", 1)):
            xs = [v_ for (p_, _, _), v_ in ut.items() if p_ == pss]
            if not xs:
                continue
            out[name] = _spread(xs)
            per_pack = [_spread([v_ for (p_, i_, _), v_ in ut.items() if p_ == pss and i_ == i]) for i in range(n_packs)]
            out[name]["cv_within_pack"] = [round(x["cv"], 4) for x in per_pack if x]
            out[name]["max_over_mean_within_pack"] = [round(x["max_ms"] * x["n_units"] / sum_ms, 4) for x, sum_ms in
                                                      ((x, x["n_units"] * x["mean_ms"]) for x in per_pack if x)]
        return out

    main_flags = S.FLAG_PER_UNIT_LAUNCH if args.per_unit else 0
    wall, tot_pairs, rec = measure(main_flags, args.steps, args.warmup)
    main_sum, per = summarise(wall, tot_pairs, rec, args.steps)
    host_enqueue_ms = measure.host_enqueue_s * 1e3 / max(args.steps, 1)

    # Per kernel: algorithmic and executed throughput, algorithmic HBM rate.  Executed pairs and bytes are those
    # of the scopes the main measurement launched.
    T_mean = sum(int(p.tables.total_tokens) for p in probs) / n_packs
    alg_bytes = _algorithmic_bytes(T_mean, hq, hkv, d)
    exec_pairs = {"fwd": 0, "dq": 0, "dkdv": 0}
    for i in range(args.steps):
        cu, sl, fu, bu = tabs[i % n_packs]
        if args.per_unit:
            for c, (up, us) in (("fwd", fu), ("bwd", bu)):
                for u in range(len(up) - 1):
                    e = _executed_pairs(_runs_of_scope(sl, us[up[u]:up[u + 1]]))
                    if c == "fwd":
                        exec_pairs["fwd"] += e["fwd"]
                    else:
                        exec_pairs["dq"] += e["dq"]; exec_pairs["dkdv"] += e["dkdv"]
        else:
            e = _executed_pairs(_runs_of_scope(sl, range(len(sl))))
            for c in exec_pairs:
                exec_pairs[c] += e[c]
    kernels = {}
    for c in ("fwd", "dq", "dkdv"):
        ms_c, n_c = per[c]
        if ms_c <= 0:
            continue
        sec = ms_c * 1e-3
        kernels[c] = {"avg_launch_ms": ms_c / max(n_c, 1), "launches": n_c,
                      "algorithmic_tflops": CREDITED[c] * 2 * d * hq * tot_pairs / sec / 1e12,
                      "executed_mfma_tflops": EXECUTED[c] * 2 * d * hq * exec_pairs[c] / sec / 1e12,
                      "tile_padding": exec_pairs[c] / max(tot_pairs, 1)}
        kernels[c]["frac_of_bf16_peak"] = kernels[c]["algorithmic_tflops"] / BF16_MFMA_PEAK_TFLOPS
        if not args.per_unit:
            kernels[c]["hbm_gbs_algorithmic"] = alg_bytes[c] * args.steps / sec / 1e9
            kernels[c]["hbm_frac_of_peak_algorithmic"] = kernels[c]["hbm_gbs_algorithmic"] / HBM_PEAK_GBS

    # Roofline of the dominant kernel (largest share of kernel time).  `traffic` (HBM bytes per launch from
    # rocprofv3 counters) is not measured by this run: it is read from the committed summary of a profiling
    # run of this command, and only when that summary names this workload and launch mode.
    dom = max(CREDITED, key=lambda c: per[c][0])
    dom_ms, dom_n = per[dom]
    dom_flops = CREDITED[dom] * 2 * d * hq * tot_pairs
    achieved = dom_flops / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    mode = "per-unit" if args.per_unit else "fused"
    traffic, traffic_src = None, None
    for c in ("fwd", "dq", "dkdv"):
        tpath = os.path.join(ROOT, "profiles", f"traffic_{c}_{args.workload}_{mode}.json")
        if os.path.exists(tpath) and c in kernels:
            tj = json.load(open(tpath))
            kernels[c]["hbm_bytes_per_launch_measured"] = tj.get("hbm_bytes_per_launch")
            kernels[c]["hbm_gbs_measured"] = tj["hbm_bytes_per_launch"] / (kernels[c]["avg_launch_ms"] * 1e-3) / 1e9
            kernels[c]["hbm_traffic_source"] = tj.get("source")
            if c == dom:
                traffic, traffic_src = tj.get("hbm_bytes_per_launch"), tj.get("source")
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / BF16_MFMA_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                "avg_launch_ms": dom_ms / max(dom_n, 1), "launches": dom_n,
                "algorithmic_flops_per_launch": dom_flops / max(dom_n, 1)}

    out = {
        "metric": "causal-effective attention TFLOP/s fwd & bwd (sliced varlen) + % bf16 MFMA peak",
        "value": main_sum["value"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_sum["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "total_tokens": w.total_tokens if w.total_tokens > 0 else int(T_mean),
                   "n_q_heads": hq, "n_kv_heads": hkv, "head_dim": d, "slice_size": w.slice_size, "seeds": seeds,
                   "launch": mode, "partition": args.partition, "fwd_policy": w.fwd_policy[0], "bwd_policy": w.bwd_policy[0],
                   "fwd_units": [p.tables.n_fwd_units for p in probs], "bwd_units": [p.tables.n_bwd_units for p in probs]},
        "fwd_tflops": main_sum["fwd_tflops"], "bwd_tflops": main_sum["bwd_tflops"],
        "fwd_pct_bf16_peak": main_sum["fwd_pct_bf16_peak"], "bwd_pct_bf16_peak": main_sum["bwd_pct_bf16_peak"],
        "kernel_ms_per_step": main_sum["kernel_ms_per_step"], "call_ms_per_step": main_sum["call_ms_per_step"],
        "host_enqueue_ms_per_step": host_enqueue_ms, "kernels": kernels,
        "table_build_ms": {k_: statistics.median(v_) for k_, v_ in build_ms.items()},
        "roofline": roofline,
    }
    if args.per_unit:
        out["unit_ms"] = unit_spread(rec, args.steps)
        out["pipeline_1f1b"] = pipeline_sim(rec)
        if not args.brief:
            out["hip_graph_replay"] = measure_graph(main_flags, args.steps, min(args.warmup, 4))
            out["unit_count_search"] = unit_count_search(rec)

    if not args.brief:
        # every seed's pack on its own (same launch mode as the main measurement), and the median over seeds
        per_seed = {}
        for i, seed in enumerate(seeds):
            wl, pr, rc = measure(main_flags, 12, 4, which=[i])
            s_, _ = summarise(wl, pr, rc, 12)
            per_seed[str(seed)] = {"value": s_["value"], "fwd_tflops": s_["fwd_tflops"], "bwd_tflops": s_["bwd_tflops"],
                                   "pairs": pairs[i], "samples": int(len(packs[i][0])), "longest": int(packs[i][0].max())}
        out["per_seed"] = per_seed
        out["value_median_over_seeds"] = statistics.median(v_["value"] for v_ in per_seed.values())
        if not args.per_unit:
            # the same packs, one launch per unit in list order
            wl, pr, rc = measure(S.FLAG_PER_UNIT_LAUNCH, args.steps, min(args.warmup, 4))
            s_, _ = summarise(wl, pr, rc, args.steps)
            s_["unit_ms"] = unit_spread(rc, args.steps)
            s_["pipeline_1f1b"] = pipeline_sim(rc)
            s_["hip_graph_replay"] = measure_graph(S.FLAG_PER_UNIT_LAUNCH, args.steps, min(args.warmup, 4))
            s_["unit_count_search"] = unit_count_search(rc)
            out["per_unit"] = s_
            if args.partition == "policy":
                # the same packs partitioned by the exact solver instead of the greedy policies (same unit counts):
                # what it does to the spread of per-unit times
                for p_ in probs:
                    p_.tables.destroy()
                keep = (probs, pairs, tabs)
                del probs[:]
                probs2, pairs2, tabs2, bms2 = make_problems(solver_tables)
                probs.extend(probs2); pairs[:] = pairs2; tabs[:] = tabs2
                wl, pr, rc = measure(S.FLAG_PER_UNIT_LAUNCH, args.steps, min(args.warmup, 4))
                s2, _ = summarise(wl, pr, rc, args.steps)
                s2["unit_ms"] = unit_spread(rc, args.steps)
                s2["pipeline_1f1b"] = pipeline_sim(rc)
                s2["hip_graph_replay"] = measure_graph(S.FLAG_PER_UNIT_LAUNCH, args.steps, min(args.warmup, 4))
                s2["fwd_units"] = [p_.tables.n_fwd_units for p_ in probs]
                s2["bwd_units"] = [p_.tables.n_bwd_units for p_ in probs]
                s2["slices"] = [len(t_[1]) for t_ in tabs]
                s2["solve_ms"] = statistics.median(bms2["slices_and_units"])
                out["per_unit_solver"] = s2
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(w, packs, seeds[0])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
