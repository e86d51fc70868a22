"""DAG oracle: the execution timeline of a task graph and the 1F1B task graph over asymmetric unit lists.

Paper, DAG-based Pipeline Simulator.  A vertex is a task (stage, action, data unit) with a weight w(v), its
time.  Edges are the data dependencies (inter-stage: a unit goes down the stages forward and back up backward;
inter-slice: a slice's forward needs the KV cache of the sample's earlier slices, its backward the KV
gradients of the later ones) and the schedule dependencies (the order of the tasks of one stage).  DAG
resolution, in the paper's notation:
    Start(v) = max({0} U {Finish(u) : (u, v) in E}),   Finish(v) = Start(v) + w(v),   T_total = max_v Finish(v),
computed in a topological order of G, each finished vertex relaxing the start of its successors.

`timeline` is that procedure.  `build_1f1b` writes the graph down for forward and backward unit lists that
group the slices differently (the paper's figure has one data id per chain; with two lists a backward unit at
the last stage follows every forward unit it shares a slice with).  Per stage: p - 1 - s forwards to fill the
pipeline, then one forward and -- if all forward units holding slices of its samples have been issued -- one
backward in turn (otherwise the stage goes on with the next forward: the extra forward unit of the PackFlow
section), then the remaining backwards.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

FWD, BWD = 0, 1
EDGE_STAGE, EDGE_SLICE, EDGE_SCHEDULE = 0, 1, 2


def topological_sort(n: int, edges: Sequence[Tuple[int, int]]) -> List[int]:
    indeg = [0] * n
    succ: List[List[int]] = [[] for _ in range(n)]
    for u, v in edges:
        succ[u].append(v)
        indeg[v] += 1
    order = [v for v in range(n) if indeg[v] == 0]
    for u in order:                      # the list grows while it is walked
        for v in succ[u]:
            indeg[v] -= 1
            if indeg[v] == 0:
                order.append(v)
    if len(order) != n:
        raise ValueError("the graph has a cycle")
    return order


def timeline(weights: Sequence[int], edges: Sequence[Tuple[int, int]]):
    """(Start, Finish, T_total) of the paper's execution-timeline procedure."""
    n = len(weights)
    start = [0] * n
    finish = [0] * n
    succ: List[List[int]] = [[] for _ in range(n)]
    for u, v in edges:
        succ[u].append(v)
    for u in topological_sort(n, edges):
        finish[u] = start[u] + weights[u]
        for v in succ[u]:
            start[v] = max(start[v], finish[u])
    return start, finish, (max(finish) if n else 0)


def build_1f1b(slices, fwd_units, bwd_units, n_stages: int, fwd_cost: Sequence[int], bwd_cost: Sequence[int]):
    """Vertices [(stage, action, unit)], weights, edges [(u, v, kind)] of the 1F1B pipeline.  Vertex ids: forward
    task (s, u) = s * n_fwd + u; backward task (s, v) = n_stages * n_fwd + s * n_bwd + v."""
    (fp, fs), (bp, bs) = fwd_units, bwd_units
    nf, nb = len(fp) - 1, len(bp) - 1
    fwd_of = {int(t): u for u in range(nf) for t in fs[fp[u]:fp[u + 1]]}
    bwd_of = {int(t): v for v in range(nb) for t in bs[bp[v]:bp[v + 1]]}
    F = lambda s, u: s * nf + u
    B = lambda s, v: n_stages * nf + s * nb + v
    vertices = [(s, FWD, u) for s in range(n_stages) for u in range(nf)] + [(s, BWD, v) for s in range(n_stages) for v in range(nb)]
    weights = [fwd_cost[u] for _ in range(n_stages) for u in range(nf)] + [bwd_cost[v] for _ in range(n_stages) for v in range(nb)]
    by_sample: Dict[int, List[int]] = {}
    for t, rec in enumerate(slices):
        by_sample.setdefault(int(rec[0]), []).append(t)
    for ts in by_sample.values():
        ts.sort(key=lambda t: int(slices[t][1]))
    edges = []
    # inter-stage
    for s in range(n_stages - 1):
        edges += [(F(s, u), F(s + 1, u), EDGE_STAGE) for u in range(nf)]
    edges += [(F(n_stages - 1, u), B(n_stages - 1, v), EDGE_STAGE) for u, v in sorted({(fwd_of[t], bwd_of[t]) for t in range(len(slices))})]
    for s in range(n_stages - 1, 0, -1):
        edges += [(B(s, v), B(s - 1, v), EDGE_STAGE) for v in range(nb)]
    # inter-slice
    ff = sorted({(fwd_of[a], fwd_of[b]) for ts in by_sample.values() for a, b in zip(ts, ts[1:]) if fwd_of[a] != fwd_of[b]})
    bb = sorted({(bwd_of[b], bwd_of[a]) for ts in by_sample.values() for a, b in zip(ts, ts[1:]) if bwd_of[a] != bwd_of[b]})
    for s in range(n_stages):
        edges += [(F(s, a), F(s, b), EDGE_SLICE) for a, b in ff]
        edges += [(B(s, a), B(s, b), EDGE_SLICE) for a, b in bb]
    # schedule
    need = [0] * nb
    for ts in by_sample.values():
        last = max(fwd_of[t] for t in ts)
        for t in ts:
            need[bwd_of[t]] = max(need[bwd_of[t]], last + 1)
    for s in range(n_stages):
        order, i, j = [], 0, 0
        warm = min(n_stages - 1 - s, nf)
        while i < warm:
            order.append(F(s, i)); i += 1
        while i < nf:
            order.append(F(s, i)); i += 1
            if j < nb and need[j] <= i:
                order.append(B(s, j)); j += 1
        while j < nb:
            order.append(B(s, j)); j += 1
        edges += [(a, b, EDGE_SCHEDULE) for a, b in zip(order, order[1:])]
    return vertices, weights, edges


# ---- memory footprint over the timeline ---------------------------------------------------------------------

def memory_peaks(start: Sequence[int], finish: Sequence[int], buffers, n_stages: int, base: Sequence[int]):
    """Peak live bytes per stage, and the earliest time it is reached, straight from the definition.

    Paper, Memory footprint simulation: with the execution timeline known, allocations and releases are events
    in time, and the live size is followed chronologically.  A buffer (stage, bytes, alloc_vertex, free_vertex)
    is live from Start(alloc_vertex) up to, not including, Finish(free_vertex): what is released at an instant
    is gone before what is allocated at that instant arrives.  `base` is the stage's constant part (weights,
    optimizer states).  The live size only rises at allocation instants, so those are the only candidates."""
    peaks, times = [], []
    for s in range(n_stages):
        mine = [(int(by), start[a], finish[f]) for st, by, a, f in buffers if st == s]
        for by, t0, t1 in mine:
            if t1 < t0:
                raise ValueError("a buffer is released before it is allocated")
        best, at = 0, 0
        for t in sorted({t0 for _, t0, _ in mine}):
            live = sum(by for by, t0, t1 in mine if t0 <= t < t1)
            if live > best:
                best, at = live, t
        peaks.append(int(base[s]) + best)
        times.append(at)
    return peaks, times


def buffers_1f1b(slices, fwd_units, bwd_units, n_stages: int, act_bytes: int, kv_bytes: int, grad_bytes: int, per_slice: bool):
    """Buffers of the 1F1B graph of `build_1f1b` (same vertex ids), three per (stage, slice), in that order:

    activations   act_bytes per token of the slice: from the slice's forward task to its backward task
                  (Memory footprint simulation: held until consumption by the corresponding backward task);
    KV cache      kv_bytes per token: from the slice's forward task to the last backward task of the stage
                  that needs it, i.e. the last unit with a slice of the same sample at or after it
                  (KV cache managed per slice according to the schedule);
    KV gradients  grad_bytes per token: from the first backward task that adds to them -- the first unit with a
                  slice of the sample at or after it -- to the last one.
    With per_slice False the KV cache and the gradients live sample-wise instead: the whole sample's cache
    from the sample's first forward task to its last backward task, its gradients from its first backward task
    to its last."""
    (fp, fs), (bp, bs) = fwd_units, bwd_units
    nf, nb = len(fp) - 1, len(bp) - 1
    fwd_of = {int(t): u for u in range(nf) for t in fs[fp[u]:fp[u + 1]]}
    bwd_of = {int(t): v for v in range(nb) for t in bs[bp[v]:bp[v + 1]]}
    F = lambda s, u: s * nf + u
    B = lambda s, v: n_stages * nf + s * nb + v
    out = []
    for s in range(n_stages):
        for t, rec in enumerate(slices):
            sample, idx, q_len = int(rec[0]), int(rec[1]), int(rec[3])
            same = [x for x, r in enumerate(slices) if int(r[0]) == sample]
            after = [x for x in same if int(slices[x][1]) >= idx] if per_slice else same
            first_b, last_b = min(bwd_of[x] for x in after), max(bwd_of[x] for x in after)
            kv_from = fwd_of[t] if per_slice else min(fwd_of[x] for x in same)
            out.append((s, act_bytes * q_len, F(s, fwd_of[t]), B(s, bwd_of[t])))
            out.append((s, kv_bytes * q_len, F(s, kv_from), B(s, last_b)))
            out.append((s, grad_bytes * q_len, B(s, first_b), B(s, last_b)))
    return out
