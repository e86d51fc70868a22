"""Partition oracle: exact min-max cut of the packed samples into m scheduling units per pass.

What it decides (paper: Balanced Packing & Asymmetric Partitioning Solver -- Phase 2 cuts long samples into
slices and packs short ones so that every unit's work is close to the per-unit target tau = W / m, and the
slice boundaries come out of the optimisation; Asymmetric Partition -- the backward pass gets a partition of
its own for the same samples, computed from backward costs, without changing the order of the units).

Model.  Samples are walked in the order the paper prescribes (descending forward cost, i.e. descending
length, ties by index); inside a sample the forward pass walks the rows upwards, the backward pass
downwards (first-in last-out).  Row i (0-based inside its sample) costs  w_quad * (i + 1) + w_lin:  it sees
i + 1 keys.  A unit is a contiguous piece of the walk; its cost is the sum of its rows' costs, so the cost of
rows [a, b) of a sample is w_quad * pairs + w_lin * (b - a) with pairs = (b-a)*a + (b-a)(b-a+1)/2, exactly
the slice cost of the table oracle.  Cuts may fall only on multiples of `granule` rows from a sample's start
(and on sample boundaries).  Optionally a unit may hold at most `token_cap` rows (memory grows linearly with
tokens).  Wanted: at most m units with the smallest possible largest unit cost B*.

This file states that by dynamic programming over the granules, in plain Python integers -- slow and obviously
right.  Because many cuts reach B*, the cuts are then fixed canonically: walk the sequence and close a unit only
when the next granule would push it over B* (or over the token cap).  The slice table is the union of the
forward and backward cuts (plus cuts every `max_slice` rows if asked), so that both unit lists group whole
slices of one table.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def _walk_samples(lengths: Sequence[int]) -> List[int]:
    return sorted(range(len(lengths)), key=lambda s: (-int(lengths[s]), s))


def granules(lengths: Sequence[int], granule: int, backward: bool) -> List[Tuple[int, int, int]]:
    """The walk as a list of (sample, a, b): rows [a, b) of the sample, a multiple of `granule` (last one ragged)."""
    out = []
    for s in _walk_samples(lengths):
        L = int(lengths[s])
        pieces = [(s, a, min(L, a + granule)) for a in range(0, L, granule)]
        out.extend(reversed(pieces) if backward else pieces)
    return out


def piece_cost(a: int, b: int, w_quad: int, w_lin: int) -> int:
    n = b - a
    return w_quad * (n * a + n * (n + 1) // 2) + w_lin * n


def min_max_bottleneck(costs: List[int], tokens: List[int], m: int, token_cap: int = 0):
    """Smallest B such that the sequence splits into at most m contiguous parts, each of cost <= B and (if
    token_cap > 0) of at most token_cap tokens; None if no split exists (a single granule over the cap is
    allowed to stand alone: a unit always takes at least one granule).  O(N^2 m) dynamic programme."""
    n = len(costs)
    if n == 0:
        return 0
    INF = float("inf")
    pc, pt = [0], [0]
    for c, t in zip(costs, tokens):
        pc.append(pc[-1] + c)
        pt.append(pt[-1] + t)

    def ok_tokens(j, i):          # part = granules j .. i-1
        return token_cap <= 0 or pt[i] - pt[j] <= token_cap or i - j == 1

    best = [[INF] * (n + 1) for _ in range(m + 1)]
    best[0][0] = 0
    for k in range(1, m + 1):
        for i in range(1, n + 1):
            for j in range(i):
                if best[k - 1][j] < INF and ok_tokens(j, i):
                    best[k][i] = min(best[k][i], max(best[k - 1][j], pc[i] - pc[j]))
    ans = min(best[k][n] for k in range(1, m + 1))
    return None if ans == INF else ans


def greedy_cuts(costs: List[int], tokens: List[int], bound: int, token_cap: int = 0) -> List[int]:
    """Canonical cuts for a bound: a unit is closed when the next granule would push it over `bound` or over the
    token cap.  Returns the start index of every unit (first is 0)."""
    starts, c, t = [], 0, 0
    for i, (ci, ti) in enumerate(zip(costs, tokens)):
        if i == 0 or c + ci > bound or (token_cap > 0 and t + ti > token_cap):
            starts.append(i)
            c, t = 0, 0
        c += ci
        t += ti
    return starts


def solve_pass(lengths, m: int, w_quad: int, w_lin: int, granule: int, backward: bool, token_cap: int = 0):
    """(bottleneck B*, units) for one pass; units = list of lists of (sample, a, b) granules in walk order."""
    gr = granules(lengths, granule, backward)
    costs = [piece_cost(a, b, w_quad, w_lin) for _, a, b in gr]
    toks = [b - a for _, a, b in gr]
    B = min_max_bottleneck(costs, toks, m, token_cap)
    if B is None:
        raise ValueError("no partition into at most m units under the token cap")
    starts = greedy_cuts(costs, toks, B, token_cap) + [len(gr)]
    return B, [gr[starts[u]:starts[u + 1]] for u in range(len(starts) - 1)]


def solve_partition(lengths, m_fwd: int, m_bwd: int, w_quad_fwd: int, w_lin_fwd: int, w_quad_bwd: int, w_lin_bwd: int,
                    granule: int = 1, token_cap_fwd: int = 0, token_cap_bwd: int = 0, max_slice: int = 0):
    """Slice bounds and both unit lists.  Returns dict with `bounds` (interior cut points per sample), `cu`, `slices`
    (8-int records), `fwd` / `bwd` = (unit_ptr, unit_slices), `bottleneck_fwd`, `bottleneck_bwd`."""
    n = len(lengths)
    Bf, uf = solve_pass(lengths, m_fwd, w_quad_fwd, w_lin_fwd, granule, False, token_cap_fwd)
    Bb, ub = solve_pass(lengths, m_bwd, w_quad_bwd, w_lin_bwd, granule, True, token_cap_bwd)
    cuts = [set() for _ in range(n)]
    for units in (uf, ub):
        for unit in units:
            by_sample = {}
            for s, a, b in unit:
                lo, hi = by_sample.get(s, (a, b))
                by_sample[s] = (min(lo, a), max(hi, b))
            for s, (lo, hi) in by_sample.items():        # a unit holds one contiguous row range of a sample
                for c in (lo, hi):
                    if 0 < c < int(lengths[s]):
                        cuts[s].add(c)
    if max_slice > 0:
        for s in range(n):
            cuts[s].update(range(max_slice, int(lengths[s]), max_slice))
    bounds = [sorted(c) for c in cuts]
    cu = [0]
    for L in lengths:
        cu.append(cu[-1] + int(L))
    rows, index = [], {}
    for s in range(n):
        if int(lengths[s]) == 0:
            continue
        edges = [0] + bounds[s] + [int(lengths[s])]
        for idx in range(len(edges) - 1):
            a, b = edges[idx], edges[idx + 1]
            index[(s, a)] = len(rows)
            rows.append([s, idx, cu[s] + a, b - a, cu[s], b, 0, 0])

    def unit_lists(units, backward):
        ptr, flat = [0], []
        for unit in units:
            seen = []
            for s, a, b in unit:                          # slices whose rows lie in the unit, in walk order
                starts = [x for x in ([0] + bounds[s]) if a <= x < b]
                for x in (reversed(starts) if backward else starts):
                    seen.append(index[(s, x)])
            flat.extend(seen)
            ptr.append(len(flat))
        return np.asarray(ptr, np.int32), np.asarray(flat, np.int32)

    return {"bounds": bounds, "cu": np.asarray(cu, np.int32), "slices": np.asarray(rows, np.int32).reshape(-1, 8),
            "fwd": unit_lists(uf, False), "bwd": unit_lists(ub, True), "bottleneck_fwd": Bf, "bottleneck_bwd": Bb}
