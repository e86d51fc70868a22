"""Search oracle: which number of scheduling units gives the shortest simulated iteration.

Paper: Balanced Packing & Asymmetric Partitioning Solver (the MicroPack count m sets the per-unit budget W / m and
several m are evaluated), Primitive Measurements and Search Space (m is quantised to multiples of the pipeline
width and sampled on a roughly logarithmic grid; a unit's runtime is its theoretical cost converted with
calibrated utilisations), DAG-based Pipeline Simulator (time and memory of a candidate schedule).

Written as the composition of the other oracles, one candidate after the other: the exact partition for m units
per pass (solver.py), every unit priced as  fixed + cost * num // den  with cost = w_quad * pairs + w_lin * rows
of its slices (tables.py), the 1F1B graph and its timeline (dag.py), the per-slice buffers and the worst
stage's peak (dag.py).  The best candidate has the smallest simulated time among those whose peak stays within
the limit; ties go to the earlier candidate.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

from . import dag as D
from . import solver as V
from . import tables as T


def candidate_unit_counts(n_stages: int, m_max: int) -> List[int]:
    """m = i * n_stages <= m_max for i = 1, 2, 3, 4, 6, 8, 12, 16, 24, ...: the powers of two and the values halfway
    between two of them (this build's grid for the paper's roughly logarithmic sampling of i)."""
    grid, p2 = [], 1
    while p2 * n_stages <= m_max:
        grid.append(p2)
        if p2 >= 2:
            grid.append(p2 + p2 // 2)
        p2 *= 2
    return [i * n_stages for i in sorted(grid) if i * n_stages <= m_max]


def evaluate(lengths: Sequence[int], m: int, solver: dict, n_stages: int, fwd_rate, bwd_rate, act_bytes: int, kv_bytes: int,
             grad_bytes: int):
    """(t_total, worst stage's peak) of candidate m, or None if the token cap rules m units out.  fwd_rate, bwd_rate =
    (fixed, num, den)."""
    params = dict(solver)
    params["m_fwd"] = params["m_bwd"] = m
    try:
        r = V.solve_partition(lengths, **params)
    except ValueError:
        return None
    sl, fwd, bwd = r["slices"], r["fwd"], r["bwd"]

    def times(units, w_quad, w_lin, rate):
        fixed, num, den = rate
        return [fixed + c * num // den for c in T.unit_costs(sl, units[0], units[1], w_quad, w_lin)]
    fc = times(fwd, params["w_quad_fwd"], params["w_lin_fwd"], fwd_rate)
    bc = times(bwd, params["w_quad_bwd"], params["w_lin_bwd"], bwd_rate)
    vertices, weights, edges = D.build_1f1b(sl, fwd, bwd, n_stages, fc, bc)
    start, finish, total = D.timeline(weights, [(u, v) for u, v, _ in edges])
    bufs = D.buffers_1f1b(sl, fwd, bwd, n_stages, act_bytes, kv_bytes, grad_bytes, True)
    peaks, _ = D.memory_peaks(start, finish, bufs, n_stages, [0] * n_stages)
    return total, max(peaks)


def search_unit_count(lengths: Sequence[int], m_list: Sequence[int], solver: dict, n_stages: int, fwd_rate, bwd_rate, act_bytes: int = 0,
                      kv_bytes: int = 0, grad_bytes: int = 0, stage_bytes_cap: int = 0):
    """(t_total per candidate, peak per candidate, index of the best or -1); -1 entries where a candidate is infeasible."""
    t_total, peak = [], []
    for m in m_list:
        r = evaluate(lengths, int(m), solver, n_stages, fwd_rate, bwd_rate, act_bytes, kv_bytes, grad_bytes)
        t_total.append(-1 if r is None else r[0])
        peak.append(-1 if r is None else r[1])
    best: Optional[int] = None
    for i in range(len(t_total)):
        if t_total[i] < 0 or (stage_bytes_cap > 0 and peak[i] > stage_bytes_cap):
            continue
        if best is None or t_total[i] < t_total[best]:
            best = i
    return t_total, peak, (-1 if best is None else best)
