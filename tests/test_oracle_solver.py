"""Pins for the partition oracle (oracle/solver.py): a hand-worked fixture, brute force over every set of
cuts on tiny inputs, closed forms and bounds."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import solver as SV
from oracle import tables as T

GOLD = os.path.join(os.path.dirname(__file__), "golden", "solver_tiny.json")


def _units_rows(units):
    """[(sample, a, b) granules] per unit -> merged row ranges per sample, in walk order."""
    out = []
    for unit in units:
        rows = []
        for s, a, b in unit:
            if rows and rows[-1][0] == s:
                rows[-1] = [s, min(rows[-1][1], a), max(rows[-1][2], b)]
            else:
                rows.append([s, a, b])
        out.append(rows)
    return out


def test_golden_hand_worked_partitions():
    g = json.load(open(GOLD))
    for case in g["cases"]:
        B, units = SV.solve_pass(g["lengths"], case["m"], case["w_quad"], case["w_lin"], g["granule"],
                                 case["pass"] == "backward", case["token_cap"])
        assert B == case["bottleneck"], case["_derivation"][:40]
        assert _units_rows(units) == case["units_rows"]
    p = g["partition"]
    r = SV.solve_partition(g["lengths"], p["m_fwd"], p["m_bwd"], 2, 0, 5, 0, granule=1)
    assert r["slices"].tolist() == p["slices"]
    for key, want in (("fwd", p["fwd_units"]), ("bwd", p["bwd_units"])):
        up, us = r[key]
        assert [us[up[u]:up[u + 1]].tolist() for u in range(len(up) - 1)] == want


def _brute_force(costs, tokens, m, cap):
    n = len(costs)
    best = None
    for k in range(0, min(m, n)):
        for cuts in itertools.combinations(range(1, n), k):
            edges = (0,) + cuts + (n,)
            parts = [(edges[i], edges[i + 1]) for i in range(len(edges) - 1)]
            if cap > 0 and any(sum(tokens[a:b]) > cap and b - a > 1 for a, b in parts):
                continue
            worst = max(sum(costs[a:b]) for a, b in parts)
            best = worst if best is None else min(best, worst)
    return best


def test_bottleneck_equals_brute_force_over_all_cuts():
    r = np.random.default_rng(11)
    for _ in range(60):
        lengths = r.integers(1, 9, size=r.integers(1, 4)).tolist()
        granule = int(r.integers(1, 4))
        wq, wl = int(r.integers(0, 6)), int(r.integers(0, 4))
        if wq == 0 and wl == 0:
            wl = 1
        for backward in (False, True):
            gr = SV.granules(lengths, granule, backward)
            if len(gr) > 12:
                continue
            costs = [SV.piece_cost(a, b, wq, wl) for _, a, b in gr]
            toks = [b - a for _, a, b in gr]
            for m in (1, 2, 3, 5, 12):
                for cap in (0, 3, 7):
                    want = _brute_force(costs, toks, m, cap)
                    got = SV.min_max_bottleneck(costs, toks, m, cap)
                    assert got == want, (lengths, granule, wq, wl, backward, m, cap)
                    if want is not None:        # the canonical cuts reach the optimum with at most m units
                        starts = SV.greedy_cuts(costs, toks, want, cap) + [len(gr)]
                        assert len(starts) - 1 <= m
                        assert max(sum(costs[starts[u]:starts[u + 1]]) for u in range(len(starts) - 1)) == want


def test_closed_forms_and_bounds():
    lengths = [40, 7, 19, 1]
    W2 = sum(2 * T.pairs_of_sample(L) for L in lengths)
    assert SV.solve_pass(lengths, 1, 2, 0, 1, False)[0] == W2                        # one unit holds everything
    assert SV.solve_pass(lengths, sum(lengths), 2, 0, 1, False)[0] == 2 * 40        # one row per unit: the costliest row
    assert SV.solve_pass(lengths, 5, 0, 1, 1, True)[0] == -(-sum(lengths) // 5)      # unit cost = rows: ceil(T / m)
    assert SV.solve_pass(lengths, 3, 0, 1, 8, False)[0] == 24                        # granules of 8 rows: 67 rows, 3 units
    prev = None
    for m in range(1, 12):
        for wq, wl, bw in ((2, 0, False), (5, 3, True)):
            B, units = SV.solve_pass(lengths, m, wq, wl, 4, bw)
            gr = SV.granules(lengths, 4, bw)
            costs = [SV.piece_cost(a, b, wq, wl) for _, a, b in gr]
            W = sum(costs)
            assert -(-W // m) <= B <= W // m + max(costs)      # within one granule of tau = W / m
            assert len(units) <= m
        Bf = SV.solve_pass(lengths, m, 2, 0, 4, False)[0]
        assert prev is None or Bf <= prev                       # more units never raise the optimum
        prev = Bf


def test_partition_is_a_valid_asymmetric_table():
    r = np.random.default_rng(3)
    for _ in range(25):
        lengths = r.integers(0, 60, size=r.integers(1, 7)).tolist()
        if sum(lengths) == 0:
            continue
        mf, mb = int(r.integers(1, 7)), int(r.integers(1, 9))
        res = SV.solve_partition(lengths, mf, mb, 2, 1, 5, 2, granule=int(r.integers(1, 6)), max_slice=int(r.choice([0, 16])))
        cu, sl = res["cu"], res["slices"]
        for key, backward, wq, wl, B, m in (("fwd", False, 2, 1, res["bottleneck_fwd"], mf), ("bwd", True, 5, 2, res["bottleneck_bwd"], mb)):
            up, us = res[key]
            assert T.check_structure(cu, sl, up, us) == [] and T.check_order(sl, up, us, backward) == []
            costs = T.unit_costs(sl, up, us, wq, wl)
            assert len(costs) <= m and max(costs) == B
        # the same slices, cut by the table oracle's own routine from the bounds
        cu2, sl2 = T.build_slices_from_bounds(lengths, res["bounds"])
        assert np.array_equal(cu, cu2) and np.array_equal(sl, sl2)


def test_backward_partition_differs_from_forward_one():
    # one long sample, quadratic costs: forward units get shorter towards the sample's end, backward units are
    # walked from the end; same multiset of row ranges is not required and in general not obtained
    res = SV.solve_partition([64], 4, 4, 2, 0, 5, 0, granule=1)
    f = [int(res["slices"][t][2]) for t in res["fwd"][1]]
    b = [int(res["slices"][t][2]) for t in res["bwd"][1]]
    assert f == sorted(f) and b == sorted(b, reverse=True)
    fu = T.unit_costs(res["slices"], *res["fwd"], 2, 0)
    bu = T.unit_costs(res["slices"], *res["bwd"], 5, 0)
    assert max(fu) == res["bottleneck_fwd"] and max(bu) == res["bottleneck_bwd"]
    assert res["bottleneck_fwd"] * 5 != res["bottleneck_bwd"] * 2 or res["fwd"][0].tolist() != res["bwd"][0].tolist()
