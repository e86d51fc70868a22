"""Pins for the table oracle: a hand-derived fixture, brute-force enumeration on tiny inputs,
counting identities and the paper's forward:backward cost ratio."""
import itertools
import json
import os

import numpy as np
import pytest

import workloads as W
from oracle import tables as T

GOLD = os.path.join(os.path.dirname(__file__), "golden", "cfg0_tables.json")
GOLD_POLICIES = os.path.join(os.path.dirname(__file__), "golden", "policies_tiny.json")


def _units(up, us):
    return [us[up[u]:up[u + 1]].tolist() for u in range(len(up) - 1)]


def _golden_policy_mismatches(build_slices, build_units):
    """Every case of the hand-worked fixture that (build_slices, build_units) does not reproduce."""
    g = json.load(open(GOLD_POLICIES))
    bad = []
    for key in ("input_A", "input_B"):
        inp = g[key]
        cu, sl = build_slices(inp["lengths"], inp["slice_size"])
        assert cu.tolist() == inp["cu"]
        assert [T.pairs_of_slice(r) for r in sl] == inp["pairs"] and [int(r[3]) for r in sl] == inp["q_len"]
        for case in inp["cases"]:
            up, us = build_units(cu, sl, case["policy"], **case["params"])
            if _units(up, us) != case["units"]:
                bad.append((key, case["policy"], case["params"], _units(up, us)))
    return bad


def test_golden_cfg0_tables():
    g = json.load(open(GOLD))
    cu, sl = T.build_slices(g["lengths"], g["slice_size"])
    assert cu.tolist() == g["cu"] and sl.tolist() == g["slices"]
    w = W.WORKLOADS["cfg0_tiny_f32"]
    up, us = T.build_units(cu, sl, w.fwd_policy[0], **w.fwd_policy[1])
    assert up.tolist() == g["fwd_unit_ptr"] and us.tolist() == g["fwd_unit_slices"]
    up, us = T.build_units(cu, sl, w.bwd_policy[0], **w.bwd_policy[1])
    assert up.tolist() == g["bwd_unit_ptr"] and us.tolist() == g["bwd_unit_slices"]
    assert sum(T.pairs_of_slice(r) for r in sl) == g["pairs_total"]
    assert [T.pairs_of_sample(L) for L in g["lengths"]] == g["pairs_per_sample"]


def test_golden_hand_worked_policies():
    """PREFIX_FILL (forward, backward, mixed cost), TOKEN_CAP, SEEDED_LPT, ISOLATE_FILL, PER_SAMPLE and
    ROUND_ROBIN on two tiny inputs worked by hand; the inputs are chosen so that a start-point or end-point
    rule in place of the midpoint rule, or an ISOLATE_FILL that fills m instead of m - n_isolated units,
    gives other lists (the fixture records those too)."""
    assert _golden_policy_mismatches(T.build_slices, T.build_units) == []
    g = json.load(open(GOLD_POLICIES))
    for inp in (g["input_A"], g["input_B"]):
        cu, sl = T.build_slices(inp["lengths"], inp["slice_size"])
        assert T._walk(cu, sl, False) == inp["walk_forward"] and T._walk(cu, sl, True) == inp["walk_backward"]
        for case in inp["cases"]:
            for wrong in ("start_point_units", "end_point_units", "fill_m_units"):
                assert case.get(wrong) != case["units"]
            flat = sorted(t for u in case["units"] for t in u)
            assert flat == list(range(len(sl)))


def test_golden_catches_planted_rule_changes(monkeypatch):
    """A mistake planted in the oracle (here, on the CPU) must fail the fixture: the start-point and the
    end-point variants of the fill rule, and a walk that ignores the descending-length order."""
    real_fill, real_walk = T._prefix_fill, T._walk

    def fill_variant(kind):
        def f(walk, slices, m, w_quad, w_lin):
            total = sum(T._cost(slices[t], w_quad, w_lin) for t in walk)
            groups = [[] for _ in range(m)]
            before = 0
            for t in walk:
                c = T._cost(slices[t], w_quad, w_lin)
                num = before if kind == "start" else before + c
                groups[min(m - 1, (m * num) // total if total > 0 else 0)].append(t)
                before += c
            return groups
        return f

    for kind in ("start", "end"):
        monkeypatch.setattr(T, "_prefix_fill", fill_variant(kind))
        bad = _golden_policy_mismatches(T.build_slices, T.build_units)
        assert any(b[1] == "PREFIX_FILL" for b in bad), kind
    monkeypatch.setattr(T, "_prefix_fill", lambda walk, slices, m, wq, wl: real_fill(walk, slices, m + 1, wq, wl))
    assert any(b[1] == "ISOLATE_FILL" for b in _golden_policy_mismatches(T.build_slices, T.build_units))
    monkeypatch.setattr(T, "_prefix_fill", real_fill)

    def table_order_walk(cu, slices, backward):                      # samples in index order
        out = []
        for s in range(len(cu) - 1):
            ts = [t for t in range(len(slices)) if int(slices[t][0]) == s]
            out.extend(ts[::-1] if backward else ts)
        return out
    monkeypatch.setattr(T, "_walk", table_order_walk)
    assert _golden_policy_mismatches(T.build_slices, T.build_units) != []
    monkeypatch.setattr(T, "_walk", real_walk)
    assert _golden_policy_mismatches(T.build_slices, T.build_units) == []


def test_pairs_by_brute_force():
    lengths = [1, 2, 9, 17]
    for S in (1, 2, 4, 7, 32):
        cu, sl = T.build_slices(lengths, S)
        for rec in sl:
            s, _, qs, ql, ks, kl = [int(x) for x in rec[:6]]
            brute = sum(1 for i in range(qs, qs + ql) for j in range(ks, ks + kl) if j <= i)
            assert T.pairs_of_slice(rec) == brute
        assert sum(T.pairs_of_slice(r) for r in sl) == sum(L * (L + 1) // 2 for L in lengths)


def test_flop_ratio_is_two_and_a_half():
    # paper, Asymmetric Cost Profile: attention backward ~2.5x forward (scores recomputed)
    for pairs in (1, 12345, 34_411_815_512):
        assert 2 * T.flops_bwd(pairs, 128, 32) == 5 * T.flops_fwd(pairs, 128, 32)
        assert T.flops_fwd(pairs, 128, 32) == 4 * 128 * 32 * pairs


ALL_POLICIES = [
    ("ALL", {}), ("PER_SAMPLE", {}), ("PER_SAMPLE", {"backward": True}),
    ("ROUND_ROBIN", {"m": 3}), ("ROUND_ROBIN", {"m": 4, "descending": True}),
    ("PREFIX_FILL", {"m": 3, "w_quad": 2, "w_lin": 0, "backward": False}),
    ("PREFIX_FILL", {"m": 5, "w_quad": 5, "w_lin": 7, "backward": True}),
    ("TOKEN_CAP", {"cap": 10, "backward": False}), ("TOKEN_CAP", {"cap": 3, "backward": True}),
    ("SEEDED_LPT", {"w_quad": 2, "w_lin": 0}), ("SEEDED_LPT", {"w_quad": 2, "w_lin": 1, "m_min": 3}),
    ("ISOLATE_FILL", {"m": 4, "w_quad": 5, "w_lin": 0, "theta_num": 1, "theta_den": 1, "backward": True}),
    ("ISOLATE_FILL", {"m": 3, "w_quad": 2, "w_lin": 1, "theta_num": 1, "theta_den": 2, "backward": False}),
]


@pytest.mark.parametrize("policy,params", ALL_POLICIES)
def test_every_policy_covers_each_slice_once(policy, params):
    for lengths, S in itertools.product([[5], [1, 1, 1], [9, 2, 14, 3], [4, 4, 4, 4, 4]], [1, 3, 4, 8]):
        cu, sl = T.build_slices(lengths, S)
        up, us = T.build_units(cu, sl, policy, **params)
        assert T.check_structure(cu, sl, up, us) == []
        assert sorted(us.tolist()) == list(range(len(sl)))
        assert all(up[i + 1] > up[i] for i in range(len(up) - 1))      # no empty units


@pytest.mark.parametrize("policy,params", [p for p in ALL_POLICIES if p[0] not in ("ROUND_ROBIN", "ALL")])
def test_walk_order_policies_obey_pipeline_rules(policy, params):
    backward = bool(params.get("backward", False))
    for lengths, S in itertools.product([[9, 2, 14, 3], [30], [2, 2, 40]], [2, 4, 8]):
        cu, sl = T.build_slices(lengths, S)
        up, us = T.build_units(cu, sl, policy, **params)
        assert T.check_order(sl, up, us, backward) == []


def test_prefix_fill_units_close_to_target():
    # every unit's cost stays within one maximal slice cost of W/m (midpoint rule)
    r = np.random.default_rng(5)
    for _ in range(20):
        lengths = r.integers(1, 400, size=r.integers(1, 12)).tolist()
        S = int(r.integers(1, 64)); m = int(r.integers(1, 9))
        cu, sl = T.build_slices(lengths, S)
        for wq, wl, bw in ((2, 0, False), (5, 3, True)):
            up, us = T.build_units(cu, sl, "PREFIX_FILL", m=m, w_quad=wq, w_lin=wl, backward=bw)
            costs = T.unit_costs(sl, up, us, wq, wl)
            total = sum(costs)
            cmax = max(wq * T.pairs_of_slice(x) + wl * int(x[3]) for x in sl)
            assert len(costs) <= m and all(abs(c * m - total) <= cmax * m for c in costs)
            pos = {int(t): i for i, t in enumerate(us)}            # units contiguous in walk order
            assert us.tolist() == [t for t in sorted(pos, key=pos.get)]


def test_token_cap_respected_and_maximal():
    cu, sl = T.build_slices([100, 7, 33, 64], 16)
    up, us = T.build_units(cu, sl, "TOKEN_CAP", cap=40, backward=False)
    toks = [int(sum(sl[t][3] for t in us[up[u]:up[u + 1]])) for u in range(len(up) - 1)]
    assert all(t <= 40 for t in toks)
    for u in range(len(up) - 2):                                    # next-fit: the next slice did not fit
        assert toks[u] + int(sl[us[up[u + 1]]][3]) > 40


def test_seeded_lpt_brute_force():
    lengths = [40, 3, 9, 5, 8]
    cu, sl = T.build_slices(lengths, 16)          # sample 0 -> 3 seed slices; others single
    up, us = T.build_units(cu, sl, "SEEDED_LPT", w_quad=2, w_lin=0)
    units = [us[up[u]:up[u + 1]].tolist() for u in range(len(up) - 1)]
    assert [u[0] for u in units] == [0, 1, 2]
    # replay by hand: singles in descending length (9,8,5,3) -> slices 4,6,5,3; loads 2*pairs
    load = [2 * T.pairs_of_slice(sl[t]) for t in (0, 1, 2)]
    want = [[0], [1], [2]]
    for t in (4, 6, 5, 3):
        i = load.index(min(load))
        want[i].append(t); load[i] += 2 * T.pairs_of_slice(sl[t])
    assert units == want


def test_isolate_fill_isolates_heavy_slices():
    cu, sl = T.build_slices([64, 4, 4, 4], 8)
    up, us = T.build_units(cu, sl, "ISOLATE_FILL", m=4, w_quad=5, w_lin=0, theta_num=1, theta_den=1,
                           backward=True)
    total = sum(5 * T.pairs_of_slice(x) for x in sl)
    for u in range(len(up) - 1):
        ts = us[up[u]:up[u + 1]]
        heavy = [t for t in ts if 5 * T.pairs_of_slice(sl[t]) * 4 >= total]
        assert not heavy or len(ts) == 1


def test_validator_flags_each_planted_fault():
    cu, sl = T.build_slices([10, 6], 4)
    up, us = T.build_units(cu, sl, "PER_SAMPLE")
    assert T.check_structure(cu, sl, up, us) == []
    bad = sl.copy(); bad[1, 3] += 1
    assert "tiling" in T.check_structure(cu, bad, up, us) or "kv_range" in T.check_structure(cu, bad, up, us)
    bad = sl.copy(); bad[2, 5] -= 1
    assert "kv_range" in T.check_structure(cu, bad, up, us)
    bad = sl.copy(); bad[3, 4] += 1
    assert "kv_range" in T.check_structure(cu, bad, up, us)
    dup = us.copy(); dup[0] = dup[1]
    assert "coverage" in T.check_structure(cu, sl, up, dup)
    oob = us.copy(); oob[0] = 99
    assert "slice_range" in T.check_structure(cu, sl, up, oob)
    assert "unit_ptr" in T.check_structure(cu, sl, np.array([0, 2, 1, 5]), us)
    rev = np.array([1, 0, 2, 3, 4], np.int32)
    assert "adjacency" in T.check_order(sl, up, rev, False) or "unit_order" in T.check_order(sl, up, rev, False)
    assert T.check_order(sl, up, us, True) != []                     # ascending order is not FILO


def test_workload_policies_are_valid_for_every_seed():
    for name, w in W.WORKLOADS.items():
        if name.startswith("cfg4") and name != "cfg4_d128_s1024":
            continue
        for seed in W.SEEDS:
            L = W.draw_lengths(w, np.random.default_rng(seed))
            cu, sl = T.build_slices(L, w.slice_size)
            for pol, p in (w.fwd_policy, w.bwd_policy):
                up, us = T.build_units(cu, sl, pol, **p)
                assert T.check_structure(cu, sl, up, us) == []
