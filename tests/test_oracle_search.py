"""Pins for the search oracle (oracle/search.py) and the native search against it: the candidate grid written out by
hand, the closed form of equal units through a uniform pipeline, the single-stage case (the iteration is the sum
of its tasks), the memory limit changing the choice, and agreement of the C++ routine on random inputs."""
import numpy as np
import pytest

import paper_2509_26246_amd as S
from oracle import search as Q
from oracle import solver as V

WEIGHTS = dict(w_quad_fwd=2, w_lin_fwd=0, w_quad_bwd=5, w_lin_bwd=0)


def test_candidate_grid():
    # i = 1, 2, 3, 4, 6, 8, 12, 16, 24, 32, ... times the pipeline width, up to the limit
    assert Q.candidate_unit_counts(4, 100) == [4, 8, 12, 16, 24, 32, 48, 64, 96]
    assert Q.candidate_unit_counts(1, 13) == [1, 2, 3, 4, 6, 8, 12]
    assert Q.candidate_unit_counts(8, 7) == []
    assert Q.candidate_unit_counts(3, 3) == [3]
    for p, m_max in [(4, 100), (1, 13), (8, 7), (3, 3), (2, 1000), (5, 64), (1, 0)]:
        assert S.candidate_unit_counts(p, m_max).tolist() == Q.candidate_unit_counts(p, m_max)
    got = Q.candidate_unit_counts(2, 1000)
    assert all(m % 2 == 0 for m in got) and got == sorted(set(got))
    ratios = [b / a for a, b in zip(got[2:], got[3:])]
    assert all(1.3 <= r <= 1.51 for r in ratios)                        # roughly logarithmic


@pytest.mark.parametrize("p", [1, 3, 4])
def test_equal_units_through_a_uniform_pipeline(p):
    # 12 equal samples of one granule each: m | 12 units of 12/m samples, all of the same cost, and the textbook
    # iteration time (m + p - 1)(f + b) with f = F + cost_f * num // den per unit
    n_s, g = 12, 8
    lengths = [g] * n_s
    c_f, c_b = 2 * g * (g + 1) // 2, 5 * g * (g + 1) // 2                # one sample: w_quad * pairs
    solver = dict(WEIGHTS, granule=g)
    fwd_rate, bwd_rate = (40, 3, 2), (55, 7, 4)
    m_list = [1, 2, 3, 4, 6, 12]
    want = []
    for m in m_list:
        f = fwd_rate[0] + (n_s // m) * c_f * fwd_rate[1] // fwd_rate[2]
        b = bwd_rate[0] + (n_s // m) * c_b * bwd_rate[1] // bwd_rate[2]
        want.append((m + p - 1) * (f + b))
    t, peak, best = Q.search_unit_count(lengths, m_list, solver, p, fwd_rate, bwd_rate, act_bytes=3)
    assert t == want and best == want.index(min(want))
    # activations of min(m, p) units of 12/m samples are held on the first stage at most
    assert peak == [3 * g * (n_s // m) * min(m, p) for m in m_list]
    t2, peak2, best2 = S.search_unit_count(lengths, m_list, solver, p, fwd_rate, bwd_rate, act_bytes=3)
    assert t2.tolist() == want and peak2.tolist() == peak and best2 == best


def test_single_stage_iteration_is_the_sum_of_its_tasks_and_the_memory_limit_decides():
    r = np.random.default_rng(5)
    lengths = [int(x) for x in r.integers(1, 60, 6)]
    solver = dict(WEIGHTS, granule=4)
    m_list = [1, 2, 4, 7]
    F, B = 11, 23
    t, peak, best = Q.search_unit_count(lengths, m_list, solver, 1, (F, 1, 1), (B, 1, 1), kv_bytes=2, grad_bytes=1)
    W_f = sum(2 * L * (L + 1) // 2 for L in lengths)
    W_b = sum(5 * L * (L + 1) // 2 for L in lengths)
    for m, ti in zip(m_list, t):
        part = V.solve_partition(lengths, m_fwd=m, m_bwd=m, **solver)
        nf, nb = len(part["fwd"][0]) - 1, len(part["bwd"][0]) - 1
        assert ti == W_f + W_b + F * nf + B * nb                          # costs are additive: only the fixed parts depend on m
    assert best == 0                                                      # one stage: fewer launches is all that matters
    # a limit below the single unit's peak rules it out, and the best moves on
    assert peak[0] == max(peak)
    cap = max(x for x in peak if x < peak[0])
    t3, peak3, best3 = Q.search_unit_count(lengths, m_list, solver, 1, (F, 1, 1), (B, 1, 1), kv_bytes=2, grad_bytes=1, stage_bytes_cap=cap)
    assert (t3, peak3) == (t, peak) and best3 > 0 and peak[best3] <= cap
    n3 = S.search_unit_count(lengths, m_list, solver, 1, (F, 1, 1), (B, 1, 1), kv_bytes=2, grad_bytes=1, stage_bytes_cap=cap)
    assert (n3[0].tolist(), n3[1].tolist(), n3[2]) == (t, peak, best3)
    assert Q.search_unit_count(lengths, m_list, solver, 1, (F, 1, 1), (B, 1, 1), kv_bytes=2, stage_bytes_cap=1)[2] == -1


def test_native_search_equals_the_oracle():
    r = np.random.default_rng(17)
    for case in range(12):
        lengths = [int(x) for x in r.integers(1, 50, int(r.integers(1, 6)))]
        g = int(r.integers(3, 9))
        solver = dict(w_quad_fwd=int(r.integers(1, 4)), w_lin_fwd=int(r.integers(0, 30)), w_quad_bwd=int(r.integers(2, 7)),
                      w_lin_bwd=int(r.integers(0, 50)), granule=g, max_slice=int(r.choice([0, 2 * g])),
                      token_cap_fwd=int(r.choice([0, 3 * g, 40])), token_cap_bwd=int(r.choice([0, 4 * g])))
        m_list = [1, 2, 3, 5, 8]
        p = int(r.integers(1, 4))
        fr, br = (int(r.integers(0, 40)), int(r.integers(1, 9)), int(r.integers(1, 5))), (int(r.integers(0, 60)), int(r.integers(1, 9)), int(r.integers(1, 5)))
        mem = [int(x) for x in r.integers(0, 6, 3)]
        t, peak, best = Q.search_unit_count(lengths, m_list, solver, p, fr, br, *mem)
        nt, npk, nbest = S.search_unit_count(lengths, m_list, solver, p, fr, br, *mem, n_threads=int(r.integers(1, 5)))
        assert (nt.tolist(), npk.tolist(), nbest) == (t, peak, best), f"case {case}"
        feasible = [x for x in peak if x >= 0]
        if feasible:
            cap = sorted(feasible)[len(feasible) // 2]
            assert S.search_unit_count(lengths, m_list, solver, p, fr, br, *mem, stage_bytes_cap=cap)[2] == \
                Q.search_unit_count(lengths, m_list, solver, p, fr, br, *mem, stage_bytes_cap=cap)[2]
    with pytest.raises(S.SlimAttnError):
        S.search_unit_count([4, 4], [0], dict(WEIGHTS), 1, (0, 1, 1), (0, 1, 1))
    with pytest.raises(S.SlimAttnError):
        S.search_unit_count([4, 4], [1], dict(WEIGHTS), 0, (0, 1, 1), (0, 1, 1))
