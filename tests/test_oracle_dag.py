"""Pins for the DAG oracle (oracle/dag.py) and the native simulator against it: the defining recurrences
checked directly, longest paths by exhaustive enumeration, the closed form of a uniform 1F1B pipeline, the
structure of the paper's worked figure, and bit-exact agreement of the C++ routines."""
import itertools

import numpy as np
import pytest

import paper_2509_26246_amd as S
from oracle import dag as D
from oracle import tables as T


def _check_recurrences(weights, edges, start, finish, total):
    # the paper's two equations, for every vertex, and T_total
    pred = {}
    for u, v in edges:
        pred.setdefault(v, []).append(u)
    for v in range(len(weights)):
        assert start[v] == max([0] + [finish[u] for u in pred.get(v, [])])
        assert finish[v] == start[v] + weights[v]
    assert total == (max(finish) if len(weights) else 0)


def _longest_path_exhaustive(weights, edges):
    succ = {}
    for u, v in edges:
        succ.setdefault(u, []).append(v)
    best = 0

    def walk(v, acc):
        nonlocal best
        acc += weights[v]
        best = max(best, acc)
        for x in succ.get(v, []):
            walk(x, acc)
    for v in range(len(weights)):
        walk(v, 0)
    return best


def test_timeline_satisfies_the_defining_equations_and_is_the_longest_path():
    r = np.random.default_rng(2)
    for _ in range(40):
        n = int(r.integers(1, 9))
        perm = r.permutation(n)                        # a hidden order makes the random graph acyclic
        edges = [(int(perm[a]), int(perm[b])) for a, b in itertools.combinations(range(n), 2) if r.random() < 0.4]
        weights = [int(x) for x in r.integers(0, 20, n)]
        start, finish, total = D.timeline(weights, edges)
        _check_recurrences(weights, edges, start, finish, total)
        assert total == _longest_path_exhaustive(weights, edges)          # critical path
        s2, f2, t2 = S.dag_timeline(weights, [e[0] for e in edges], [e[1] for e in edges])
        assert s2.tolist() == start and f2.tolist() == finish and t2 == total
    assert D.timeline([], []) == ([], [], 0)
    with pytest.raises(ValueError):
        D.timeline([1, 1], [(0, 1), (1, 0)])
    with pytest.raises(S.SlimAttnError) as e:
        S.dag_timeline([1, 1, 1], [0, 1, 2], [1, 2, 1])
    assert e.value.code == -2


def _whole_sample_tables(m):
    cu, sl = T.build_slices([8] * m, 8)                # m samples, one slice each, one unit per sample
    units = T.build_units(cu, sl, "PER_SAMPLE")
    return sl, units


@pytest.mark.parametrize("p,m,f,b", [(1, 1, 3, 5), (1, 6, 2, 7), (2, 2, 1, 2), (4, 4, 3, 6), (4, 9, 2, 5), (8, 16, 10, 25), (3, 2, 4, 4)])
def test_uniform_1f1b_has_the_textbook_makespan(p, m, f, b):
    # m equal micro-batches through p equal stages under 1F1B: (m + p - 1)(f + b)
    sl, units = _whole_sample_tables(m)
    vertices, weights, edges = D.build_1f1b(sl, units, units, p, [f] * m, [b] * m)
    assert len(vertices) == 2 * p * m
    start, finish, total = D.timeline(weights, [(u, v) for u, v, _ in edges])
    assert total == (m + p - 1) * (f + b)
    # no stage runs two tasks at once, and each stage is busy m (f + b)
    for s in range(p):
        spans = sorted((start[i], finish[i]) for i, (st, _, _) in enumerate(vertices) if st == s)
        assert all(a[1] <= c[0] for a, c in zip(spans, spans[1:]))
        assert sum(y - x for x, y in spans) == m * (f + b)


def test_structure_of_the_papers_worked_figure():
    """Two stages, two micro-batches, the first cut into two slices (the paper's figure of the dependency graph): 12
    vertices; 9 inter-stage, 4 inter-slice and 10 schedule edges; the backward of the first slice waits for the
    backward of the second one."""
    cu, sl = T.build_slices([16, 8], 8)                 # sample 0 -> slices 0, 1; sample 1 -> slice 2
    fwd = T.build_units(cu, sl, "TOKEN_CAP", cap=8, backward=False)     # [0] [1] [2]
    bwd = T.build_units(cu, sl, "TOKEN_CAP", cap=8, backward=True)      # [1] [0] [2]
    assert [fwd[1][fwd[0][u]:fwd[0][u + 1]].tolist() for u in range(3)] == [[0], [1], [2]]
    assert [bwd[1][bwd[0][u]:bwd[0][u + 1]].tolist() for u in range(3)] == [[1], [0], [2]]
    vertices, weights, edges = D.build_1f1b(sl, fwd, bwd, 2, [1, 1, 1], [2, 2, 2])
    assert len(vertices) == 12
    kinds = [k for _, _, k in edges]
    assert (kinds.count(D.EDGE_STAGE), kinds.count(D.EDGE_SLICE), kinds.count(D.EDGE_SCHEDULE)) == (9, 4, 10)
    name = {i: v for i, v in enumerate(vertices)}
    slice_edges = sorted((name[u], name[v]) for u, v, k in edges if k == D.EDGE_SLICE)
    assert slice_edges == [((0, D.FWD, 0), (0, D.FWD, 1)), ((0, D.BWD, 0), (0, D.BWD, 1)),
                           ((1, D.FWD, 0), (1, D.FWD, 1)), ((1, D.BWD, 0), (1, D.BWD, 1))]
    # the last stage alternates from the start, but its first backward unit (the second slice) needs both slices'
    # forward first: F F B F B B
    order1 = [name[u] for u, v, k in edges if k == D.EDGE_SCHEDULE and name[u][0] == 1] + [(1, D.BWD, 2)]
    assert order1 == [(1, D.FWD, 0), (1, D.FWD, 1), (1, D.BWD, 0), (1, D.FWD, 2), (1, D.BWD, 1), (1, D.BWD, 2)]
    start, finish, total = D.timeline(weights, [(u, v) for u, v, _ in edges])
    _check_recurrences(weights, [(u, v) for u, v, _ in edges], start, finish, total)


def test_native_graph_builder_bit_exact_and_asymmetric_lists_resolve():
    r = np.random.default_rng(8)
    for _ in range(30):
        lengths = r.integers(1, 90, size=r.integers(1, 7)).tolist()
        cu, sl = T.build_slices(lengths, int(r.integers(4, 40)))
        fwd = T.build_units(cu, sl, "PREFIX_FILL", m=int(r.integers(1, 7)), w_quad=2, w_lin=0, backward=False)
        bwd = T.build_units(cu, sl, "PREFIX_FILL", m=int(r.integers(1, 9)), w_quad=5, w_lin=0, backward=True)
        nf, nb = len(fwd[0]) - 1, len(bwd[0]) - 1
        fc = [int(x) for x in r.integers(1, 50, nf)]
        bc = [int(x) for x in r.integers(1, 120, nb)]
        for p in (1, 2, 4):
            vertices, weights, edges = D.build_1f1b(sl, fwd, bwd, p, fc, bc)
            g = S.dag_build_1f1b(sl, fwd, bwd, p, fc, bc)
            assert g["vertex"].tolist() == [list(v) for v in vertices] and g["weight"].tolist() == weights
            assert list(zip(g["edge_from"].tolist(), g["edge_to"].tolist(), g["edge_kind"].tolist())) == edges
            start, finish, total = D.timeline(weights, [(u, v) for u, v, _ in edges])          # acyclic: it resolves
            s2, f2, t2 = S.dag_timeline(g["weight"], g["edge_from"], g["edge_to"])
            assert s2.tolist() == start and f2.tolist() == finish and t2 == total
            assert total >= sum(fc) + sum(bc)                      # a stage cannot do better than its own work
            assert total <= p * (sum(fc) + sum(bc))                # nor worse than everything in sequence
            for s in range(p):                                     # one task at a time per stage
                spans = sorted((start[i], finish[i]) for i, v in enumerate(vertices) if v[0] == s)
                assert all(a[1] <= c[0] for a, c in zip(spans, spans[1:]))
            # a backward task never starts before the forward task of any slice it holds has finished on its stage
            fwd_of = {int(t): u for u in range(nf) for t in fwd[1][fwd[0][u]:fwd[0][u + 1]]}
            for v in range(nb):
                for t in bwd[1][bwd[0][v]:bwd[0][v + 1]]:
                    for s in range(p):
                        assert start[p * nf + s * nb + v] >= finish[s * nf + fwd_of[int(t)]]


# ---- memory footprint ---------------------------------------------------------------------------------------

def _csr(units):
    ptr = np.cumsum([0] + [len(u) for u in units]).astype(np.int32)
    return ptr, np.array([t for u in units for t in u], np.int32)


def test_memory_footprint_of_the_hand_worked_schedule():
    import json
    import os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "dag_memory_tiny.json")))
    cu, sl = T.build_slices(g["lengths"], g["slice_size"])
    fwd, bwd = _csr(g["fwd_units"]), _csr(g["bwd_units"])
    p = g["n_stages"]
    vertices, weights, edges = D.build_1f1b(sl, fwd, bwd, p, g["fwd_cost"], g["bwd_cost"])
    start, finish, total = D.timeline(weights, [(u, v) for u, v, _ in edges])
    assert start[:4] == g["start_fwd"] and start[4:] == g["start_bwd"] and total == g["total"]
    for c in g["cases"]:
        bufs = D.buffers_1f1b(sl, fwd, bwd, p, c["act"], c["kv"], c["grad"], c["per_slice"])
        assert D.memory_peaks(start, finish, bufs, p, [0]) == ([c["peak"]], [c["at"]])
        assert D.memory_peaks(start, finish, bufs, p, [1000]) == ([1000 + c["peak"]], [c["at"]])      # weights on top
        nb = S.dag_buffers_1f1b(sl, fwd, bwd, p, c["act"], c["kv"], c["grad"], c["per_slice"])
        assert list(zip(nb["stage"].tolist(), nb["bytes"].tolist(), nb["alloc_vertex"].tolist(), nb["free_vertex"].tolist())) == bufs
        peak, when = S.dag_memory(start, finish, nb, p)
        assert (peak.tolist(), when.tolist()) == ([c["peak"]], [c["at"]])


@pytest.mark.parametrize("p,m,f,b", [(1, 3, 2, 5), (2, 2, 1, 2), (4, 4, 3, 6), (4, 9, 2, 5), (8, 16, 10, 25), (5, 3, 4, 4)])
def test_uniform_1f1b_keeps_p_minus_s_micro_batches_of_activations(p, m, f, b):
    # the textbook property of 1F1B: stage s holds the activations of at most min(m, p - s) micro-batches, and
    # reaches that; a release and an allocation at the same instant do not add up
    sl, units = _whole_sample_tables(m)                 # 8 tokens per micro-batch
    vertices, weights, edges = D.build_1f1b(sl, units, units, p, [f] * m, [b] * m)
    start, finish, _ = D.timeline(weights, [(u, v) for u, v, _ in edges])
    bufs = D.buffers_1f1b(sl, units, units, p, 7, 0, 0, True)
    peaks, _ = D.memory_peaks(start, finish, bufs, p, [0] * p)
    assert peaks == [7 * 8 * min(m, p - s) for s in range(p)]
    peak, _ = S.dag_memory(start, finish, S.dag_buffers_1f1b(sl, units, units, p, 7, 0, 0, True), p)
    assert peak.tolist() == peaks


def test_memory_peaks_against_a_scan_of_every_instant_and_the_native_sweep():
    r = np.random.default_rng(12)
    for _ in range(40):
        n_v, n_b, p = int(r.integers(1, 10)), int(r.integers(0, 14)), int(r.integers(1, 4))
        start = [int(x) for x in r.integers(0, 12, n_v)]
        finish = [s + int(x) for s, x in zip(start, r.integers(0, 6, n_v))]
        bufs = []
        for _ in range(n_b):
            a, f = int(r.integers(n_v)), int(r.integers(n_v))
            if finish[f] < start[a]:
                a, f = f, a                              # start[f] <= finish[f] < start[a] <= finish[a]
            bufs.append((int(r.integers(p)), int(r.integers(0, 50)), a, f))
        base = [int(x) for x in r.integers(0, 9, p)]
        peaks, times = D.memory_peaks(start, finish, bufs, p, base)
        # every integer instant of the timeline, half-open lifetimes
        for s in range(p):
            live = [sum(by for st, by, a, f in bufs if st == s and start[a] <= t < finish[f]) for t in range(0, 20)]
            assert peaks[s] == base[s] + max(live) and (max(live) == 0 or live.index(max(live)) == times[s])
        d = {"stage": [b[0] for b in bufs], "bytes": [b[1] for b in bufs], "alloc_vertex": [b[2] for b in bufs], "free_vertex": [b[3] for b in bufs]}
        peak, when = S.dag_memory(start, finish, d, p, base)
        assert peak.tolist() == peaks and when.tolist() == times
    with pytest.raises(ValueError):
        D.memory_peaks([5, 0], [6, 1], [(0, 1, 0, 1)], 1, [0])
    with pytest.raises(S.SlimAttnError) as e:
        S.dag_memory([5, 0], [6, 1], {"stage": [0], "bytes": [1], "alloc_vertex": [0], "free_vertex": [1]}, 1)
    assert e.value.code == -2


def test_native_buffers_bit_exact_and_per_slice_lifetimes_never_cost_more():
    r = np.random.default_rng(21)
    for _ in range(25):
        lengths = r.integers(1, 90, size=r.integers(1, 7)).tolist()
        cu, sl = T.build_slices(lengths, int(r.integers(4, 40)))
        fwd = T.build_units(cu, sl, "PREFIX_FILL", m=int(r.integers(1, 7)), w_quad=2, w_lin=0, backward=False)
        bwd = T.build_units(cu, sl, "PREFIX_FILL", m=int(r.integers(1, 9)), w_quad=5, w_lin=0, backward=True)
        nf, nb = len(fwd[0]) - 1, len(bwd[0]) - 1
        fc, bc = [int(x) for x in r.integers(1, 50, nf)], [int(x) for x in r.integers(1, 120, nb)]
        for p in (1, 3):
            vertices, weights, edges = D.build_1f1b(sl, fwd, bwd, p, fc, bc)
            start, finish, _ = D.timeline(weights, [(u, v) for u, v, _ in edges])
            act, kv, grad = (int(x) for x in r.integers(0, 9, 3))
            peaks = {}
            for per_slice in (True, False):
                bufs = D.buffers_1f1b(sl, fwd, bwd, p, act, kv, grad, per_slice)
                nbuf = S.dag_buffers_1f1b(sl, fwd, bwd, p, act, kv, grad, per_slice)
                assert list(zip(nbuf["stage"].tolist(), nbuf["bytes"].tolist(), nbuf["alloc_vertex"].tolist(), nbuf["free_vertex"].tolist())) == bufs
                peaks[per_slice], times = D.memory_peaks(start, finish, bufs, p, [0] * p)
                got, when = S.dag_memory(start, finish, nbuf, p)
                assert got.tolist() == peaks[per_slice] and when.tolist() == times
            # a per-slice lifetime lies inside the sample-wise one, buffer by buffer
            assert all(a <= b for a, b in zip(peaks[True], peaks[False]))
