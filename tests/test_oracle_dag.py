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
