"""Table oracle: slice table, unit lists and the integer cost model.  Plain Python integers.

A *slice* is a run of consecutive query rows of one sample (paper: the solver slices sequences
into primitives by exploiting causality); a *unit* is a list of slices (the paper's MicroPack:
consecutive slices of one long sample, whole short samples, or a mix).  The forward pass and
the backward pass each get their own unit list (Asymmetric Partition subsection).

Slice record (8 x int32): sample, idx_in_sample, q_start, q_len, kv_start, kv_len, 0, 0 with
q_start a global token index, kv_start the first token of the sample and
kv_len = q_start + q_len - kv_start (all keys the slice can see).

Cost model (paper gives only the ratios: attention backward = 2.5 x forward because scores are
recomputed): in units of 2*d*Hq flops a slice costs
    forward  2*pairs + lam*q_len,      backward  5*pairs + 2*lam*q_len,
with pairs = number of visible (query, key) pairs.  Policies take the two weights explicitly.

Grouping policies are deterministic; their walk order follows the paper's conventions: samples
by descending forward cost (ties: lower index first), a sample's slices ascending in the
forward pass and descending in the backward pass (first-in, last-out).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np


def pairs_of_sample(length: int) -> int:
    return length * (length + 1) // 2


def pairs_of_slice(rec) -> int:
    q_len, kv_len = int(rec[3]), int(rec[5])
    prior = kv_len - q_len
    return q_len * prior + q_len * (q_len + 1) // 2


def flops_fwd(pairs: int, d: int, hq: int) -> int:
    """Two tile products (scores, weighted values) per visible pair."""
    return 2 * (2 * d * hq) * pairs


def flops_bwd(pairs: int, d: int, hq: int) -> int:
    """Five tile products (scores again, dP, dV, dK, dQ) per visible pair."""
    return 5 * (2 * d * hq) * pairs


def build_slices(lengths: Sequence[int], slice_size: int):
    """Fixed-size slices from each sample's start; the last slice of a sample may be short."""
    cu = [0]
    for L in lengths:
        cu.append(cu[-1] + int(L))
    rows = []
    for s, L in enumerate(lengths):
        idx = 0
        for off in range(0, int(L), slice_size):
            ql = min(slice_size, int(L) - off)
            rows.append([s, idx, cu[s] + off, ql, cu[s], off + ql, 0, 0])
            idx += 1
    return np.asarray(cu, np.int32), np.asarray(rows, np.int32).reshape(-1, 8)


def build_slices_from_bounds(lengths: Sequence[int], bounds: Sequence[Sequence[int]]):
    """Arbitrary consecutive partition: bounds[s] lists the interior cut points of sample s."""
    cu = [0]
    for L in lengths:
        cu.append(cu[-1] + int(L))
    rows = []
    for s, L in enumerate(lengths):
        if int(L) == 0:
            continue                               # an empty sample has no slices
        cuts = [0] + [int(c) for c in bounds[s]] + [int(L)]
        for idx in range(len(cuts) - 1):
            a, b = cuts[idx], cuts[idx + 1]
            rows.append([s, idx, cu[s] + a, b - a, cu[s], b, 0, 0])
    return np.asarray(cu, np.int32), np.asarray(rows, np.int32).reshape(-1, 8)


# ------------------------------------------------------------------------------------------
# Walk order
# ------------------------------------------------------------------------------------------

def _walk(cu, slices, backward: bool) -> List[int]:
    n = len(cu) - 1
    by_sample: Dict[int, List[int]] = {s: [] for s in range(n)}
    for t, rec in enumerate(slices):
        by_sample[int(rec[0])].append(t)
    order = sorted(range(n), key=lambda s: (-(int(cu[s + 1]) - int(cu[s])), s))
    out: List[int] = []
    for s in order:
        ts = sorted(by_sample[s], key=lambda t: int(slices[t][1]))
        out.extend(reversed(ts) if backward else ts)
    return out


def _csr(groups: List[List[int]]):
    groups = [g for g in groups if g]
    ptr = [0]
    flat: List[int] = []
    for g in groups:
        flat.extend(g)
        ptr.append(len(flat))
    return np.asarray(ptr, np.int32), np.asarray(flat, np.int32)


def _cost(rec, w_quad: int, w_lin: int) -> int:
    return w_quad * pairs_of_slice(rec) + w_lin * int(rec[3])


def _prefix_fill(walk: List[int], slices, m: int, w_quad: int, w_lin: int) -> List[List[int]]:
    """Midpoint rule against the per-unit target W/m: a slice whose cost interval is [C, C+c)
    goes to unit floor(m*(2C+c)/(2W)), clamped to m-1."""
    total = sum(_cost(slices[t], w_quad, w_lin) for t in walk)
    groups: List[List[int]] = [[] for _ in range(m)]
    before = 0
    for t in walk:
        c = _cost(slices[t], w_quad, w_lin)
        u = (m * (2 * before + c)) // (2 * total) if total > 0 else 0
        groups[min(m - 1, u)].append(t)
        before += c
    return groups


def build_units(cu, slices, policy: str, **p) -> Tuple[np.ndarray, np.ndarray]:
    """(unit_ptr, unit_slices) for one pass.  Empty units are dropped."""
    n_slices = len(slices)
    if policy == "ALL":
        return _csr([list(range(n_slices))])
    if policy == "PER_SAMPLE":
        groups = [[] for _ in range(len(cu) - 1)]
        for t in range(n_slices):
            groups[int(slices[t][0])].append(t)
        if p.get("backward", False):
            groups = [g[::-1] for g in groups]
        return _csr(groups)
    if policy == "ROUND_ROBIN":
        m = int(p["m"])
        groups = [[] for _ in range(m)]
        for t in range(n_slices):
            groups[t % m].append(t)
        if p.get("descending", False):          # each sample's slices descend inside a unit
            groups = [g[::-1] for g in groups]
        return _csr(groups)
    backward = bool(p.get("backward", False))
    walk = _walk(cu, slices, backward)
    if policy == "PREFIX_FILL":
        return _csr(_prefix_fill(walk, slices, int(p["m"]), int(p["w_quad"]), int(p["w_lin"])))
    if policy == "TOKEN_CAP":
        cap = int(p["cap"])
        groups: List[List[int]] = [[]]
        tokens = 0
        for t in walk:
            ql = int(slices[t][3])
            if groups[-1] and tokens + ql > cap:
                groups.append([])
                tokens = 0
            groups[-1].append(t)
            tokens += ql
        return _csr(groups)
    if policy == "SEEDED_LPT":
        wq, wl = int(p["w_quad"]), int(p["w_lin"])
        n_in_sample = np.bincount(np.asarray(slices)[:, 0], minlength=len(cu) - 1)
        groups = []
        load: List[int] = []
        rest = []
        for t in walk:
            if n_in_sample[int(slices[t][0])] > 1:
                groups.append([t])
                load.append(_cost(slices[t], wq, wl))
            else:
                rest.append(t)
        while len(groups) < int(p.get("m_min", 1)):
            groups.append([])
            load.append(0)
        for t in rest:
            u = min(range(len(groups)), key=lambda i: (load[i], i))
            groups[u].append(t)
            load[u] += _cost(slices[t], wq, wl)
        return _csr(groups)
    if policy == "ISOLATE_FILL":
        m, wq, wl = int(p["m"]), int(p["w_quad"]), int(p["w_lin"])
        num, den = int(p["theta_num"]), int(p["theta_den"])
        total = sum(_cost(slices[t], wq, wl) for t in walk)
        # isolated: c >= theta * W / m   <=>   c * m * den >= num * W
        iso = {t for t in walk if _cost(slices[t], wq, wl) * m * den >= num * total}
        rest = [t for t in walk if t not in iso]
        filled = _prefix_fill(rest, slices, max(1, m - len(iso)), wq, wl) if rest else []
        fill_of = {t: i for i, g in enumerate(filled) for t in g}
        groups, open_fill = [], None                # units stay contiguous in walk order:
        for t in walk:                              # an isolated slice closes the open unit
            if t in iso:
                groups.append([t])
                open_fill = None
            else:
                if fill_of[t] != open_fill:
                    groups.append([])
                    open_fill = fill_of[t]
                groups[-1].append(t)
        return _csr(groups)
    raise ValueError(f"unknown policy {policy}")


# ------------------------------------------------------------------------------------------
# Validation (returns a list of violated rule names; empty list = valid)
# ------------------------------------------------------------------------------------------

def check_structure(cu, slices, unit_ptr, unit_slices) -> List[str]:
    bad = []
    n = len(cu) - 1
    if int(cu[0]) != 0 or any(int(cu[i + 1]) < int(cu[i]) for i in range(n)):
        bad.append("cu")
    per = {s: [] for s in range(n)}
    for rec in slices:
        s = int(rec[0])
        if not 0 <= s < n:
            return bad + ["sample_range"]
        per[s].append(rec)
    for s in range(n):
        pos, idx = int(cu[s]), 0
        for rec in per[s]:                        # table order must be ascending within a sample
            if int(rec[1]) != idx or int(rec[2]) != pos or int(rec[3]) <= 0:
                bad.append("tiling")
                break
            if int(rec[4]) != int(cu[s]) or int(rec[5]) != pos + int(rec[3]) - int(cu[s]):
                bad.append("kv_range")
                break
            pos += int(rec[3]); idx += 1
        else:
            if pos != int(cu[s + 1]):
                bad.append("tiling")
    if int(unit_ptr[0]) != 0 or int(unit_ptr[-1]) != len(unit_slices) or \
            any(int(unit_ptr[i + 1]) < int(unit_ptr[i]) for i in range(len(unit_ptr) - 1)):
        return bad + ["unit_ptr"]
    seen = [0] * len(slices)
    for t in unit_slices:
        if not 0 <= int(t) < len(slices):
            return bad + ["slice_range"]
        seen[int(t)] += 1
    if any(c != 1 for c in seen):
        bad.append("coverage")
    return bad


def check_order(slices, unit_ptr, unit_slices, backward: bool) -> List[str]:
    """The paper's pipeline rules: forward units see a sample's slices in ascending order,
    backward units in descending order (first-in last-out), and inside a unit a sample's slices
    are adjacent."""
    bad = []
    unit_of, pos_of = {}, {}
    for u in range(len(unit_ptr) - 1):
        for pos in range(int(unit_ptr[u]), int(unit_ptr[u + 1])):
            unit_of[int(unit_slices[pos])] = u
            pos_of[int(unit_slices[pos])] = pos
    by_sample: Dict[int, List[int]] = {}
    for t, rec in enumerate(slices):
        by_sample.setdefault(int(rec[0]), []).append(t)
    for ts in by_sample.values():
        ts = sorted(ts, key=lambda t: int(slices[t][1]))
        for a, b in zip(ts, ts[1:]):
            ua, ub = unit_of[a], unit_of[b]
            if (ua < ub) if backward else (ua > ub):
                bad.append("unit_order")
            if ua == ub:
                want = -1 if backward else 1
                if pos_of[b] - pos_of[a] != want:
                    bad.append("adjacency")
    return sorted(set(bad))


def unit_costs(slices, unit_ptr, unit_slices, w_quad: int, w_lin: int) -> List[int]:
    return [sum(_cost(slices[int(t)], w_quad, w_lin)
                for t in unit_slices[int(unit_ptr[u]):int(unit_ptr[u + 1])])
            for u in range(len(unit_ptr) - 1)]
