"""Causal attention over packed variable-length samples, fp64, by definition.

What the method computes (paper: PackFlow section, slice-level causal attention
with a KV cache; DAG simulator section, inter-slice dependencies): each query
row of a sample attends to the keys/values of the same sample at positions not
later than its own.  Cutting a sample into slices and grouping slices into
forward or backward units is an exact reorganisation of that sum, so the
oracle has two forms that must agree:

  * `*_packed`  : per whole sample, ignoring every table (the definition);
  * `*_units`   : walking units -> slices -> rows using only the slice table's
                  (q_start, q_len, kv_start, kv_len), accumulating dK/dV in
                  unit order (this is what exercises the tables).

Conventions fixed where the paper is silent: the diagonal is included (j <= i);
scores are scaled by `scale` before the softmax; `lse` is the natural log of
the row's sum of exponentials of the scaled scores; grouped-query attention
maps query head h to KV head h // (Hq // Hkv); dK/dV sum over the group.

Backward follows the memory-efficient formulation the paper assumes (scores
recomputed from q, k and the saved lse; Asymmetric Cost Profile paragraph):
  P = exp(S - lse), dP = dO V^T, delta = rowsum(dO * O), dS = P * (dP - delta),
  dQ = scale * dS K, dK = scale * dS^T Q, dV = P^T dO.

Layouts: q, o, dO, dQ [T, Hq, d]; k, v, dK, dV [T, Hkv, d]; lse [Hq, T].
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _rows_chunk(L: int, d: int) -> int:
    # Rows are independent in the definition; chunking only bounds the size of the score matrix.
    return max(1, min(L, (1 << 24) // max(L, 1)))


def fwd_sample(q, k, v, scale):
    """One sample, all heads.  q [L,Hq,d], k,v [L,Hkv,d] -> O [L,Hq,d], lse [Hq,L] (fp64)."""
    q = np.asarray(q, F64); k = np.asarray(k, F64); v = np.asarray(v, F64)
    L, Hq, d = q.shape
    g = Hq // k.shape[1]
    o = np.zeros((L, Hq, d), F64)
    lse = np.zeros((Hq, L), F64)
    step = _rows_chunk(L, d)
    for h in range(Hq):
        kh, vh = k[:, h // g, :], v[:, h // g, :]
        for a in range(0, L, step):
            b = min(L, a + step)
            s = scale * (q[a:b, h, :] @ kh[:b].T)                       # [b-a, b]
            allowed = np.arange(b)[None, :] <= np.arange(a, b)[:, None]  # key j <= query i
            s = np.where(allowed, s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            z = e.sum(axis=1, keepdims=True)
            lse[h, a:b] = (m + np.log(z))[:, 0]
            o[a:b, h, :] = (e / z) @ vh[:b]
    return o, lse


def bwd_sample(q, k, v, o, lse, do, scale):
    """One sample, all heads: dQ, dK, dV from q, k, v, the saved o and lse, and dO."""
    q = np.asarray(q, F64); k = np.asarray(k, F64); v = np.asarray(v, F64)
    o = np.asarray(o, F64); lse = np.asarray(lse, F64); do = np.asarray(do, F64)
    L, Hq, d = q.shape
    Hkv = k.shape[1]
    g = Hq // Hkv
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    step = _rows_chunk(L, d)
    for h in range(Hq):
        hk = h // g
        kh, vh = k[:, hk, :], v[:, hk, :]
        for a in range(0, L, step):
            b = min(L, a + step)
            s = scale * (q[a:b, h, :] @ kh[:b].T)
            allowed = np.arange(b)[None, :] <= np.arange(a, b)[:, None]
            p = np.where(allowed, np.exp(s - lse[h, a:b, None]), 0.0)
            dp = do[a:b, h, :] @ vh[:b].T
            delta = (do[a:b, h, :] * o[a:b, h, :]).sum(axis=1, keepdims=True)
            ds = p * (dp - delta)
            dq[a:b, h, :] = scale * (ds @ kh[:b])
            dk[:b, hk, :] += scale * (ds.T @ q[a:b, h, :])
            dv[:b, hk, :] += p.T @ do[a:b, h, :]
    return dq, dk, dv


def fwd_packed(q, k, v, cu, scale):
    """Definition form: every sample [cu[s], cu[s+1]) on its own; no cross-sample terms."""
    T, Hq, d = q.shape
    o = np.zeros((T, Hq, d), F64)
    lse = np.zeros((Hq, T), F64)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b > a:
            o[a:b], lse[:, a:b] = fwd_sample(q[a:b], k[a:b], v[a:b], scale)
    return o, lse


def bwd_packed(q, k, v, o, lse, do, cu, scale):
    dq = np.zeros(q.shape, F64); dk = np.zeros(k.shape, F64); dv = np.zeros(v.shape, F64)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b > a:
            dq[a:b], dk[a:b], dv[a:b] = bwd_sample(q[a:b], k[a:b], v[a:b], o[a:b], lse[:, a:b],
                                                   do[a:b], scale)
    return dq, dk, dv


def _slice_rows(rec):
    """(q_start, q_len, kv_start, kv_len) of a slice-table record (any 8-int row or mapping)."""
    if isinstance(rec, dict):
        return rec["q_start"], rec["q_len"], rec["kv_start"], rec["kv_len"]
    return int(rec[2]), int(rec[3]), int(rec[4]), int(rec[5])


def fwd_units(q, k, v, slices, unit_ptr, unit_slices, scale):
    """Table-driven form.  For every unit, for every slice in it: the slice's query rows attend
    to key rows [kv_start, kv_start + kv_len) -- the earlier slices of the sample (in full) and
    the slice itself (causally).  Row i (global index) sees keys kv_start .. i."""
    q = np.asarray(q, F64); k = np.asarray(k, F64); v = np.asarray(v, F64)
    T, Hq, d = q.shape
    g = Hq // k.shape[1]
    o = np.zeros((T, Hq, d), F64)
    lse = np.zeros((Hq, T), F64)
    for u in range(len(unit_ptr) - 1):
        for t in unit_slices[unit_ptr[u]:unit_ptr[u + 1]]:
            qs, ql, ks, kl = _slice_rows(slices[int(t)])
            n_prior = kl - ql                       # keys of earlier slices: fully visible
            for h in range(Hq):
                kh, vh = k[ks:ks + kl, h // g, :], v[ks:ks + kl, h // g, :]
                s = scale * (q[qs:qs + ql, h, :] @ kh.T)              # [ql, kl]
                allowed = np.arange(kl)[None, :] <= (n_prior + np.arange(ql))[:, None]
                s = np.where(allowed, s, -np.inf)
                m = s.max(axis=1, keepdims=True)
                e = np.exp(s - m)
                z = e.sum(axis=1, keepdims=True)
                lse[h, qs:qs + ql] = (m + np.log(z))[:, 0]
                o[qs:qs + ql, h, :] = (e / z) @ vh
    return o, lse


def bwd_units(q, k, v, o, lse, do, slices, unit_ptr, unit_slices, scale):
    """Table-driven backward.  A slice's queries add dK/dV contributions to every earlier slice
    of the sample and to itself; contributions are accumulated in unit order."""
    q = np.asarray(q, F64); k = np.asarray(k, F64); v = np.asarray(v, F64)
    o = np.asarray(o, F64); lse = np.asarray(lse, F64); do = np.asarray(do, F64)
    T, Hq, d = q.shape
    g = Hq // k.shape[1]
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for u in range(len(unit_ptr) - 1):
        for t in unit_slices[unit_ptr[u]:unit_ptr[u + 1]]:
            qs, ql, ks, kl = _slice_rows(slices[int(t)])
            n_prior = kl - ql
            for h in range(Hq):
                hk = h // g
                kh, vh = k[ks:ks + kl, hk, :], v[ks:ks + kl, hk, :]
                s = scale * (q[qs:qs + ql, h, :] @ kh.T)
                allowed = np.arange(kl)[None, :] <= (n_prior + np.arange(ql))[:, None]
                p = np.where(allowed, np.exp(s - lse[h, qs:qs + ql, None]), 0.0)
                dp = do[qs:qs + ql, h, :] @ vh.T
                delta = (do[qs:qs + ql, h, :] * o[qs:qs + ql, h, :]).sum(axis=1, keepdims=True)
                ds = p * (dp - delta)
                dq[qs:qs + ql, h, :] = scale * (ds @ kh)
                dk[ks:ks + kl, hk, :] += scale * (ds.T @ q[qs:qs + ql, h, :])
                dv[ks:ks + kl, hk, :] += p.T @ do[qs:qs + ql, h, :]
    return dq, dk, dv


# ---------------------------------------------------------------------------------------------
# Sampled forms for workloads whose full fp64 evaluation is too large: exact values of chosen
# output rows, each computed straight from the definition.
# ---------------------------------------------------------------------------------------------

def _sample_of(cu, row):
    s = int(np.searchsorted(np.asarray(cu), row, side="right") - 1)
    return s, int(cu[s])


def fwd_rows(q, k, v, cu, scale, rows, heads):
    """Exact O[row, head, :] and lse[head, row] for the listed (row, head) pairs."""
    g = q.shape[1] // k.shape[1]
    out_o, out_lse = [], []
    for r, h in zip(rows, heads):
        _, a = _sample_of(cu, r)
        kk = np.asarray(k[a:r + 1, h // g, :], F64)
        vv = np.asarray(v[a:r + 1, h // g, :], F64)
        s = scale * (kk @ np.asarray(q[r, h, :], F64))
        m = s.max()
        e = np.exp(s - m)
        z = e.sum()
        out_lse.append(m + np.log(z))
        out_o.append((e / z) @ vv)
    return np.asarray(out_o), np.asarray(out_lse)


def dq_rows(q, k, v, do, cu, scale, rows, heads):
    """Exact dQ[row, head, :] for the listed pairs; o and lse of the row are recomputed here."""
    g = q.shape[1] // k.shape[1]
    out = []
    for r, h in zip(rows, heads):
        _, a = _sample_of(cu, r)
        kk = np.asarray(k[a:r + 1, h // g, :], F64)
        vv = np.asarray(v[a:r + 1, h // g, :], F64)
        s = scale * (kk @ np.asarray(q[r, h, :], F64))
        m = s.max()
        e = np.exp(s - m)
        p = e / e.sum()
        o_row = p @ vv
        d_o = np.asarray(do[r, h, :], F64)
        dp = vv @ d_o
        ds = p * (dp - d_o @ o_row)
        out.append(scale * (ds @ kk))
    return np.asarray(out)


def dkdv_rows(q, k, v, do, cu, scale, sample, kv_head, key_rows, block=2048):
    """Exact dK[j, kv_head, :], dV[j, kv_head, :] for global key rows `key_rows` of `sample`.

    A key row j sums over the queries i >= j of its sample only, so the row statistics (lse, delta) are
    computed, from the definition, for the queries from the smallest requested key row on (each over its
    whole prefix of keys) and for every head of the group; then each requested key row takes its sum."""
    g = q.shape[1] // k.shape[1]
    a, b = int(cu[sample]), int(cu[sample + 1])
    L = b - a
    kk = np.asarray(k[a:b, kv_head, :], F64)
    vv = np.asarray(v[a:b, kv_head, :], F64)
    key_local = np.asarray(key_rows) - a
    first = int(key_local.min()) if len(key_local) else L      # queries before it are in no requested sum
    d_k = np.zeros((len(key_rows), kk.shape[1]), F64)
    d_v = np.zeros_like(d_k)
    for h in range(kv_head * g, (kv_head + 1) * g):
        qq = np.asarray(q[a:b, h, :], F64)
        dd = np.asarray(do[a:b, h, :], F64)
        lse = np.full(L, np.nan, F64)
        delta = np.full(L, np.nan, F64)
        for r0 in range(first, L, block):
            r1 = min(L, r0 + block)
            s = scale * (qq[r0:r1] @ kk[:r1].T)
            s = np.where(np.arange(r1)[None, :] <= np.arange(r0, r1)[:, None], s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            z = e.sum(axis=1, keepdims=True)
            lse[r0:r1] = (m + np.log(z))[:, 0]
            delta[r0:r1] = ((e / z) @ vv[:r1] * dd[r0:r1]).sum(axis=1)
        for n, j in enumerate(key_local):
            s = scale * (qq[j:] @ kk[j])                 # queries i >= j against key j
            p = np.exp(s - lse[j:])
            dp = dd[j:] @ vv[j]
            ds = p * (dp - delta[j:])
            d_v[n] += p @ dd[j:]
            d_k[n] += scale * (ds @ qq[j:])
    return d_k, d_v
