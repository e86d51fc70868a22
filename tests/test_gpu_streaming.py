"""Incremental use of the library, as a pipeline runtime that handles one scheduling unit at a time would
make it (paper: PackFlow Pipeline Parallelism Scheduling -- a slice's queries see the KV cache of the earlier
slices; DAG-based pipeline representation -- a slice's KV gradients depend on the later slices; Memory
footprint simulation -- KV cache and gradients live per slice).

Forward: K/V (and q) arrive unit by unit; everything that has not arrived yet holds NaN.  Backward: dO, o and
lse of a unit arrive with that unit; dK/dV rows are handed out as soon as the last unit that contributes to them
has run (slimattn_bwd_released_rows), and must then already hold their final values.  Every result is compared
with the CPU fp64 oracle on the complete inputs."""
import numpy as np
import pytest
import torch

import paper_2509_26246_amd as S
import workloads as W
from oracle import attention as A
from paper_2509_26246_amd import harness as H

pytestmark = pytest.mark.gpu

CASES = [
    # lengths, slice size, Hq, Hkv, d, bf16, extra flags
    ([700, 130, 64, 1, 300, 257], 96, 4, 2, 128, True, 0),
    ([700, 130, 64, 1, 300, 257], 96, 4, 2, 128, True, S.FLAG_STATS_PREPASS),
    ([4500, 300, 64, 900], 512, 4, 1, 128, True, 0),              # key tiles divided among blocks inside the units
    ([700, 130, 64, 1, 300, 257], 96, 2, 1, 64, True, 0),
    ([3000, 64, 515], 200, 6, 2, 64, True, S.FLAG_STATS_PREPASS),
    ([200, 37, 128, 1, 300], 48, 4, 2, 64, False, 0),
    ([200, 37, 128, 1, 300], 48, 3, 1, 32, False, 0),
]


def _rows_of(sl, ids):
    return np.concatenate([np.arange(sl[t][2], sl[t][2] + sl[t][3]) for t in ids]).astype(np.int64)


@pytest.mark.parametrize("L,slice_size,hq,hkv,d,bf16,flags", CASES)
def test_unit_by_unit_with_inputs_arriving_late(L, slice_size, hq, hkv, d, bf16, flags):
    T_ = sum(L)
    r = np.random.default_rng(sum(L) + hq)
    arrs = [r.standard_normal((T_, h, d), dtype=np.float32) * np.float32(s) for h, s in ((hq, 0.5), (hkv, 0.5), (hkv, 0.5), (hq, 0.1))]
    q, k, v, dO = [W.bf16_round(a) if bf16 else a for a in arrs]
    scale = d ** -0.5
    cu, sl = S.build_slices(L, slice_size)
    fu = S.build_units(cu, sl, "TOKEN_CAP", cap=3 * slice_size)
    bu = S.build_units(cu, sl, "PREFIX_FILL", m=7, w_quad=5, w_lin=0, backward=True)
    assert S.validate(cu, sl, *fu, S.CHECK_FORWARD | S.CHECK_ORDER) == (0, "")
    assert S.validate(cu, sl, *bu, S.CHECK_BACKWARD | S.CHECK_ORDER) == (0, "")
    o_ref, lse_ref = A.fwd_packed(q, k, v, cu, scale)
    dq_ref, dk_ref, dv_ref = A.bwd_packed(q, k, v, o_ref, lse_ref, dO, cu, scale)
    tol_o, tol_g = (2e-2, 5e-2) if bf16 else (1e-5, 1e-5)

    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=bf16, scale=scale)
    full = {n: getattr(prob, n).clone() for n in ("q", "k", "v", "dO")}
    nan = float("nan")
    for t in (prob.q, prob.k, prob.v, prob.dO, prob.o, prob.dQ, prob.dK, prob.dV):
        t.fill_(nan)
    prob.lse.fill_(nan)
    prob.workspace.fill_(0xFF)

    # ---- forward, one unit at a time; a unit's q, k, v rows arrive just before its call
    for u in range(len(fu[0]) - 1):
        rows = torch.from_numpy(_rows_of(sl, fu[1][fu[0][u]:fu[0][u + 1]])).cuda()
        for n in ("q", "k", "v"):
            getattr(prob, n)[rows] = full[n][rows]
        prob.forward(unit_lo=u, unit_hi=u + 1, flags=flags & S.FLAG_PER_UNIT_LAUNCH)
        torch.cuda.synchronize()
        rr = rows.cpu().numpy()
        got_o, got_lse = H.device_to_f32(prob.o)[rr], prob.lse.cpu().numpy()[:, rr]
        assert np.isfinite(got_o).all() and np.isfinite(got_lse).all(), f"forward unit {u}: not finite"
        assert np.max(np.abs(got_o - o_ref[rr])) <= tol_o and np.max(np.abs(got_lse - lse_ref[:, rr])) <= tol_o, f"forward unit {u}"
    assert np.isfinite(H.device_to_f32(prob.o)).all()          # every row was written by exactly its unit

    # ---- backward, one unit at a time; dO, o and lse of a unit arrive just before its call
    o_all, lse_all = prob.o.clone(), prob.lse.clone()
    prob.o.fill_(nan)
    prob.lse.fill_(nan)
    released = np.zeros(T_, bool)
    early = {}
    for u in range(len(bu[0]) - 1):
        rows = torch.from_numpy(_rows_of(sl, bu[1][bu[0][u]:bu[0][u + 1]])).cuda()
        prob.dO[rows] = full["dO"][rows]
        prob.o[rows] = o_all[rows]
        prob.lse[:, rows] = lse_all[:, rows]
        prob.backward(unit_lo=u, unit_hi=u + 1, flags=flags)
        torch.cuda.synchronize()
        rr = rows.cpu().numpy()
        got_dq = H.device_to_f32(prob.dQ)[rr]
        assert np.isfinite(got_dq).all() and np.max(np.abs(got_dq - dq_ref[rr])) <= tol_g, f"backward unit {u}: dQ"
        dk, dv = H.device_to_f32(prob.dK), H.device_to_f32(prob.dV)
        for a, b in S.bwd_released_rows(prob.tables, u):
            assert not released[a:b].any(), "a key row was released twice"
            released[a:b] = True
            assert np.max(np.abs(dk[a:b] - dk_ref[a:b])) <= tol_g and np.max(np.abs(dv[a:b] - dv_ref[a:b])) <= tol_g, \
                f"backward unit {u}: rows [{a}, {b}) released but not final"
            early[(a, b)] = (dk[a:b].copy(), dv[a:b].copy())
        # rows whose last contributor has not run yet have not been written
        assert np.isnan(dk[~released]).all() and np.isnan(dv[~released]).all(), f"backward unit {u}: unreleased rows written"
    assert released.all()
    dk, dv = H.device_to_f32(prob.dK), H.device_to_f32(prob.dV)
    for (a, b), (xk, xv) in early.items():                      # released rows were never touched again
        assert np.array_equal(xk, dk[a:b]) and np.array_equal(xv, dv[a:b])


def test_released_rows_follow_the_unit_lists():
    """A key row is released by the last backward unit that has query rows of the sample at or after it; worked
    out by hand for first-in last-out units over one sample of 5 slices of 100 rows and a short second sample."""
    cu, sl = S.build_slices([500, 40], 100)
    one = S.build_units(cu, sl, "ALL")
    bu = S.build_units(cu, sl, "TOKEN_CAP", cap=100, backward=True)      # sample 0: slices 4,3,2,1,0 one per unit; then sample 1
    tables = S.tables_create(cu, sl, one[0], one[1], bu[0], bu[1])
    units = [bu[1][bu[0][u]:bu[0][u + 1]].tolist() for u in range(len(bu[0]) - 1)]
    assert units == [[4], [3], [2], [1], [0], [5]]
    # unit 0 holds rows 400..499: no later unit has rows at or after key 400, so keys 400..499 are complete; unit 1
    # (rows 300..399) completes keys 300..399, and so on: with first-in last-out units a slice's gradient is released
    # by the slice's own unit.  Sample 1 (rows 500..539) is complete with its unit.
    got = [S.bwd_released_rows(tables, u).tolist() for u in range(6)]
    assert got == [[[400, 500]], [[300, 400]], [[200, 300]], [[100, 200]], [[0, 100]], [[500, 540]]]
    # the same slices in forward order (not what a pipeline would do, but a valid list): every key waits for the
    # sample's last slice
    fu = S.build_units(cu, sl, "TOKEN_CAP", cap=100, backward=False)
    tables = S.tables_create(cu, sl, one[0], one[1], fu[0], fu[1])
    got = [S.bwd_released_rows(tables, u).tolist() for u in range(6)]
    assert got == [[], [], [], [], [[0, 500]], [[500, 540]]]
