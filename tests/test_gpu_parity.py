"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the same
seeded inputs.  Tolerances (max-abs vs fp64): fp32 mode 1e-5; bf16 mode 2e-2 on O and 5e-2 on
dQ/dK/dV (inputs are bf16-exact, so the error measured is the kernels')."""
import numpy as np
import pytest
import torch

import paper_2509_26246_amd as S
import workloads as W
from oracle import attention as A
from paper_2509_26246_amd import harness as H

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_O, TOL_G = 2e-2, 5e-2


def _draw(T_, hq, hkv, d, seed, bf16, qs=1.0, dos=1.0):
    r = np.random.default_rng(seed)
    arrs = [r.standard_normal((T_, hq, d), dtype=np.float32) * np.float32(qs),
            r.standard_normal((T_, hkv, d), dtype=np.float32) * np.float32(qs),
            r.standard_normal((T_, hkv, d), dtype=np.float32) * np.float32(qs),
            r.standard_normal((T_, hq, d), dtype=np.float32) * np.float32(dos)]
    return [W.bf16_round(a) if bf16 else a for a in arrs]


def _oracle(q, k, v, dO, cu, scale):
    o, lse = A.fwd_packed(q, k, v, cu, scale)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, dO, cu, scale)
    return o, lse, dq, dk, dv


def _check(prob, ref, tol_o, tol_g, tag=""):
    o, lse, dq, dk, dv = ref
    got = {"o": H.device_to_f32(prob.o), "lse": prob.lse.cpu().numpy(), "dq": H.device_to_f32(prob.dQ),
           "dk": H.device_to_f32(prob.dK), "dv": H.device_to_f32(prob.dV)}
    want = {"o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv}
    for name in ("o", "lse", "dq", "dk", "dv"):
        err = float(np.max(np.abs(got[name].astype(np.float64) - want[name]))) if want[name].size else 0.0
        tol = tol_o if name in ("o", "lse") else tol_g
        assert err <= tol, f"{tag} {name}: max-abs {err:.3e} > {tol}"
        assert np.isfinite(got[name]).all(), f"{tag} {name} not finite"


def _poison(prob):
    for t in (prob.o, prob.dQ, prob.dK, prob.dV):
        t.fill_(float("nan"))
    prob.lse.fill_(float("nan"))
    prob.workspace.fill_(0xFF)


def _run_modes(prob, ref, tol_o, tol_g, tag):
    """Fused launch, one launch per unit, and the list split over two calls: all must match."""
    nf, nb = prob.tables.n_fwd_units, prob.tables.n_bwd_units
    _poison(prob)
    prob.forward(); prob.backward(); torch.cuda.synchronize()
    _check(prob, ref, tol_o, tol_g, tag + "/fused")
    _poison(prob)
    prob.forward(flags=S.FLAG_PER_UNIT_LAUNCH); prob.backward(flags=S.FLAG_PER_UNIT_LAUNCH); torch.cuda.synchronize()
    _check(prob, ref, tol_o, tol_g, tag + "/per-unit")
    _poison(prob)
    cf, cb = nf // 2, nb // 2
    prob.forward(unit_lo=0, unit_hi=cf); prob.forward(unit_lo=cf, unit_hi=nf)
    prob.backward(unit_lo=0, unit_hi=cb); prob.backward(unit_lo=cb, unit_hi=nb); torch.cuda.synchronize()
    _check(prob, ref, tol_o, tol_g, tag + "/split")
    # the backward's row statistics from a launch of their own (what the library chooses for very long samples)
    for flags, mode in ((S.FLAG_STATS_PREPASS, "fused"), (S.FLAG_STATS_PREPASS | S.FLAG_PER_UNIT_LAUNCH, "per-unit")):
        _poison(prob)
        prob.forward(flags=flags & S.FLAG_PER_UNIT_LAUNCH); prob.backward(flags=flags); torch.cuda.synchronize()
        _check(prob, ref, tol_o, tol_g, tag + "/stats-prepass/" + mode)


def _tables(lengths, slice_size, fwd_pol, bwd_pol):
    cu, sl = S.build_slices(lengths, slice_size)
    return cu, sl, S.build_units(cu, sl, fwd_pol[0], **fwd_pol[1]), S.build_units(cu, sl, bwd_pol[0], **bwd_pol[1])


def test_cfg0_tiny_pack_fp32():
    w = W.WORKLOADS["cfg0_tiny_f32"]
    for seed in W.SEEDS:
        rng = np.random.default_rng(seed)
        L = W.draw_lengths(w, rng)
        q, k, v, dO = W.draw_values(w, int(L.sum()), rng)
        cu, sl, fu, bu = _tables(L, w.slice_size, w.fwd_policy, w.bwd_policy)
        scale = 1.0 / np.sqrt(w.head_dim)
        ref = _oracle(q, k, v, dO, cu, scale)
        prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=False, scale=scale)
        _run_modes(prob, ref, TOL_F32, TOL_F32, f"cfg0 seed {seed}")
        # the single-unit variant gives the same result
        one = S.build_units(cu, sl, "ALL")
        prob1 = H.make_problem(q, k, v, dO, cu, sl, one, one, bf16=False, scale=scale)
        _run_modes(prob1, ref, TOL_F32, TOL_F32, f"cfg0/ALL seed {seed}")


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 16), (3, 1, 32), (2, 2, 128)])
def test_fp32_gqa_and_head_dims(hq, hkv, d):
    L = [70, 1, 129, 5, 64]
    cu, sl, fu, bu = _tables(L, 48, ("TOKEN_CAP", {"cap": 100}), ("PREFIX_FILL", {"m": 5, "w_quad": 5, "w_lin": 0, "backward": True}))
    q, k, v, dO = _draw(sum(L), hq, hkv, d, 5, False)
    scale = d ** -0.5          # the 1e-5 bound is stated for N(0,1) inputs at the usual 1/sqrt(d) scale
    ref = _oracle(q, k, v, dO, cu, scale)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=False, scale=scale)
    _run_modes(prob, ref, TOL_F32, TOL_F32, f"f32 {hq}/{hkv}/{d}")


@pytest.mark.parametrize("hq,hkv,d,slice_size", [(4, 2, 128, 64), (2, 1, 64, 64), (8, 2, 128, 192), (4, 4, 64, 1000),
                                                   (8, 1, 128, 256), (8, 1, 64, 500), (3, 1, 128, 128), (6, 2, 64, 96)])
def test_bf16_small_packs_full_oracle(hq, hkv, d, slice_size):
    L = [37, 128, 200, 511, 1, 1000, 0, 129]
    cu, sl, fu, bu = _tables(L, slice_size, ("PREFIX_FILL", {"m": 4, "w_quad": 2, "w_lin": 0}),
                             ("ROUND_ROBIN", {"m": 3, "descending": True}))
    q, k, v, dO = _draw(sum(L), hq, hkv, d, 11, True, 0.5, 0.1)
    scale = d ** -0.5
    ref = _oracle(q, k, v, dO, cu, scale)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)
    _run_modes(prob, ref, TOL_O, TOL_G, f"bf16 {hq}/{hkv}/{d}/S{slice_size}")


@pytest.mark.parametrize("seed", [103, 104, 108, 115, 124, 126])
def test_bf16_random_packs(seed):
    """Seeded random packs: length mixes with empty, one-row, sub-tile and multi-tile samples, slice sizes that are
    no multiple of any tile, group sizes 1..8 at both head dims, so that ragged query tiles, slices that start
    inside a key tile, persistent blocks with more work numbers than blocks and with fewer all occur."""
    r = np.random.default_rng(seed)
    n = int(r.integers(3, 40))
    L = [int(x) for x in np.minimum(r.pareto(1.2, n) * 60, 1500).astype(np.int64)]
    L[int(r.integers(0, n))] = 1
    hkv = int(r.choice([1, 2, 3]))
    g = int(r.choice([1, 2, 4, 8]))
    d = int(r.choice([64, 128]))
    slice_size = int(r.integers(40, 700))
    cu, sl, fu, bu = _tables(L, slice_size, ("TOKEN_CAP", {"cap": int(r.integers(200, 1500))}),
                             ("PREFIX_FILL", {"m": int(r.integers(2, 7)), "w_quad": 5, "w_lin": 0, "backward": True}))
    q, k, v, dO = _draw(sum(L), hkv * g, hkv, d, seed, True, 0.5, 0.1)
    scale = d ** -0.5
    ref = _oracle(q, k, v, dO, cu, scale)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)
    _run_modes(prob, ref, TOL_O, TOL_G, f"random pack seed {seed}: n {n} T {sum(L)} {hkv * g}/{hkv}/{d} S{slice_size}")


def test_bf16_unit_variance_inputs():
    # N(0,1) inputs (larger scores, sharper softmax) still inside the stated tolerances
    L = [300, 77]
    cu, sl, fu, bu = _tables(L, 128, ("PER_SAMPLE", {}), ("PER_SAMPLE", {"backward": True}))
    q, k, v, dO = _draw(sum(L), 4, 2, 128, 13, True, 1.0, 0.1)
    ref = _oracle(q, k, v, dO, cu, 128 ** -0.5)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True)
    _run_modes(prob, ref, TOL_O, TOL_G, "bf16 N(0,1)")


def test_bitwise_repeatable_and_grouping_invariant():
    L = [700, 130, 64]
    q, k, v, dO = _draw(sum(L), 4, 1, 128, 17, True, 0.5, 0.1)
    outs = []
    for fpol, bpol in ((("ALL", {}), ("ALL", {})),
                       (("TOKEN_CAP", {"cap": 128}), ("ROUND_ROBIN", {"m": 4, "descending": True}))):
        cu, sl, fu, bu = _tables(L, 64, fpol, bpol)
        prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True)
        runs = []
        for flags in (0, 0, S.FLAG_PER_UNIT_LAUNCH, S.FLAG_PER_UNIT_LAUNCH):
            _poison(prob)
            prob.forward(flags=flags); prob.backward(flags=flags); torch.cuda.synchronize()
            runs.append([t.view(torch.int16).cpu().numpy().copy() for t in (prob.o, prob.dQ, prob.dK, prob.dV)])
        for mode, (a, b) in (("fused", (runs[0], runs[1])), ("per-unit", (runs[2], runs[3]))):   # same mode twice
            for name, x, y in zip(("o", "dQ", "dK", "dV"), a, b):
                diff = np.argwhere(x != y)
                assert diff.size == 0, f"{fpol[0]}/{mode}: {name} differs between two identical runs at {diff[:4].tolist()} ({len(diff)} elements)"
        outs.append([H.device_to_f32(t) for t in (prob.o, prob.dQ, prob.dK, prob.dV)])
        # O and dQ do not depend on the grouping at all (each row is computed by one block, same order)
        assert np.array_equal(runs[0][0], runs[2][0]) and np.array_equal(runs[0][1], runs[2][1])
    for x, y in zip(outs[0], outs[1]):                                  # across groupings: to tolerance
        assert float(np.max(np.abs(x - y))) <= TOL_G


@pytest.mark.parametrize("hq,hkv,d", [(4, 1, 64), (4, 2, 128)])
def test_bf16_divided_key_tiles(hq, hkv, d):
    # One sample long enough that the dK/dV work of its first key tiles is divided among several
    # blocks (partial fp32 tiles + a reduction in fixed order), in the whole-list scope and, with two
    # backward units of interleaved slices, inside the per-unit scopes, where the cuts fall inside
    # runs of query rows.  Same oracle, same tolerances, and bitwise repeatable.
    L = [4500, 300, 64]
    cu, sl, fu, bu = _tables(L, 512, ("PER_SAMPLE", {}), ("ROUND_ROBIN", {"m": 2, "descending": True}))
    q, k, v, dO = _draw(sum(L), hq, hkv, d, 23, True, 0.5, 0.1)
    scale = d ** -0.5
    ref = _oracle(q, k, v, dO, cu, scale)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)
    cls = {1: 0, 2: 1}[hkv]
    assert prob.tables.count(5 + cls) > 0, "no key tile was divided: the case does not cover the reduction path"
    _run_modes(prob, ref, TOL_O, TOL_G, f"divided {hq}/{hkv}/{d}")
    runs = []
    for flags in (0, 0, S.FLAG_PER_UNIT_LAUNCH, S.FLAG_PER_UNIT_LAUNCH):
        _poison(prob)
        prob.forward(flags=flags); prob.backward(flags=flags); torch.cuda.synchronize()
        runs.append([t.view(torch.int16).cpu().numpy().copy() for t in (prob.dK, prob.dV)])
    for a, b in ((runs[0], runs[1]), (runs[2], runs[3])):
        for x, y in zip(a, b):
            assert np.array_equal(x, y), "dK/dV differ between two identical runs"


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 128), (2, 1, 64), (3, 1, 128)])
@pytest.mark.parametrize("jump", [6.0, 40.0, 200.0])
def test_bf16_forward_reference_moves(hq, hkv, d, jump):
    """Scores that climb far above a row's score against the sample's first key (by `jump` in natural
    units at one key position, beyond fp32's exponent range for the largest): kernels that take the
    exponentials against a running reference have to move it, whichever way they choose it.  One
    feature carries the climb, so the bf16 rounding of the scaled queries is a common factor."""
    L = [300, 64, 1, 190]
    T_ = sum(L)
    q, k, v, dO = _draw(T_, hq, hkv, d, 17, True, qs=0.5, dos=0.1)
    scale = d ** -0.5
    a = np.float32(4.0)
    b = np.float32(jump / (2 * 4.0 * scale))            # q0 * k0 * scale = +-jump / 2
    q[:, :, 0] = a
    st = 0
    for l in L:
        k[st:st + l, :, 0] = -b                         # the first keys of a sample score low ...
        k[st + min(l - 1, 70):st + l, :, 0] = b         # ... later ones high
        st += l
    q, k = W.bf16_round(q), W.bf16_round(k)
    cu, sl, fu, bu = _tables(L, 128, ("ALL", {}), ("ALL", {}))
    o, lse = A.fwd_packed(q, k, v, cu, scale)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)
    _poison(prob)
    prob.forward(); torch.cuda.synchronize()
    got_o, got_lse = H.device_to_f32(prob.o), prob.lse.cpu().numpy()
    assert np.isfinite(got_o).all() and np.isfinite(got_lse).all()
    assert float(np.max(np.abs(got_o - o))) <= TOL_O
    # lse carries the score's own rounding (|score| * 2^-9 from the bf16 scaled query): relative bound
    assert float(np.max(np.abs(got_lse - lse) / (1.0 + np.abs(lse)))) <= TOL_O


# ---- the benchmark workloads at full size ------------------------------------------------------------------
# A full fp64 evaluation is out of reach there, so each case checks (i) sampled output rows the oracle computes
# one by one from the definition (O, lse, dQ rows anywhere; dK/dV rows of a whole mid-sized multi-slice sample
# and of the end of the longest sample, whose sums the oracle can afford), (ii) two conservation laws over the
# whole tensors, (iii) that the per-unit launches (fp32 accumulation across launches in list order) and the
# fused launch agree everywhere.
#
# Conservation laws and their tolerances.  Rows of P sum to 1, so per sample, KV head and column c
#     sum_j dV[j, c] = sum_{i, h in group} dO[i, h, c]                                                (V)
# and sum_j dS_ij = 0, so per sample and KV head
#     sum_{i, h in group, c} q[i, h, c] dQ[i, h, c] = sum_{j, c} k[j, c] dK[j, c]                         (K)
# The kernels round P and dS to bf16 before the gradient products and the outputs to bf16 afterwards: each
# term t of a sum then carries an independent relative error uniform in +-2^-9 (rms 2^-9 / sqrt 3), and a sum
# of such terms has rms error 2^-9 / sqrt 3 * ||t||_2.  For (V): the output terms dV[j, c] and, from the rounding
# of P, the terms P_ij dO[i, h, c], whose squares sum to at most ||dO[:, group, c]||^2 (sum_j P_ij^2 <= 1); the
# scores' own rounding (q or k times scale * log2 e, rounded to bf16, differently in the forward that made
# lse and in this kernel) adds a few per cent of that for inputs of this size.  For (K): the output terms
# q dQ and k dK, and the rounding of dS inside both kernels, which is of the size of the output rounding again
# (taken as a factor 2 on the norm).  The bounds below are kSigmas of these rms values plus an absolute 1e-4
# for the fp32 summation; a dropped tile, run or head shows up as hundreds of sigmas.  (Observed on the workloads
# below: at most 1.8 sigma for (V), 3.3 for (K).)
kSigmas = 6.0
_RMS = 2.0 ** -9 / np.sqrt(3.0)


def _sq_sum(x, axes):
    return (x.astype(np.float64) ** 2).sum(axes)


def _conservation(L, cu, q, k, dO, dq, dk, dv, hkv, g, chunk=16384, samples=None):
    """Largest error of (V) and (K) over all (or the listed) samples, in units of the rms error the roundings imply."""
    worst_v = worst_k = 0.0
    for s in (range(len(L)) if samples is None else samples):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        d = q.shape[2]
        lhs = np.zeros((hkv, d)); rhs = np.zeros((hkv, d)); n2 = np.zeros((hkv, d))
        qdq = np.zeros(hkv); kdk = np.zeros(hkv); m2 = np.zeros(hkv)
        for r0 in range(a, b, chunk):
            r1 = min(b, r0 + chunk)
            dvc, doc = dv[r0:r1].astype(np.float64), dO[r0:r1].astype(np.float64).reshape(r1 - r0, hkv, g, d)
            lhs += dvc.sum(0); rhs += doc.sum((0, 2))
            n2 += (dvc ** 2).sum(0) + (doc ** 2).sum((0, 2))
            t1 = q[r0:r1].astype(np.float64).reshape(r1 - r0, hkv, g, d) * dq[r0:r1].astype(np.float64).reshape(r1 - r0, hkv, g, d)
            t2 = k[r0:r1].astype(np.float64) * dk[r0:r1].astype(np.float64)
            qdq += t1.sum((0, 2, 3)); kdk += t2.sum((0, 2))
            m2 += (t1 ** 2).sum((0, 2, 3)) + (t2 ** 2).sum((0, 2))
        ev = np.abs(lhs - rhs) - 1e-4
        worst_v = max(worst_v, float(np.max(ev / (_RMS * np.sqrt(n2) + 1e-30))))
        ek = np.abs(qdq - kdk) - 1e-4
        worst_k = max(worst_k, float(np.max(ek / (2 * _RMS * np.sqrt(m2) + 1e-30))))
    return worst_v, worst_k


FULL_SIZE_CASES = [
    ("cfg1_llama8b_32k", ("fused", "per-unit")),
    ("cfg2_tp8_70b_128k", ("fused", "per-unit")),
    ("cfg2_tail_forced", ("fused", "per-unit")),
    ("cfg3_extreme_skew", ("fused", "per-unit")),
    ("cfg4_d64_s4096", ("fused",)),
    ("cfg4_d64_s1024", ("per-unit",)),
    ("cfg4_d128_s1024", ("fused", "per-unit")),
    ("cfg4_d128_s8192", ("fused",)),
]


@pytest.mark.parametrize("name,modes", FULL_SIZE_CASES, ids=[c[0] for c in FULL_SIZE_CASES])
def test_full_size_sampled_rows_and_identities(name, modes):
    _full_size(name, modes, 1)


@pytest.mark.parametrize("seed", [s for s in W.SEEDS if s != 1])
def test_full_size_every_pack_the_benchmark_times(seed):
    # bench.py cycles over the packs of all seeds of the 32K workload; the case above covers the first
    _full_size("cfg1_llama8b_32k", ("fused", "per-unit"), seed)


@pytest.mark.parametrize("name,seed", [("cfg1_llama8b_32k", 3), ("cfg2_tail_forced", 1)])
def test_full_size_with_the_solvers_partition(name, seed):
    # the tables bench.py's `per_unit_solver` record times: slice boundaries and both unit lists from the exact
    # partition (non-uniform slices), same unit counts as the policies, cuts on the chip-filling granule
    _full_size(name, ("fused", "per-unit"), seed, solver=True)


def _solver_tables(w, L):
    _, _, fu, bu = _tables(L, w.slice_size, w.fwd_policy, w.bwd_policy)
    granule = max(256, 256 * 128 // max(1, w.n_q_heads // 2))
    r = S.solve_partition(L, m_fwd=len(fu[0]) - 1, m_bwd=len(bu[0]) - 1, w_quad_fwd=w.fwd_policy[1].get("w_quad", 2),
                          w_lin_fwd=w.fwd_policy[1].get("w_lin", 0), w_quad_bwd=w.bwd_policy[1].get("w_quad", 5),
                          w_lin_bwd=w.bwd_policy[1].get("w_lin", 0), granule=granule, max_slice=max(w.slice_size, granule))
    assert S.validate(r["cu"], r["slices"], *r["fwd"], S.CHECK_FORWARD | S.CHECK_ORDER) == (0, "")
    assert S.validate(r["cu"], r["slices"], *r["bwd"], S.CHECK_BACKWARD | S.CHECK_ORDER) == (0, "")
    return r["cu"], r["slices"], r["fwd"], r["bwd"]


def _full_size(name, modes, seed, solver=False):
    w = W.WORKLOADS[name]
    rng = np.random.default_rng(seed)
    L = W.draw_lengths(w, rng)
    T_ = int(L.sum())
    name = (name if seed == 1 else f"{name}/seed{seed}") + ("/solver" if solver else "")
    print(f"[{name}] T {T_} samples {len(L)} longest {int(L.max())}", flush=True)
    q, k, v, dO = W.draw_values(w, T_, rng)
    cu, sl, fu, bu = _solver_tables(w, L) if solver else _tables(L, w.slice_size, w.fwd_policy, w.bwd_policy)
    scale = w.head_dim ** -0.5
    g = w.n_q_heads // w.n_kv_heads
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)

    # what the oracle computes, once: rows anywhere (among them every sample's first and last row) ...
    r = np.random.default_rng(99)
    rows = np.concatenate([r.integers(0, T_, 48), cu[:-1][:64], (cu[1:] - 1)[:64]]).astype(np.int64)
    heads = r.integers(0, w.n_q_heads, len(rows))
    ro, rl = A.fwd_rows(q, k, v, cu, scale, rows, heads)
    rdq = A.dq_rows(q, k, v, dO, cu, scale, rows, heads)
    # ... key rows over a whole multi-slice sample of moderate length (its first rows collect from every later
    # slice, i.e. from several backward units) and the last rows of the longest sample
    s_long = int(np.argmax(L))
    mid = [s for s in range(len(L)) if L[s] <= 12288]
    s_mid = max(mid, key=lambda s: L[s])
    key_sets = [(s_mid, np.unique(np.concatenate([[cu[s_mid], cu[s_mid + 1] - 1], r.integers(cu[s_mid], cu[s_mid + 1], 16)])))]
    if s_long != s_mid:
        tail = min(int(L[s_long]), 768)
        key_sets.append((s_long, np.unique(np.concatenate([[cu[s_long + 1] - tail, cu[s_long + 1] - 1],
                                                           r.integers(cu[s_long + 1] - tail, cu[s_long + 1], 16)]))))
    want = []
    for smp, keys in key_sets:
        for hk in sorted({0, w.n_kv_heads - 1}):
            want.append((smp, hk, keys) + A.dkdv_rows(q, k, v, dO, cu, scale, smp, hk, keys))
    print(f"[{name}] oracle rows done (mid sample {int(L[s_mid])} rows)", flush=True)

    results = {}
    for mode in modes:
        flags = S.FLAG_PER_UNIT_LAUNCH if mode == "per-unit" else 0
        _poison(prob)
        S.profile_enable(8 * (prob.tables.n_fwd_units + prob.tables.n_bwd_units) + 16)
        prob.forward(flags=flags); prob.backward(flags=flags); torch.cuda.synchronize()
        prof = S.profile_read()
        S.profile_enable(0)
        # the statistics prepass is what the library picks for a sample whose K and V exceed 128 MB, and only then
        long_kv = int(L.max()) * w.n_kv_heads * w.head_dim * 4 > (128 << 20)
        assert (prof["delta"][1] > 0) == long_kv, (name, mode, prof)
        assert prof["dkdv"][1] == (prob.tables.n_bwd_units if mode == "per-unit" else 1)
        o, lse = H.device_to_f32(prob.o), prob.lse.cpu().numpy()
        dq, dk, dv = H.device_to_f32(prob.dQ), H.device_to_f32(prob.dK), H.device_to_f32(prob.dV)
        for x in (o, lse, dq, dk, dv):
            assert np.isfinite(x).all()
        tag = f"{name}/{mode}"
        assert np.max(np.abs(o[rows, heads] - ro)) <= TOL_O and np.max(np.abs(lse[heads, rows] - rl)) <= TOL_O, tag
        assert np.max(np.abs(dq[rows, heads] - rdq)) <= TOL_G, tag
        for smp, hk, keys, rdk, rdv in want:
            ek, ev = np.max(np.abs(dk[keys, hk] - rdk)), np.max(np.abs(dv[keys, hk] - rdv))
            assert ek <= TOL_G and ev <= TOL_G, f"{tag}: sample {smp} kv head {hk}: dK {ek:.3e} dV {ev:.3e}"
        wv, wk = _conservation(L, cu, q, k, dO, dq, dk, dv, w.n_kv_heads, g)
        print(f"[{tag}] conservation: dV {wv:.2f} sigma, q.dQ = k.dK {wk:.2f} sigma", flush=True)
        assert wv <= kSigmas and wk <= kSigmas, f"{tag}: conservation off by {wv:.1f} / {wk:.1f} sigma"
        results[mode] = (o, lse, dq, dk, dv)
    if "per-unit" in results and "fused" in results:
        a, b = results["fused"], results["per-unit"]
        # O, lse, dQ: one block per row, same order in both modes; dK/dV: other summation order
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
        assert np.max(np.abs(a[3] - b[3])) <= TOL_G and np.max(np.abs(a[4] - b[4])) <= TOL_G


def test_pack_larger_than_2gib_per_tensor():
    """80 samples of 4096 rows with 32 query heads of 128: q, o, dO, dQ are 2.7 GB each, so rows of the later samples lie
    beyond 2^31 bytes from the tensors' start (what has to stay below 2^31 is one sample's extent).  Sampled rows and key
    rows of the last sample, of the sample that straddles the 2 GiB mark and of the first one; conservation laws there."""
    hq, hkv, d, n, Ls = 32, 8, 128, 80, 4096
    assert n * Ls * hq * d * 2 > 2 ** 31 and S.shape_supported(n * Ls, Ls, hq, hkv, d, S.BF16)
    L = [Ls] * n
    T_ = n * Ls
    r = np.random.default_rng(7)
    q, k, v, dO = [W.bf16_round(r.standard_normal((T_, h, d), dtype=np.float32) * np.float32(sc))
                   for h, sc in ((hq, 0.5), (hkv, 0.5), (hkv, 0.5), (hq, 0.1))]
    print("inputs drawn", flush=True)
    cu, sl, fu, bu = _tables(L, 2048, ("PREFIX_FILL", {"m": 16, "w_quad": 2, "w_lin": 0}),
                             ("PREFIX_FILL", {"m": 24, "w_quad": 5, "w_lin": 0, "backward": True}))
    scale = d ** -0.5
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)
    straddle = (2 ** 31) // (hq * d * 2 * Ls)                   # the sample holding the row at byte offset 2^31
    picks = [0, straddle, n - 1]
    rows = np.concatenate([[cu[s], cu[s] + 1, cu[s + 1] - 1] + r.integers(cu[s], cu[s + 1], 6).tolist() for s in picks]).astype(np.int64)
    heads = r.integers(0, hq, len(rows))
    ro, rl = A.fwd_rows(q, k, v, cu, scale, rows, heads)
    rdq = A.dq_rows(q, k, v, dO, cu, scale, rows, heads)
    want = []
    for s in picks:
        keys = np.unique(np.concatenate([[cu[s], cu[s + 1] - 1], r.integers(cu[s], cu[s + 1], 10)]))
        want.append((s, keys) + A.dkdv_rows(q, k, v, dO, cu, scale, s, hkv - 1, keys))
    print("oracle rows done", flush=True)
    results = []
    for flags in (0, S.FLAG_PER_UNIT_LAUNCH):
        _poison(prob)
        prob.forward(flags=flags); prob.backward(flags=flags); torch.cuda.synchronize()
        o, lse = H.device_to_f32(prob.o), prob.lse.cpu().numpy()
        dq, dk, dv = H.device_to_f32(prob.dQ), H.device_to_f32(prob.dK), H.device_to_f32(prob.dV)
        assert np.max(np.abs(o[rows, heads] - ro)) <= TOL_O and np.max(np.abs(lse[heads, rows] - rl)) <= TOL_O
        assert np.max(np.abs(dq[rows, heads] - rdq)) <= TOL_G
        for s, keys, rdk, rdv in want:
            assert np.max(np.abs(dk[keys, hkv - 1] - rdk)) <= TOL_G and np.max(np.abs(dv[keys, hkv - 1] - rdv)) <= TOL_G, (flags, s)
        wv, wk = _conservation(L, cu, q, k, dO, dq, dk, dv, hkv, hq // hkv, samples=picks + [1, n - 2])
        assert wv <= kSigmas and wk <= kSigmas, (flags, wv, wk)
        for x in (o, dq, dk, dv):
            assert np.isfinite(x[-Ls:]).all() and np.isfinite(x[:Ls]).all()
        results.append((prob.o.view(torch.int16).clone(), prob.dQ.view(torch.int16).clone()))
        del o, dq, dk, dv
    assert torch.equal(results[0][0], results[1][0]) and torch.equal(results[0][1], results[1][1])


def test_bf16_non_uniform_slice_bounds():
    """Slices from explicit cut points (any consecutive partition of a sample is a valid slice table): cuts that
    fall inside query tiles and key tiles, one-row slices, a sample left whole; every launch mode."""
    r = np.random.default_rng(41)
    L = [1500, 333, 64, 1, 700]
    bounds = [sorted(set(int(x) for x in r.integers(1, l, n))) if l > 1 else [] for l, n in zip(L, (7, 3, 0, 0, 2))]
    bounds[0] = sorted(set(bounds[0]) | {1, 2, 129})                 # one-row slices at the start, a cut just past a tile
    cu, sl = S.build_slices_from_bounds(L, bounds)
    assert len(sl) == sum(len(b) + 1 for b in bounds)
    fu = S.build_units(cu, sl, "PREFIX_FILL", m=5, w_quad=2, w_lin=0)
    bu = S.build_units(cu, sl, "PREFIX_FILL", m=7, w_quad=5, w_lin=0, backward=True)
    for hq, hkv, d in ((4, 2, 128), (2, 1, 64)):
        q, k, v, dO = _draw(sum(L), hq, hkv, d, 43, True, 0.5, 0.1)
        scale = d ** -0.5
        ref = _oracle(q, k, v, dO, cu, scale)
        prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True, scale=scale)
        _run_modes(prob, ref, TOL_O, TOL_G, f"bounds {hq}/{hkv}/{d}")


def test_tables_uploaded_on_the_callers_stream():
    # the tables' upload queued on a side stream, compute calls queued right behind it on the same stream
    L = [300, 77, 1, 129]
    cu, sl, fu, bu = _tables(L, 64, ("TOKEN_CAP", {"cap": 128}), ("PREFIX_FILL", {"m": 3, "w_quad": 5, "w_lin": 0, "backward": True}))
    q, k, v, dO = _draw(sum(L), 4, 2, 128, 3, True, 0.5, 0.1)
    ref = _oracle(q, k, v, dO, cu, 128 ** -0.5)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            prob.tables.destroy()
            prob.tables = S.tables_create(cu, sl, fu[0], fu[1], bu[0], bu[1], stream=side.cuda_stream)
            _poison(prob)
            prob.forward(flags=S.FLAG_PER_UNIT_LAUNCH); prob.backward(flags=S.FLAG_PER_UNIT_LAUNCH)
            prob.forward(); prob.backward()
    side.synchronize()
    _check(prob, ref, TOL_O, TOL_G, "async tables")


def test_rejects_bad_arguments():
    L = [64]
    cu, sl, fu, bu = _tables(L, 64, ("ALL", {}), ("ALL", {}))
    q, k, v, dO = _draw(64, 2, 2, 64, 1, True)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=True)
    for over in ({"head_dim": 96}, {"n_kv_heads": 3}, {"dtype": 7}, {"unit_lo": 2}, {"unit_hi": 5}):
        with pytest.raises(S.SlimAttnError) as e:
            prob.forward(**over)
        assert e.value.code == -1
    with pytest.raises(S.SlimAttnError):
        S.fwd(prob.q.data_ptr() + 2, prob.k, prob.v, prob.tables, prob.o, prob.lse, n_q_heads=2, n_kv_heads=2,
              head_dim=64, dtype=S.BF16, scale=0.125)
    with pytest.raises(S.SlimAttnError) as e:
        S.tables_create(cu, sl, fu[0], fu[1] + 5, bu[0], bu[1])          # slice index out of range
    assert e.value.code == -2
