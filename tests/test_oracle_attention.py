"""Pins for the CPU fp64 attention oracle.  None of these re-types the oracle's formulas: they
use a library routine with autograd, finite differences, closed forms and conservation laws."""
import numpy as np
import pytest
import torch

from oracle import attention as A
from oracle import tables as T


def _rand(T_, Hq, Hkv, d, seed=0, scale=1.0):
    r = np.random.default_rng(seed)
    return (r.standard_normal((T_, Hq, d)) * scale, r.standard_normal((T_, Hkv, d)) * scale,
            r.standard_normal((T_, Hkv, d)) * scale, r.standard_normal((T_, Hq, d)) * scale)


def _torch_ref(q, k, v, do, cu, scale):
    """PyTorch fp64 scaled-dot-product attention, causal, per sample, gradients by autograd."""
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tk = torch.tensor(k, dtype=torch.float64, requires_grad=True)
    tv = torch.tensor(v, dtype=torch.float64, requires_grad=True)
    g = q.shape[1] // k.shape[1]
    outs = []
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        qq = tq[a:b].transpose(0, 1)[None]                         # [1,Hq,L,d]
        kk = tk[a:b].transpose(0, 1).repeat_interleave(g, dim=0)[None]
        vv = tv[a:b].transpose(0, 1).repeat_interleave(g, dim=0)[None]
        o = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=True, scale=scale)
        outs.append(o[0].transpose(0, 1))
    o = torch.cat(outs, 0)
    (o * torch.tensor(do, dtype=torch.float64)).sum().backward()
    return o.detach().numpy(), tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("Hq,Hkv,d,lengths", [(2, 2, 16, [5, 1, 33]), (4, 2, 8, [17, 40]), (6, 1, 32, [64, 3])])
def test_library_crosscheck_sdpa_autograd(Hq, Hkv, d, lengths):
    cu = np.concatenate([[0], np.cumsum(lengths)])
    q, k, v, do = _rand(cu[-1], Hq, Hkv, d, seed=11)
    scale = 0.37                                                     # not 1/sqrt(d): catches a hard-wired scale
    o, lse = A.fwd_packed(q, k, v, cu, scale)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, scale)
    ro, rdq, rdk, rdv = _torch_ref(q, k, v, do, cu, scale)
    for mine, ref in ((o, ro), (dq, rdq), (dk, rdk), (dv, rdv)):
        assert np.max(np.abs(mine - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_finite_differences_tiny():
    lengths = [7, 12, 1]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    Hq, Hkv, d = 4, 2, 4
    q, k, v, do = _rand(cu[-1], Hq, Hkv, d, seed=3)
    scale = 0.5
    o, lse = A.fwd_packed(q, k, v, cu, scale)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, scale)

    def loss(q_, k_, v_):
        return float((A.fwd_packed(q_, k_, v_, cu, scale)[0] * do).sum())

    h = 1e-6
    r = np.random.default_rng(0)
    for arr, grad, which in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(40):
            idx = tuple(r.integers(0, n) for n in arr.shape)
            hi = [q.copy(), k.copy(), v.copy()]; lo = [q.copy(), k.copy(), v.copy()]
            hi[which][idx] += h; lo[which][idx] -= h
            fd = (loss(*hi) - loss(*lo)) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd))


def test_rows_of_p_sum_to_one_and_lse_matches():
    cu = np.array([0, 9, 30])
    q, k, v, _ = _rand(30, 2, 1, 8, seed=5)
    scale = 1 / np.sqrt(8)
    _, lse = A.fwd_packed(q, k, v, cu, scale)
    for s in range(2):
        for i in range(cu[s], cu[s + 1]):
            for h in range(2):
                scores = np.array([scale * np.dot(q[i, h], k[j, 0]) for j in range(cu[s], i + 1)])
                assert abs(np.exp(scores - lse[h, i]).sum() - 1.0) < 1e-12


def test_closed_form_zero_queries():
    # q = 0: every visible key has weight 1/(i+1); O is the running mean of v; lse = log(i+1);
    # dV_j = sum_{i>=j} dO_i/(i+1) summed over the head group; dK = 0; dQ_i = scale * sum_j dS_ij k_j.
    L, Hq, Hkv, d = 23, 4, 2, 6
    cu = np.array([0, L])
    _, k, v, do = _rand(L, Hq, Hkv, d, seed=7)
    q = np.zeros((L, Hq, d))
    o, lse = A.fwd_packed(q, k, v, cu, 0.3)
    run_mean = np.cumsum(v, axis=0) / np.arange(1, L + 1)[:, None, None]
    assert np.allclose(o, np.repeat(run_mean, 2, axis=1), atol=1e-13)
    assert np.allclose(lse, np.log(np.arange(1, L + 1))[None, :], atol=1e-13)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, 0.3)
    w = do / np.arange(1, L + 1)[:, None, None]
    suffix = np.cumsum(w[::-1], axis=0)[::-1]                       # sum_{i>=j}
    want_dv = suffix.reshape(L, Hkv, 2, d).sum(axis=2)
    assert np.allclose(dv, want_dv, atol=1e-13)
    assert np.max(np.abs(dk)) < 1e-13


def test_single_token_samples():
    # L = 1: O = v, lse = scale*q.k, dV = dO (summed over the group), dQ = dK = 0.
    n, Hq, Hkv, d = 5, 2, 1, 4
    cu = np.arange(n + 1)
    q, k, v, do = _rand(n, Hq, Hkv, d, seed=9)
    o, lse = A.fwd_packed(q, k, v, cu, 0.7)
    assert np.allclose(o, np.repeat(v, 2, axis=1))
    assert np.allclose(lse, 0.7 * np.einsum("thd,td->ht", q, k[:, 0]))
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, 0.7)
    assert np.allclose(dv[:, 0], do.sum(axis=1)) and np.max(np.abs(dq)) < 1e-14 and np.max(np.abs(dk)) < 1e-14


def test_key_shift_invariance():
    cu = np.array([0, 19])
    q, k, v, do = _rand(19, 2, 2, 8, seed=13)
    c = np.random.default_rng(1).standard_normal(8)
    o1, l1 = A.fwd_packed(q, k, v, cu, 0.4)
    o2, l2 = A.fwd_packed(q, k + c, v, cu, 0.4)
    assert np.allclose(o1, o2, atol=1e-12)
    assert np.allclose(l2 - l1, 0.4 * np.einsum("thd,d->ht", q, c), atol=1e-12)
    _, _, dv1 = A.bwd_packed(q, k, v, o1, l1, do, cu, 0.4)
    _, _, dv2 = A.bwd_packed(q, k + c, v, o2, l2, do, cu, 0.4)
    assert np.allclose(dv1, dv2, atol=1e-12)


def test_no_cross_sample_terms():
    # changing sample 1's k, v must not move sample 0's outputs or gradients, and vice versa
    cu = np.array([0, 10, 25])
    q, k, v, do = _rand(25, 2, 1, 4, seed=17)
    o1, l1 = A.fwd_packed(q, k, v, cu, 0.5)
    k2, v2 = k.copy(), v.copy(); k2[10:] += 3.0; v2[10:] -= 2.0
    o2, l2 = A.fwd_packed(q, k2, v2, cu, 0.5)
    assert np.array_equal(o1[:10], o2[:10]) and not np.allclose(o1[10:], o2[10:])
    g1 = A.bwd_packed(q, k, v, o1, l1, do, cu, 0.5)
    g2 = A.bwd_packed(q, k2, v2, o2, l2, do, cu, 0.5)
    for a, b in zip(g1, g2):
        assert np.array_equal(a[:10], b[:10])


def test_conservation_identities():
    # rows of P sum to 1  =>  sum_j dV_j = sum over group heads and queries of dO;
    # rows of dS sum to 0 and S is bilinear  =>  sum_i <q_i,dQ_i> = sum_j <k_j,dK_j> per KV head.
    lengths = [31, 8]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    q, k, v, do = _rand(cu[-1], 4, 2, 8, seed=19)
    o, lse = A.fwd_packed(q, k, v, cu, 0.35)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, 0.35)
    for s in range(2):
        a, b = cu[s], cu[s + 1]
        for hk in range(2):
            assert np.allclose(dv[a:b, hk].sum(0), do[a:b, 2 * hk:2 * hk + 2].sum((0, 1)), atol=1e-12)
            lhs = (q[a:b, 2 * hk:2 * hk + 2] * dq[a:b, 2 * hk:2 * hk + 2]).sum()
            rhs = (k[a:b, hk] * dk[a:b, hk]).sum()
            assert abs(lhs - rhs) < 1e-11


@pytest.mark.parametrize("slice_size", [1, 5, 16, 64])
def test_sliced_units_equal_unsliced(slice_size):
    lengths = [37, 64, 3, 50]
    cu, sl = T.build_slices(lengths, slice_size)
    q, k, v, do = _rand(int(cu[-1]), 4, 2, 8, seed=23)
    scale = 1 / np.sqrt(8)
    o, lse = A.fwd_packed(q, k, v, cu, scale)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, scale)
    groupings = [("ALL", {}), ("PER_SAMPLE", {}), ("ROUND_ROBIN", {"m": 3, "descending": True}),
                 ("PREFIX_FILL", {"m": 4, "w_quad": 5, "w_lin": 3, "backward": True}),
                 ("TOKEN_CAP", {"cap": 40, "backward": False})]
    for pol, p in groupings:
        up, us = T.build_units(cu, sl, pol, **p)
        o2, lse2 = A.fwd_units(q, k, v, sl, up, us, scale)
        dq2, dk2, dv2 = A.bwd_units(q, k, v, o, lse, do, sl, up, us, scale)
        for x, y in ((o, o2), (lse, lse2), (dq, dq2), (dk, dk2), (dv, dv2)):
            assert np.max(np.abs(x - y)) <= 1e-12 * max(1.0, np.max(np.abs(x)))


def test_non_uniform_slice_bounds_equal_unsliced():
    lengths = [29, 11]
    cu, sl = T.build_slices_from_bounds(lengths, [[1, 2, 20], [10]])
    q, k, v, do = _rand(int(cu[-1]), 2, 1, 4, seed=29)
    o, lse = A.fwd_packed(q, k, v, cu, 0.5)
    up, us = T.build_units(cu, sl, "ROUND_ROBIN", m=2)
    o2, lse2 = A.fwd_units(q, k, v, sl, up, us, 0.5)
    assert np.allclose(o, o2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)


def test_sampled_rows_match_full():
    lengths = [40, 70]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    q, k, v, do = _rand(cu[-1], 4, 2, 8, seed=31)
    scale = 0.3
    o, lse = A.fwd_packed(q, k, v, cu, scale)
    dq, dk, dv = A.bwd_packed(q, k, v, o, lse, do, cu, scale)
    rows = np.array([0, 39, 40, 77, 109]); heads = np.array([0, 3, 1, 2, 3])
    so, sl_ = A.fwd_rows(q, k, v, cu, scale, rows, heads)
    sdq = A.dq_rows(q, k, v, do, cu, scale, rows, heads)
    for n, (r, h) in enumerate(zip(rows, heads)):
        assert np.allclose(so[n], o[r, h], atol=1e-13) and abs(sl_[n] - lse[h, r]) < 1e-13
        assert np.allclose(sdq[n], dq[r, h], atol=1e-13)
    keys = np.array([40, 41, 90, 109])
    sdk, sdv = A.dkdv_rows(q, k, v, do, cu, scale, 1, 1, keys, block=16)
    assert np.allclose(sdk, dk[keys, 1], atol=1e-12) and np.allclose(sdv, dv[keys, 1], atol=1e-12)
    # key rows away from the sample's start: the statistics are then only computed from the first of them on
    for keys in (np.array([93, 109]), np.array([109]), np.array([77, 78, 79])):
        sdk, sdv = A.dkdv_rows(q, k, v, do, cu, scale, 1, 0, keys, block=16)
        assert np.allclose(sdk, dk[keys, 0], atol=1e-12) and np.allclose(sdv, dv[keys, 0], atol=1e-12)
