"""slimattn_bwd_static (the entry point for callers that cannot allocate: its workspace is an array built into
the library) against slimattn_bwd with a caller-allocated workspace: same kernels, same fixed summation
order, so the outputs must be bit-identical; two calls in a row, the second on a smaller pack; every launch
mode; a pack whose workspace need exceeds the array is refused before anything is launched."""
import numpy as np
import pytest
import torch

import paper_2509_26246_amd as S
import workloads as W
from paper_2509_26246_amd import harness as H

pytestmark = pytest.mark.gpu


def _problem(L, hq, hkv, d, slice_size, seed, bf16):
    r = np.random.default_rng(seed)
    T_ = sum(L)
    arrs = [r.standard_normal((T_, h, d), dtype=np.float32) * np.float32(s)
            for h, s in ((hq, 0.5), (hkv, 0.5), (hkv, 0.5), (hq, 0.1))]
    if bf16:
        arrs = [W.bf16_round(a) for a in arrs]
    cu, sl = S.build_slices(L, slice_size)
    fu = S.build_units(cu, sl, "PER_SAMPLE")
    bu = S.build_units(cu, sl, "ROUND_ROBIN", m=3, descending=True)
    return H.make_problem(*arrs, cu, sl, fu, bu, bf16=bf16, scale=d ** -0.5)


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy().copy()


def _both(prob, flags, split=False):
    """(dQ, dK, dV) bit patterns from slimattn_bwd and from slimattn_bwd_static on the same inputs."""
    kw = dict(n_q_heads=prob.n_q_heads, n_kv_heads=prob.n_kv_heads, head_dim=prob.head_dim, dtype=prob.dtype,
              scale=prob.scale, stream=torch.cuda.current_stream().cuda_stream, flags=flags)
    nb = prob.tables.n_bwd_units
    ranges = [(0, nb // 2), (nb // 2, nb)] if split else [(0, -1)]
    out = []
    for static in (False, True):
        for t in (prob.dQ, prob.dK, prob.dV):
            t.fill_(float("nan"))
        prob.workspace.fill_(0xFF)
        for lo, hi in ranges:
            if static:
                S.bwd_static(prob.q, prob.k, prob.v, prob.o, prob.lse, prob.dO, prob.tables, prob.dQ, prob.dK, prob.dV,
                             unit_lo=lo, unit_hi=hi, **kw)
            else:
                S.bwd(prob.q, prob.k, prob.v, prob.o, prob.lse, prob.dO, prob.tables, prob.dQ, prob.dK, prob.dV,
                      prob.workspace, unit_lo=lo, unit_hi=hi, **kw)
        torch.cuda.synchronize()
        out.append([_bits(t) for t in (prob.dQ, prob.dK, prob.dV)])
    return out


@pytest.mark.parametrize("bf16", [True, False])
def test_static_scratch_backward_matches_workspace_backward(bf16):
    # first a pack with a sample long enough for divided key tiles (partial tiles in the scratch), then a smaller
    # one: the second call finds the first call's leftovers in the array
    big = _problem([4500, 300, 64, 1, 129], 4, 1 if bf16 else 2, 128 if bf16 else 64, 512, 5, bf16)
    small = _problem([200, 37, 128], 4, 2, 64, 64, 6, bf16)
    for prob in (big, small):
        assert S.bwd_workspace_bytes(prob.tables, prob.n_q_heads, prob.n_kv_heads, prob.head_dim) <= S.STATIC_SCRATCH_BYTES
        prob.forward()
    torch.cuda.synchronize()
    for flags, split in ((0, False), (S.FLAG_PER_UNIT_LAUNCH, False), (0, True), (S.FLAG_STATS_PREPASS, False)):
        for name, prob in (("big", big), ("small", small)):
            ref, got = _both(prob, flags, split)
            for which, a, b in zip(("dQ", "dK", "dV"), ref, got):
                assert np.array_equal(a, b), f"{name} flags {flags} split {split}: {which} differs"
                f = a.view(np.float32) if a.dtype == np.int32 else (a.astype(np.uint16).astype(np.uint32) << 16).view(np.float32)
                assert np.isfinite(f).all()


def test_static_scratch_refuses_a_pack_that_does_not_fit():
    L = [40000]
    cu, sl = S.build_slices(L, 8192)
    fu = S.build_units(cu, sl, "ALL")
    tables = S.tables_create(cu, sl, fu[0], fu[1], fu[0], fu[1])
    hq, hkv, d = 8, 8, 128
    assert S.bwd_workspace_bytes(tables, hq, hkv, d) > S.STATIC_SCRATCH_BYTES
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda:0")       # never touched: the call is refused first
    with pytest.raises(S.SlimAttnError) as e:
        S.bwd_static(x, x, x, x, x, x, tables, x, x, x, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=S.BF16, scale=1.0)
    assert e.value.code == -6 and "scratch" in str(e.value)
