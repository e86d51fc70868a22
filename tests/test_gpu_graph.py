"""The forward and backward calls under HIP graph capture: a pipeline runtime that replays one step many times
(paper: PackFlow Pipeline Parallelism Scheduling -- one launch per scheduling unit, the launch-bound pattern) can
record the whole per-unit sequence once.  Every replay must reproduce the eager result bit for bit (the kernels
are deterministic), also after eager work and synchronisations between replays and after the inputs changed."""
import numpy as np
import pytest
import torch

import paper_2509_26246_amd as S
import workloads as W
from oracle import attention as A
from paper_2509_26246_amd import harness as H

pytestmark = pytest.mark.gpu

CASES = [
    ([700, 130, 64, 1, 300, 257], 96, 4, 2, 128, True, S.FLAG_PER_UNIT_LAUNCH),
    ([4500, 300, 64, 900], 512, 4, 1, 128, True, S.FLAG_PER_UNIT_LAUNCH),       # divided key tiles + reduction launches
    ([3000, 64, 515], 200, 6, 2, 64, True, 0),                                   # fused launches, d = 64
    ([200, 37, 128, 1, 300], 48, 4, 2, 64, False, S.FLAG_PER_UNIT_LAUNCH),       # fp32 kernels
]
OUTS = ("o", "lse", "dQ", "dK", "dV")


def _snapshot(prob):
    torch.cuda.synchronize()
    return {n: getattr(prob, n).clone() for n in OUTS}


def _poison(prob):
    for n in OUTS:
        getattr(prob, n).fill_(float("nan"))
    prob.workspace.fill_(0xFF)


def _same(a, b):
    return all(torch.equal(a[n].view(torch.uint8), b[n].view(torch.uint8)) for n in OUTS)


@pytest.mark.parametrize("L,slice_size,hq,hkv,d,bf16,flags", CASES)
def test_replays_equal_the_eager_calls(L, slice_size, hq, hkv, d, bf16, flags):
    T_ = sum(L)
    r = np.random.default_rng(T_ + d)
    arrs = [r.standard_normal((T_, h, d), dtype=np.float32) * np.float32(s) for h, s in ((hq, 0.5), (hkv, 0.5), (hkv, 0.5), (hq, 0.1))]
    q, k, v, dO = [W.bf16_round(a) if bf16 else a for a in arrs]
    scale = d ** -0.5
    cu, sl = S.build_slices(L, slice_size)
    fu = S.build_units(cu, sl, "TOKEN_CAP", cap=3 * slice_size)
    bu = S.build_units(cu, sl, "PREFIX_FILL", m=7, w_quad=5, w_lin=0, backward=True)
    prob = H.make_problem(q, k, v, dO, cu, sl, fu, bu, bf16=bf16, scale=scale)

    _poison(prob)
    prob.forward(flags=flags)
    prob.backward(flags=flags)
    eager = _snapshot(prob)
    o_ref, lse_ref = A.fwd_packed(q, k, v, cu, scale)                      # the eager result itself is right
    assert np.max(np.abs(H.device_to_f32(eager["o"]) - o_ref)) <= (2e-2 if bf16 else 1e-5)

    g = prob.capture_step(flags)
    for i in range(3):
        _poison(prob)                                                      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        assert _same(_snapshot(prob), eager), f"replay {i} differs from the eager calls"

    # the graph reads the buffers, not their contents at capture time
    prob.q.mul_(0.5)
    prob.dO.mul_(2.0)
    _poison(prob)
    prob.forward(flags=flags)
    prob.backward(flags=flags)
    eager2 = _snapshot(prob)
    assert not _same(eager2, eager)
    _poison(prob)
    torch.cuda.synchronize()
    g.replay()
    assert _same(_snapshot(prob), eager2)
