"""Device-memory plumbing around the binding: PyTorch allocates tensors and provides the stream;
every computation is a call into libslimattn."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as B


def bits_to_device(bits: np.ndarray, device="cuda:0") -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the device."""
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)


def device_to_f32(t: torch.Tensor) -> np.ndarray:
    """Device tensor (bf16 or f32) -> float32 numpy array (bf16 widened exactly)."""
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return t.cpu().numpy()


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


@dataclass
class Problem:
    """Device-resident inputs/outputs of one pack plus its tables."""
    tables: B.Tables
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    scale: float
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    dO: torch.Tensor
    o: torch.Tensor
    lse: torch.Tensor
    dQ: torch.Tensor
    dK: torch.Tensor
    dV: torch.Tensor
    workspace: torch.Tensor

    def _kw(self, **over):
        kw = dict(n_q_heads=self.n_q_heads, n_kv_heads=self.n_kv_heads, head_dim=self.head_dim, dtype=self.dtype,
                  scale=self.scale, stream=torch.cuda.current_stream().cuda_stream)
        kw.update(over)
        return kw

    def forward(self, **over):
        B.fwd(self.q, self.k, self.v, self.tables, self.o, self.lse, **self._kw(**over))

    def backward(self, **over):
        B.bwd(self.q, self.k, self.v, self.o, self.lse, self.dO, self.tables, self.dQ, self.dK, self.dV,
              self.workspace, **self._kw(**over))

    def capture_step(self, flags: int = 0) -> "torch.cuda.CUDAGraph":
        """Forward + backward of the pack recorded into a HIP graph.  The two calls only launch kernels on the
        stream they are given (no allocation, no synchronisation, no memset), so a stream capture takes them as
        they are; per-kernel timing must be off (its events are not part of a capture).  Replaying the graph
        re-runs every launch on the same buffers."""
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                      # once outside the capture: first-call set-up is not recorded
            self.forward(flags=flags)
            self.backward(flags=flags)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            self.forward(flags=flags)
            self.backward(flags=flags)
        return g


def make_problem(q: np.ndarray, k: np.ndarray, v: np.ndarray, dO: np.ndarray, cu, slices, fwd_units, bwd_units, *,
                 bf16: bool, scale: Optional[float] = None, device="cuda:0") -> Problem:
    """Uploads float32 host arrays (bf16-exact when bf16=True) and allocates outputs + workspace."""
    T, hq, d = q.shape
    hkv = k.shape[1]
    torch.cuda.set_device(device)
    tables = B.tables_create(cu, slices, fwd_units[0], fwd_units[1], bwd_units[0], bwd_units[1])
    if bf16:
        up = lambda a: bits_to_device(f32_to_bf16_bits(a), device)
        tdt = torch.bfloat16
    else:
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)
        tdt = torch.float32
    dq_, dk_, dv_, do_ = up(q), up(k), up(v), up(dO)
    ws = torch.empty(max(B.bwd_workspace_bytes(tables, hq, hkv, d), 256), dtype=torch.uint8, device=device)
    return Problem(tables, hq, hkv, d, B.BF16 if bf16 else B.F32, float(scale if scale is not None else d ** -0.5),
                   dq_, dk_, dv_, do_,
                   torch.empty((T, hq, d), dtype=tdt, device=device), torch.empty((hq, T), dtype=torch.float32, device=device),
                   torch.empty((T, hq, d), dtype=tdt, device=device), torch.empty((T, hkv, d), dtype=tdt, device=device),
                   torch.empty((T, hkv, d), dtype=tdt, device=device), ws)
