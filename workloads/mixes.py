"""Length mixes, value draws and per-workload policy names (data only)."""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

SEEDS = (1, 2, 3, 2509)


@dataclass(frozen=True)
class Workload:
    """One benchmark/parity configuration.

    `lengths` is a recipe tuple understood by `draw_lengths`.  `fwd_policy` and
    `bwd_policy` are (name, params) pairs naming a grouping policy; the policy
    implementations live elsewhere (one in the table oracle, one in the native
    builder) and share nothing with this file.
    """
    name: str
    dtype: str                      # "f32" or "bf16"
    total_tokens: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    slice_size: int
    lengths: Tuple
    qkv_scale: float
    do_scale: float
    fwd_policy: Tuple[str, Dict] = field(default_factory=lambda: ("PER_SAMPLE", {}))
    bwd_policy: Tuple[str, Dict] = field(default_factory=lambda: ("PER_SAMPLE", {}))


def _mean_unit_m(total_tokens: int, tokens_per_unit: int = 8192) -> int:
    return max(1, total_tokens // tokens_per_unit)


WORKLOADS: Dict[str, Workload] = {}


def _add(w: Workload) -> None:
    WORKLOADS[w.name] = w


# configs[0]: tiny fp32 pack with fixed lengths.
_add(Workload("cfg0_tiny_f32", "f32", 876, 2, 2, 64, 64, ("fixed", (37, 128, 200, 511)), 1.0, 1.0,
              ("PER_SAMPLE", {}), ("ROUND_ROBIN", {"m": 4, "descending": True})))
# configs[1]: Llama-3-8B-shaped layer, one 32K pack, lognormal lengths.
_add(Workload("cfg1_llama8b_32k", "bf16", 32768, 32, 8, 128, 4096,
              ("lognormal", 7.0, 1.2, 64, 32768), 0.5, 0.1,
              ("PREFIX_FILL", {"m": 8, "w_quad": 2, "w_lin": 0, "backward": False}),
              ("PREFIX_FILL", {"m": 20, "w_quad": 5, "w_lin": 0, "backward": True})))
# configs[2]: one GPU's share of a TP=8 70B-shaped layer, Pareto lengths.
_add(Workload("cfg2_tp8_70b_128k", "bf16", 131072, 8, 1, 128, 8192,
              ("pareto", 1.1, 256, 131072), 0.5, 0.1,
              ("TOKEN_CAP", {"cap": 16384, "backward": False}),
              ("TOKEN_CAP", {"cap": 8192, "backward": True})))
# configs[2], tail-forced variant: first sample fixed at 65536 tokens.
_add(Workload("cfg2_tail_forced", "bf16", 131072, 8, 1, 128, 8192,
              ("pareto_forced_head", 1.1, 256, 131072, 65536), 0.5, 0.1,
              ("TOKEN_CAP", {"cap": 16384, "backward": False}),
              ("TOKEN_CAP", {"cap": 8192, "backward": True})))
# configs[3]: extreme skew, one 262144-token sample plus 256 short ones.
_add(Workload("cfg3_extreme_skew", "bf16", -1, 16, 4, 128, 8192,
              ("long_plus_uniform", 262144, 256, 128, 1024), 0.5, 0.1,
              ("SEEDED_LPT", {"w_quad": 2, "w_lin": 0}),
              ("ISOLATE_FILL", {"m": 64, "w_quad": 5, "w_lin": 0, "theta_num": 1, "theta_den": 1,
                                "backward": True})))
# configs[4]: head-dim x slice-size sweep on a 64K lognormal pack.
for _d in (64, 128):
    for _s in (1024, 2048, 4096, 8192):
        _m = _mean_unit_m(65536)
        _add(Workload(f"cfg4_d{_d}_s{_s}", "bf16", 65536, 32, 8, _d, _s,
                      ("lognormal", 7.5, 1.5, 64, 65536), 0.5, 0.1,
                      ("PREFIX_FILL", {"m": _m, "w_quad": 2, "w_lin": 0, "backward": False}),
                      ("PREFIX_FILL", {"m": _m, "w_quad": 5, "w_lin": 0, "backward": True})))


def draw_lengths(w: Workload, rng: np.random.Generator) -> np.ndarray:
    """Sample lengths (int32) for workload `w`; consumes `rng` first, before any values."""
    kind = w.lengths[0]
    if kind == "fixed":
        return np.asarray(w.lengths[1], dtype=np.int32)
    if kind == "long_plus_uniform":
        _, long_len, n_short, lo, hi = w.lengths
        short = rng.integers(lo, hi + 1, n_short)
        return np.concatenate([[long_len], short]).astype(np.int32)
    budget = w.total_tokens
    out = []
    if kind == "pareto_forced_head":
        out.append(int(w.lengths[4]))
        budget -= out[0]
    while budget > 0:
        if kind == "lognormal":
            _, mu, sigma, lo, hi = w.lengths
            raw = np.floor(np.exp(mu + sigma * rng.standard_normal()))
        elif kind in ("pareto", "pareto_forced_head"):
            alpha, lo, hi = w.lengths[1], w.lengths[2], w.lengths[3]
            u = rng.random()
            raw = np.floor(lo * (1.0 - u) ** (-1.0 / alpha))
        else:
            raise ValueError(kind)
        length = int(min(max(raw, lo), hi))
        length = min(length, budget)      # last sample truncated to fit the pack
        out.append(length)
        budget -= length
    return np.asarray(out, dtype=np.int32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even; finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16, returned as float32."""
    return bf16_bits_to_f32(to_bf16_bits(x))


def draw_values(w: Workload, total_tokens: int, rng: np.random.Generator):
    """q, k, v, dO (float32, in that draw order).  In bf16 workloads every value is bf16-exact."""
    shapes = [(total_tokens, w.n_q_heads, w.head_dim), (total_tokens, w.n_kv_heads, w.head_dim),
              (total_tokens, w.n_kv_heads, w.head_dim), (total_tokens, w.n_q_heads, w.head_dim)]
    scales = [w.qkv_scale, w.qkv_scale, w.qkv_scale, w.do_scale]
    out = []
    for shp, sc in zip(shapes, scales):
        a = rng.standard_normal(shp, dtype=np.float32)
        if sc != 1.0:
            a *= np.float32(sc)
        if w.dtype == "bf16":
            a = bf16_round(a)
        out.append(a)
    return tuple(out)
