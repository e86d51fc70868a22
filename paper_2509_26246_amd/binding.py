"""ctypes binding with the same names as the C ABI (include/slimattn.h).  Marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libslimattn.so")

F32, BF16 = 0, 1
FLAG_PER_UNIT_LAUNCH = 1
FLAG_STATS_PREPASS = 2
CHECK_FORWARD, CHECK_BACKWARD, CHECK_ORDER = 0, 1, 2
POLICY_KINDS = {"ALL": 0, "PER_SAMPLE": 1, "ROUND_ROBIN": 2, "PREFIX_FILL": 3, "TOKEN_CAP": 4, "SEEDED_LPT": 5,
                "ISOLATE_FILL": 6}
EXPORTED_SYMBOLS = [
    "slimattn_build_slices", "slimattn_build_slices_from_bounds", "slimattn_build_units", "slimattn_validate",
    "slimattn_solve_partition", "slimattn_solve_bottlenecks", "slimattn_dag_timeline", "slimattn_dag_build_1f1b", "slimattn_dag_memory", "slimattn_dag_buffers_1f1b", "slimattn_candidate_unit_counts", "slimattn_search_unit_count", "slimattn_shape_supported", "slimattn_slice_pairs", "slimattn_flops_fwd", "slimattn_flops_bwd", "slimattn_tables_create", "slimattn_tables_create_async",
    "slimattn_tables_destroy", "slimattn_tables_count", "slimattn_bwd_workspace_bytes", "slimattn_fwd",
    "slimattn_bwd", "slimattn_bwd_static", "slimattn_bwd_released_rows", "slimattn_strerror", "slimattn_last_hip_error", "slimattn_version", "slimattn_profile_enable",
    "slimattn_profile_read", "slimattn_profile_read_launches"]
KERNEL_CLASSES = ["fwd", "delta", "dq", "dkdv", "reduce", "unused", "fwd_call", "bwd_call"]


class SlimAttnError(RuntimeError):
    def __init__(self, code: int, where: str, extra: str = ""):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code}){extra}")


class _Policy(C.Structure):
    _fields_ = [("kind", C.c_int32), ("m", C.c_int32), ("w_quad", C.c_int64), ("w_lin", C.c_int64),
                ("backward", C.c_int32), ("descending", C.c_int32), ("cap", C.c_int32), ("m_min", C.c_int32),
                ("theta_num", C.c_int32), ("theta_den", C.c_int32)]


class _Solver(C.Structure):
    _fields_ = [("m_fwd", C.c_int32), ("m_bwd", C.c_int32), ("w_quad_fwd", C.c_int64), ("w_lin_fwd", C.c_int64),
                ("w_quad_bwd", C.c_int64), ("w_lin_bwd", C.c_int64), ("granule", C.c_int32), ("token_cap_fwd", C.c_int32),
                ("token_cap_bwd", C.c_int32), ("max_slice", C.c_int32)]


class _Params(C.Structure):
    _fields_ = [("total_tokens", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float), ("unit_lo", C.c_int32),
                ("unit_hi", C.c_int32), ("flags", C.c_int32)]


_lib = None


def load_library():
    """Loads libslimattn.so; raises if it has not been built.  There is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_26246_amd.build`")
    lib = C.CDLL(LIB_PATH)
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    lib.slimattn_build_slices.argtypes = [i32p, C.c_int32, C.c_int32, i32p, vp, C.c_int32, i32p]
    lib.slimattn_build_slices_from_bounds.argtypes = [i32p, C.c_int32, i32p, i32p, i32p, vp, C.c_int32, i32p]
    lib.slimattn_build_units.argtypes = [i32p, C.c_int32, vp, C.c_int32, C.POINTER(_Policy), i32p, i32p, C.c_int32, i32p]
    lib.slimattn_validate.argtypes = [i32p, C.c_int32, vp, C.c_int32, i32p, i32p, C.c_int32, C.c_int, C.POINTER(C.c_char_p)]
    i64p = C.POINTER(C.c_int64)
    lib.slimattn_solve_partition.argtypes = [i32p, C.c_int32, C.POINTER(_Solver), i32p, vp, C.c_int32, i32p, i32p, i32p, i32p,
                                             i32p, i32p, i32p, C.c_int32, i64p]
    lib.slimattn_solve_bottlenecks.argtypes = [i32p, C.c_int32, C.POINTER(_Solver), i32p, C.c_int32, C.c_int32, i64p, i64p]
    lib.slimattn_dag_timeline.argtypes = [C.c_int32, i64p, C.c_int32, i32p, i32p, i64p, i64p, i64p]
    lib.slimattn_dag_build_1f1b.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, i64p, i64p,
                                            i32p, i64p, C.c_int32, i32p, i32p, i32p, i32p, C.c_int32, i32p]
    lib.slimattn_dag_memory.argtypes = [C.c_int32, i64p, i64p, C.c_int32, i32p, i64p, i32p, i32p, C.c_int32, i64p, i64p, i64p]
    lib.slimattn_dag_buffers_1f1b.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, C.c_int64,
                                              C.c_int64, C.c_int64, C.c_int32, i32p, i64p, i32p, i32p, C.c_int32, i32p]
    lib.slimattn_candidate_unit_counts.argtypes = [C.c_int32, C.c_int32, i32p, C.c_int32, i32p]
    lib.slimattn_search_unit_count.argtypes = [i32p, C.c_int32, C.POINTER(_Solver), C.POINTER(_Search), i32p, C.c_int32, C.c_int32,
                                               i64p, i64p, i32p]
    lib.slimattn_shape_supported.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.slimattn_slice_pairs.argtypes = [vp]
    lib.slimattn_slice_pairs.restype = C.c_int64
    for f in (lib.slimattn_flops_fwd, lib.slimattn_flops_bwd):
        f.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        f.restype = C.c_int64
    lib.slimattn_tables_create.argtypes = [i32p, C.c_int32, vp, C.c_int32, i32p, i32p, C.c_int32, i32p, i32p, C.c_int32,
                                           C.POINTER(vp)]
    lib.slimattn_tables_create_async.argtypes = [i32p, C.c_int32, vp, C.c_int32, i32p, i32p, C.c_int32, i32p, i32p, C.c_int32,
                                                 vp, C.c_int, C.POINTER(vp)]
    lib.slimattn_tables_destroy.argtypes = [vp]
    lib.slimattn_tables_destroy.restype = None
    lib.slimattn_tables_count.argtypes = [vp, C.c_int]
    lib.slimattn_tables_count.restype = C.c_int64
    lib.slimattn_bwd_workspace_bytes.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32]
    lib.slimattn_bwd_workspace_bytes.restype = C.c_size_t
    lib.slimattn_fwd.argtypes = [C.POINTER(_Params), vp, vp, vp, vp, vp, vp, vp]
    lib.slimattn_bwd.argtypes = [C.POINTER(_Params)] + [vp] * 12
    lib.slimattn_bwd_static.argtypes = [C.POINTER(_Params)] + [vp] * 11
    lib.slimattn_bwd_released_rows.argtypes = [vp, C.c_int32, i32p, C.c_int32, i32p]
    lib.slimattn_strerror.argtypes = [C.c_int]
    lib.slimattn_strerror.restype = C.c_char_p
    lib.slimattn_last_hip_error.restype = C.c_int
    lib.slimattn_version.restype = C.c_int
    lib.slimattn_profile_enable.argtypes = [C.c_int32]
    lib.slimattn_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.slimattn_profile_read_launches.argtypes = [C.c_int32, i32p, i32p, i32p, C.POINTER(C.c_float), i32p,
                                                   C.POINTER(C.c_int64)]
    _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def strerror(code: int) -> str:
    return load_library().slimattn_strerror(code).decode()


def version() -> int:
    return load_library().slimattn_version()


def build_slices(lengths: Sequence[int], slice_size: int) -> Tuple[np.ndarray, np.ndarray]:
    lib = load_library()
    L = _i32(lengths)
    cu = np.zeros(len(L) + 1, np.int32)
    n = C.c_int32(0)
    rc = lib.slimattn_build_slices(_p(L), len(L), slice_size, _p(cu), None, 0, C.byref(n))
    if rc not in (0, -3):
        raise SlimAttnError(rc, "slimattn_build_slices")
    out = np.zeros((n.value, 8), np.int32)
    rc = lib.slimattn_build_slices(_p(L), len(L), slice_size, _p(cu), out.ctypes.data, n.value, C.byref(n))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_build_slices")
    return cu, out


def build_slices_from_bounds(lengths: Sequence[int], bounds: Sequence[Sequence[int]]):
    lib = load_library()
    L = _i32(lengths)
    ptr = _i32(np.concatenate([[0], np.cumsum([len(b) for b in bounds])]))
    flat = _i32([x for b in bounds for x in b] or [0])
    cu = np.zeros(len(L) + 1, np.int32)
    cap = len(L) + len(flat) + 1
    out = np.zeros((cap, 8), np.int32)
    n = C.c_int32(0)
    rc = lib.slimattn_build_slices_from_bounds(_p(L), len(L), _p(ptr), _p(flat), _p(cu), out.ctypes.data, cap, C.byref(n))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_build_slices_from_bounds")
    return cu, out[:n.value].copy()


def build_units(cu, slices, policy: str, **p) -> Tuple[np.ndarray, np.ndarray]:
    lib = load_library()
    cu, slices = _i32(cu), _i32(slices).reshape(-1, 8)
    pol = _Policy(kind=POLICY_KINDS[policy], m=int(p.get("m", 0)), w_quad=int(p.get("w_quad", 0)),
                  w_lin=int(p.get("w_lin", 0)), backward=int(bool(p.get("backward", False))),
                  descending=int(bool(p.get("descending", False))), cap=int(p.get("cap", 0)),
                  m_min=int(p.get("m_min", 1)), theta_num=int(p.get("theta_num", 1)), theta_den=int(p.get("theta_den", 1)))
    ns = len(slices)
    ptr = np.zeros(ns + 2, np.int32)
    flat = np.zeros(max(ns, 1), np.int32)
    nu = C.c_int32(0)
    rc = lib.slimattn_build_units(_p(cu), len(cu) - 1, slices.ctypes.data, ns, C.byref(pol), _p(ptr), _p(flat), ns + 1,
                                  C.byref(nu))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_build_units")
    return ptr[:nu.value + 1].copy(), flat[:ns].copy()


def _solver(m_fwd=1, m_bwd=1, w_quad_fwd=2, w_lin_fwd=0, w_quad_bwd=5, w_lin_bwd=0, granule=1, token_cap_fwd=0,
            token_cap_bwd=0, max_slice=0) -> _Solver:
    return _Solver(m_fwd=m_fwd, m_bwd=m_bwd, w_quad_fwd=w_quad_fwd, w_lin_fwd=w_lin_fwd, w_quad_bwd=w_quad_bwd,
                   w_lin_bwd=w_lin_bwd, granule=granule, token_cap_fwd=token_cap_fwd, token_cap_bwd=token_cap_bwd,
                   max_slice=max_slice)


def solve_partition(lengths: Sequence[int], **params):
    """slimattn_solve_partition -> dict(cu, slices, fwd=(unit_ptr, unit_slices), bwd=(...), bottleneck_fwd, bottleneck_bwd)."""
    lib = load_library()
    L = _i32(lengths)
    sp = _solver(**params)
    cu = np.zeros(len(L) + 1, np.int32)
    ns, nf, nb = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    bott = (C.c_int64 * 2)()
    one = np.zeros(1, np.int32)
    rc = lib.slimattn_solve_partition(_p(L), len(L), C.byref(sp), _p(cu), None, 0, C.byref(ns), _p(one), None, C.byref(nf),
                                      _p(one), None, C.byref(nb), 0, bott)
    if rc not in (0, -3):
        raise SlimAttnError(rc, "slimattn_solve_partition")
    cap_s, cap_u = max(ns.value, 1), max(nf.value, nb.value, 1)
    sl = np.zeros((cap_s, 8), np.int32)
    fp, bp = np.zeros(cap_u + 1, np.int32), np.zeros(cap_u + 1, np.int32)
    fs, bs = np.zeros(cap_s, np.int32), np.zeros(cap_s, np.int32)
    rc = lib.slimattn_solve_partition(_p(L), len(L), C.byref(sp), _p(cu), sl.ctypes.data, cap_s, C.byref(ns), _p(fp), _p(fs),
                                      C.byref(nf), _p(bp), _p(bs), C.byref(nb), cap_u, bott)
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_solve_partition")
    n = ns.value
    return {"cu": cu, "slices": sl[:n].copy(), "fwd": (fp[:nf.value + 1].copy(), fs[:n].copy()),
            "bwd": (bp[:nb.value + 1].copy(), bs[:n].copy()), "bottleneck_fwd": int(bott[0]), "bottleneck_bwd": int(bott[1])}


def solve_bottlenecks(lengths: Sequence[int], m_list: Sequence[int], n_threads: int = 4, **params):
    """slimattn_solve_bottlenecks -> (forward optima, backward optima) for the candidate unit counts."""
    lib = load_library()
    L, M = _i32(lengths), _i32(m_list)
    sp = _solver(**params)
    f, b = np.zeros(len(M), np.int64), np.zeros(len(M), np.int64)
    i64 = lambda a: a.ctypes.data_as(C.POINTER(C.c_int64))
    rc = lib.slimattn_solve_bottlenecks(_p(L), len(L), C.byref(sp), _p(M), len(M), n_threads, i64(f), i64(b))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_solve_bottlenecks")
    return f, b


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int64)


def _p64(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def dag_timeline(weight, edge_from, edge_to):
    """slimattn_dag_timeline -> (start, finish, total)."""
    lib = load_library()
    w, ef, et = _i64(weight), _i32(edge_from), _i32(edge_to)
    start, finish = np.zeros(len(w), np.int64), np.zeros(len(w), np.int64)
    total = C.c_int64(0)
    rc = lib.slimattn_dag_timeline(len(w), _p64(w), len(ef), _p(ef), _p(et), _p64(start), _p64(finish), C.byref(total))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_dag_timeline")
    return start, finish, int(total.value)


def dag_build_1f1b(slices, fwd_units, bwd_units, n_stages: int, fwd_cost, bwd_cost):
    """slimattn_dag_build_1f1b -> dict(vertex [n,3], weight [n], edge_from, edge_to, edge_kind)."""
    lib = load_library()
    sl = _i32(slices).reshape(-1, 8)
    fp, fs, bp, bs = _i32(fwd_units[0]), _i32(fwd_units[1]), _i32(bwd_units[0]), _i32(bwd_units[1])
    fc, bc = _i64(fwd_cost), _i64(bwd_cost)
    nv, ne = C.c_int32(0), C.c_int32(0)
    args = (sl.ctypes.data, len(sl), _p(fp), _p(fs), len(fp) - 1, _p(bp), _p(bs), len(bp) - 1, n_stages, _p64(fc), _p64(bc))
    rc = lib.slimattn_dag_build_1f1b(*args, None, None, 0, C.byref(nv), None, None, None, 0, C.byref(ne))
    if rc not in (0, -3):
        raise SlimAttnError(rc, "slimattn_dag_build_1f1b")
    vertex, weight = np.zeros((max(nv.value, 1), 3), np.int32), np.zeros(max(nv.value, 1), np.int64)
    ef, et, ek = (np.zeros(max(ne.value, 1), np.int32) for _ in range(3))
    rc = lib.slimattn_dag_build_1f1b(*args, _p(vertex), _p64(weight), nv.value, C.byref(nv), _p(ef), _p(et), _p(ek), ne.value,
                                     C.byref(ne))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_dag_build_1f1b")
    n, m = nv.value, ne.value
    return {"vertex": vertex[:n].copy(), "weight": weight[:n].copy(), "edge_from": ef[:m].copy(), "edge_to": et[:m].copy(),
            "edge_kind": ek[:m].copy()}


class _Search(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("pad0", C.c_int32), ("fwd_fixed", C.c_int64), ("fwd_num", C.c_int64), ("fwd_den", C.c_int64),
                ("bwd_fixed", C.c_int64), ("bwd_num", C.c_int64), ("bwd_den", C.c_int64), ("act_bytes_per_token", C.c_int64),
                ("kv_bytes_per_token", C.c_int64), ("grad_bytes_per_token", C.c_int64), ("stage_bytes_cap", C.c_int64)]


def candidate_unit_counts(n_stages: int, m_max: int) -> np.ndarray:
    """slimattn_candidate_unit_counts -> ascending candidate unit counts (multiples of n_stages up to m_max)."""
    lib = load_library()
    n = C.c_int32(0)
    rc = lib.slimattn_candidate_unit_counts(n_stages, m_max, None, 0, C.byref(n))
    if rc not in (0, -3):
        raise SlimAttnError(rc, "slimattn_candidate_unit_counts")
    out = np.zeros(max(n.value, 1), np.int32)
    rc = lib.slimattn_candidate_unit_counts(n_stages, m_max, _p(out), n.value, C.byref(n))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_candidate_unit_counts")
    return out[:n.value].copy()


def search_unit_count(lengths: Sequence[int], m_list: Sequence[int], solver: dict, n_stages: int, fwd_rate, bwd_rate, act_bytes: int = 0,
                      kv_bytes: int = 0, grad_bytes: int = 0, stage_bytes_cap: int = 0, n_threads: int = 4):
    """slimattn_search_unit_count -> (t_total [n_m], peak_bytes [n_m], best index or -1).  solver: the keyword
    parameters of solve_partition (m_fwd / m_bwd ignored); fwd_rate, bwd_rate = (fixed, num, den)."""
    lib = load_library()
    L, M = _i32(lengths), _i32(m_list)
    params = dict(solver)
    params.setdefault("m_fwd", 1)
    params.setdefault("m_bwd", 1)
    sp = _solver(**params)
    ss = _Search(n_stages, 0, *[int(x) for x in fwd_rate], *[int(x) for x in bwd_rate], act_bytes, kv_bytes, grad_bytes, stage_bytes_cap)
    t, pk = np.zeros(max(len(M), 1), np.int64), np.zeros(max(len(M), 1), np.int64)
    best = C.c_int32(-1)
    rc = lib.slimattn_search_unit_count(_p(L), len(L), C.byref(sp), C.byref(ss), _p(M), len(M), n_threads, _p64(t), _p64(pk), C.byref(best))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_search_unit_count")
    return t[:len(M)].copy(), pk[:len(M)].copy(), int(best.value)


def dag_buffers_1f1b(slices, fwd_units, bwd_units, n_stages: int, act_bytes: int, kv_bytes: int, grad_bytes: int, per_slice: bool = True):
    """slimattn_dag_buffers_1f1b -> dict(stage, bytes, alloc_vertex, free_vertex), three buffers per (stage, slice)."""
    lib = load_library()
    sl = _i32(slices).reshape(-1, 8)
    fp, fs, bp, bs = _i32(fwd_units[0]), _i32(fwd_units[1]), _i32(bwd_units[0]), _i32(bwd_units[1])
    n = 3 * n_stages * len(sl)
    stage, alloc, free = (np.zeros(max(n, 1), np.int32) for _ in range(3))
    size = np.zeros(max(n, 1), np.int64)
    nb = C.c_int32(0)
    rc = lib.slimattn_dag_buffers_1f1b(sl.ctypes.data, len(sl), _p(fp), _p(fs), len(fp) - 1, _p(bp), _p(bs), len(bp) - 1, n_stages,
                                       act_bytes, kv_bytes, grad_bytes, int(per_slice), _p(stage), _p64(size), _p(alloc), _p(free), n,
                                       C.byref(nb))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_dag_buffers_1f1b")
    n = nb.value
    return {"stage": stage[:n].copy(), "bytes": size[:n].copy(), "alloc_vertex": alloc[:n].copy(), "free_vertex": free[:n].copy()}


def dag_memory(start, finish, buffers, n_stages: int, stage_base=None):
    """slimattn_dag_memory -> (peak_bytes [n_stages], peak_time [n_stages]); `buffers` as dag_buffers_1f1b returns them."""
    lib = load_library()
    st, fi = _i64(start), _i64(finish)
    stage, alloc, free = _i32(buffers["stage"]), _i32(buffers["alloc_vertex"]), _i32(buffers["free_vertex"])
    size = _i64(buffers["bytes"])
    base = _i64(stage_base) if stage_base is not None else None
    peak, when = np.zeros(max(n_stages, 1), np.int64), np.zeros(max(n_stages, 1), np.int64)
    rc = lib.slimattn_dag_memory(len(st), _p64(st), _p64(fi), len(stage), _p(stage), _p64(size), _p(alloc), _p(free), n_stages,
                                 _p64(base) if base is not None else None, _p64(peak), _p64(when))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_dag_memory")
    return peak[:n_stages].copy(), when[:n_stages].copy()


def validate(cu, slices, unit_ptr, unit_slices, mode: int = CHECK_FORWARD) -> Tuple[int, str]:
    lib = load_library()
    cu, slices = _i32(cu), _i32(slices).reshape(-1, 8)
    up, us = _i32(unit_ptr), _i32(unit_slices)
    rule = C.c_char_p()
    rc = lib.slimattn_validate(_p(cu), len(cu) - 1, slices.ctypes.data, len(slices), _p(up), _p(us), len(up) - 1, mode,
                               C.byref(rule))
    return rc, (rule.value or b"").decode()


def shape_supported(total_tokens: int, max_sample_len: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int) -> bool:
    return load_library().slimattn_shape_supported(total_tokens, max_sample_len, n_q_heads, n_kv_heads, head_dim, dtype) == 0


def slice_pairs(rec) -> int:
    r = _i32(rec)
    return int(load_library().slimattn_slice_pairs(r.ctypes.data))


def flops_fwd(pairs: int, head_dim: int, n_q_heads: int) -> int:
    return int(load_library().slimattn_flops_fwd(pairs, head_dim, n_q_heads))


def flops_bwd(pairs: int, head_dim: int, n_q_heads: int) -> int:
    return int(load_library().slimattn_flops_bwd(pairs, head_dim, n_q_heads))


class Tables:
    """Owns a slimattn_tables handle (device copies of the tables on the current device)."""

    def __init__(self, handle: int, n_fwd_units: int, n_bwd_units: int, total_tokens: int):
        self.handle = handle
        self.n_fwd_units, self.n_bwd_units, self.total_tokens = n_fwd_units, n_bwd_units, total_tokens

    def count(self, what: int) -> int:
        return int(load_library().slimattn_tables_count(self.handle, what))

    def destroy(self):
        if self.handle:
            load_library().slimattn_tables_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tables_create(cu, slices, fwd_unit_ptr, fwd_unit_slices, bwd_unit_ptr, bwd_unit_slices, stream=False) -> Tables:
    """slimattn_tables_create, or slimattn_tables_create_async when `stream` is given (a hipStream_t address, or
    None for the default stream): the upload is then queued on that stream and the host does not wait."""
    lib = load_library()
    cu, slices = _i32(cu), _i32(slices).reshape(-1, 8)
    fp, fs, bp, bs = _i32(fwd_unit_ptr), _i32(fwd_unit_slices), _i32(bwd_unit_ptr), _i32(bwd_unit_slices)
    h = C.c_void_p()
    if stream is False:
        rc = lib.slimattn_tables_create(_p(cu), len(cu) - 1, slices.ctypes.data, len(slices), _p(fp), _p(fs), len(fp) - 1,
                                        _p(bp), _p(bs), len(bp) - 1, C.byref(h))
    else:
        rc = lib.slimattn_tables_create_async(_p(cu), len(cu) - 1, slices.ctypes.data, len(slices), _p(fp), _p(fs), len(fp) - 1,
                                              _p(bp), _p(bs), len(bp) - 1, stream, 1, C.byref(h))
    if rc != 0:
        extra = f" hip={lib.slimattn_last_hip_error()}" if rc == -4 else ""
        raise SlimAttnError(rc, "slimattn_tables_create", extra)
    return Tables(h.value, len(fp) - 1, len(bp) - 1, int(cu[-1]))


def bwd_workspace_bytes(tables: Tables, n_q_heads: int, n_kv_heads: int, head_dim: int) -> int:
    return int(load_library().slimattn_bwd_workspace_bytes(tables.handle, n_q_heads, n_kv_heads, head_dim))


def _ptr(t) -> int:
    """Device pointer of a torch tensor (must be contiguous) or a raw integer address."""
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _params(T, hq, hkv, d, dtype, scale, unit_lo, unit_hi, flags):
    return _Params(total_tokens=T, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=dtype, scale=scale,
                   unit_lo=unit_lo, unit_hi=unit_hi, flags=flags)


def fwd(q, k, v, tables: Tables, o, lse, *, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, scale: float,
        unit_lo: int = 0, unit_hi: int = -1, flags: int = 0, stream: Optional[int] = None) -> None:
    """slimattn_fwd: q,k,v -> o,lse on `stream` (a hipStream_t address; None = default stream)."""
    lib = load_library()
    prm = _params(tables.total_tokens, n_q_heads, n_kv_heads, head_dim, dtype, scale, unit_lo, unit_hi, flags)
    rc = lib.slimattn_fwd(C.byref(prm), _ptr(q), _ptr(k), _ptr(v), tables.handle, _ptr(o), _ptr(lse), stream)
    if rc != 0:
        extra = f" hip={lib.slimattn_last_hip_error()}" if rc == -4 else ""
        raise SlimAttnError(rc, "slimattn_fwd", extra)


def bwd(q, k, v, o, lse, dO, tables: Tables, dQ, dK, dV, workspace, *, n_q_heads: int, n_kv_heads: int, head_dim: int,
        dtype: int, scale: float, unit_lo: int = 0, unit_hi: int = -1, flags: int = 0,
        stream: Optional[int] = None) -> None:
    """slimattn_bwd: q,k,v,o,lse,dO -> dQ,dK,dV on `stream`."""
    lib = load_library()
    prm = _params(tables.total_tokens, n_q_heads, n_kv_heads, head_dim, dtype, scale, unit_lo, unit_hi, flags)
    rc = lib.slimattn_bwd(C.byref(prm), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), tables.handle,
                          _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), stream)
    if rc != 0:
        extra = f" hip={lib.slimattn_last_hip_error()}" if rc == -4 else ""
        raise SlimAttnError(rc, "slimattn_bwd", extra)


def bwd_released_rows(tables: Tables, unit: int) -> np.ndarray:
    """[n, 2] array of key-row ranges whose dK/dV become final with backward unit `unit`."""
    lib = load_library()
    n = C.c_int32(0)
    rc = lib.slimattn_bwd_released_rows(tables.handle, unit, None, 0, C.byref(n))
    if rc not in (0, -3):
        raise SlimAttnError(rc, "slimattn_bwd_released_rows")
    out = np.zeros((max(n.value, 1), 2), np.int32)
    rc = lib.slimattn_bwd_released_rows(tables.handle, unit, _p(out), n.value, C.byref(n))
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_bwd_released_rows")
    return out[:n.value].copy()


STATIC_SCRATCH_BYTES = 64 << 20


def bwd_static(q, k, v, o, lse, dO, tables: Tables, dQ, dK, dV, *, n_q_heads: int, n_kv_heads: int, head_dim: int,
               dtype: int, scale: float, unit_lo: int = 0, unit_hi: int = -1, flags: int = 0,
               stream: Optional[int] = None) -> None:
    """slimattn_bwd_static: slimattn_bwd with the library's built-in scratch array as workspace."""
    lib = load_library()
    prm = _params(tables.total_tokens, n_q_heads, n_kv_heads, head_dim, dtype, scale, unit_lo, unit_hi, flags)
    rc = lib.slimattn_bwd_static(C.byref(prm), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(dO), tables.handle,
                                 _ptr(dQ), _ptr(dK), _ptr(dV), stream)
    if rc != 0:
        extra = f" hip={lib.slimattn_last_hip_error()}" if rc == -4 else ""
        raise SlimAttnError(rc, "slimattn_bwd_static", extra)


def profile_enable(max_launches: int) -> None:
    rc = load_library().slimattn_profile_enable(max_launches)
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_profile_enable")


def profile_read():
    """{kernel class: (total ms, launches)} since the last read.  Raises if launches went untimed because the
    event pool was too small (the sums would under-count)."""
    ms = (C.c_double * len(KERNEL_CLASSES))()
    n = (C.c_int64 * len(KERNEL_CLASSES))()
    rc = load_library().slimattn_profile_read(ms, n)
    if rc != 0:
        raise SlimAttnError(rc, "slimattn_profile_read", " (event pool too small: launches ran untimed)" if rc == -3 else "")
    return {name: (ms[i], n[i]) for i, name in enumerate(KERNEL_CLASSES)}


def profile_read_launches():
    """Per launch, in launch order: arrays (kernel class, pass, unit, ms).  Raises if launches were dropped."""
    lib = load_library()
    n, dropped = C.c_int32(0), C.c_int64(0)
    rc = lib.slimattn_profile_read_launches(0, None, None, None, None, C.byref(n), C.byref(dropped))
    if rc not in (0, -3):
        raise SlimAttnError(rc, "slimattn_profile_read_launches")
    cap = n.value
    cls, ps, un = (np.zeros(cap, np.int32) for _ in range(3))
    ms = np.zeros(cap, np.float32)
    if cap:
        rc = lib.slimattn_profile_read_launches(cap, _p(cls), _p(ps), _p(un), ms.ctypes.data_as(C.POINTER(C.c_float)),
                                                C.byref(n), C.byref(dropped))
        if rc != 0:
            raise SlimAttnError(rc, "slimattn_profile_read_launches")
    if dropped.value:
        raise SlimAttnError(-3, "slimattn_profile_read_launches", f" ({dropped.value} launches ran untimed)")
    return cls, ps, un, ms
