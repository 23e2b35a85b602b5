"""Python binding of libmmee (include/mmee.h): argument marshalling only.

Every number comes out of the HIP kernels behind the C ABI.  There is no CPU
fallback: importing this package without a built libmmee.so raises, and calls
on a machine without a GPU return MMEE_EDEVICE (raised as MmeeError).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MMEE_LIB") or os.path.join(_HERE, "libmmee.so")

OBJ_ENERGY, OBJ_LATENCY, OBJ_LATENCY_THEN_ENERGY, OBJ_EDP = 0, 1, 2, 3
SEARCH_PRUNED, SEARCH_EXHAUSTIVE, SEARCH_ORDERED_SUM = 0, 1, 2
OK, EINVAL, ERANGE, ENOFEASIBLE, EDEVICE, EOVERFLOW, ETOOBIG = 0, -1, -2, -3, -4, -5, -6


class MmeeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {_strerror(code)} (code {code})")


class Workload(C.Structure):
    _fields_ = [("B", C.c_uint32), ("H", C.c_uint32), ("N", C.c_uint32), ("d", C.c_uint32),
                ("word_bytes", C.c_uint32), ("tiling_mode", C.c_uint32),
                ("c_softmax", C.c_uint32), ("reserved", C.c_uint32)]


class Chain(C.Structure):
    _fields_ = [("batch", C.c_uint32), ("I", C.c_uint32), ("K", C.c_uint32), ("L", C.c_uint32),
                ("J", C.c_uint32), ("word_bytes", C.c_uint32), ("tiling_mode", C.c_uint32),
                ("c_softmax", C.c_uint32)]


class Hw(C.Structure):
    _fields_ = [("pe_rows", C.c_uint32), ("pe_cols", C.c_uint32), ("n_arrays", C.c_uint32),
                ("rf_bytes", C.c_uint32), ("gb_bytes", C.c_uint64),
                ("e_dram", C.c_double), ("e_gb", C.c_double), ("e_rf", C.c_double),
                ("e_mac", C.c_double), ("dram_bw", C.c_double), ("gb_bw", C.c_double)]


class Mapping(C.Structure):
    _fields_ = [("idx", C.c_uint64), ("xG", C.c_uint32 * 4), ("xD", C.c_uint32 * 4),
                ("order", C.c_uint8 * 4), ("level", C.c_uint8 * 4),
                ("recompute", C.c_uint8), ("stat1", C.c_uint8), ("stat2", C.c_uint8),
                ("fused", C.c_uint8)]


class Cost(C.Structure):
    _fields_ = [("bs_words", C.c_uint64), ("da_words", C.c_uint64), ("br_words", C.c_uint64),
                ("mac_total", C.c_uint64), ("comp_cycles", C.c_uint64),
                ("energy_pj", C.c_double), ("latency_cycles", C.c_double),
                ("valid", C.c_uint32), ("reason", C.c_uint32)]


class Result(C.Structure):
    _fields_ = [("best", Mapping), ("cost", Cost), ("space", C.c_uint64), ("evaluated", C.c_uint64),
                ("seconds", C.c_double), ("kernel_seconds", C.c_double)]


class RowStats(C.Structure):
    _fields_ = [("rows_total", C.c_uint32 * 4), ("rows_valid", C.c_uint32 * 4),
                ("rows_kept", C.c_uint32 * 4)]


COST_DTYPE = np.dtype([("bs_words", "<u8"), ("da_words", "<u8"), ("br_words", "<u8"),
                       ("mac_total", "<u8"), ("comp_cycles", "<u8"),
                       ("energy_pj", "<f8"), ("latency_cycles", "<f8"),
                       ("valid", "<u4"), ("reason", "<u4")])
assert COST_DTYPE.itemsize == C.sizeof(Cost) == 64


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no CPU fallback for the MMEE kernels.")
    L = C.CDLL(LIB_PATH)
    P = C.POINTER
    L.mmee_space_size.argtypes = [P(Workload), P(Hw), P(C.c_uint64)]
    L.mmee_decode.argtypes = [P(Workload), P(Hw), P(C.c_uint64), C.c_uint64, P(Mapping)]
    L.mmee_eval_batch.argtypes = [P(Workload), P(Hw), C.c_uint64, C.c_uint64, C.c_void_p]
    L.mmee_search.argtypes = [P(Workload), P(Hw), C.c_int, P(Result)]
    L.mmee_search_ex.argtypes = [P(Workload), P(Hw), C.c_int, C.c_uint32, P(Result)]
    L.mmee_search_multi.argtypes = [P(Workload), P(Hw), P(C.c_int), C.c_uint32, C.c_uint32, P(Result)]
    L.mmee_search_many.argtypes = [P(Workload), P(Hw), P(C.c_int), C.c_uint32, C.c_uint32, P(Result),
                                   P(C.c_int)]
    L.mmee_chain_space_size.argtypes = [P(Chain), P(Hw), P(C.c_uint64)]
    L.mmee_energy_regrouped.argtypes = [P(Workload), P(Hw), C.c_uint32, P(C.c_int)]
    L.mmee_chain_energy_regrouped.argtypes = [P(Chain), P(Hw), C.c_uint32, P(C.c_int)]
    L.mmee_chain_decode.argtypes = [P(Chain), P(Hw), P(C.c_uint64), C.c_uint64, P(Mapping)]
    L.mmee_chain_eval_batch.argtypes = [P(Chain), P(Hw), C.c_uint64, C.c_uint64, C.c_void_p]
    L.mmee_chain_search_multi.argtypes = [P(Chain), P(Hw), P(C.c_int), C.c_uint32, C.c_uint32, P(Result)]
    L.mmee_chain_search_many.argtypes = [P(Chain), P(Hw), P(C.c_int), C.c_uint32, C.c_uint32, P(Result),
                                         P(C.c_int)]
    L.mmee_pareto.argtypes = [P(Workload), P(Hw), C.c_uint32, P(Result), C.c_uint32, P(C.c_uint32)]
    L.mmee_chain_pareto.argtypes = [P(Chain), P(Hw), C.c_uint32, P(Result), C.c_uint32, P(C.c_uint32)]
    L.mmee_front_bs_da.argtypes = [P(Workload), P(Hw), C.c_uint32, P(Result), C.c_uint32, P(C.c_uint32)]
    L.mmee_chain_front_bs_da.argtypes = [P(Chain), P(Hw), C.c_uint32, P(Result), C.c_uint32, P(C.c_uint32)]
    L.mmee_search_noalloc.argtypes = [P(Workload), P(Hw), C.c_int, C.c_uint32, C.c_void_p]
    L.mmee_offline_stats.argtypes = [P(RowStats)]
    L.mmee_offline_rows.argtypes = [C.c_uint32, C.c_uint32, P(C.c_uint32), C.c_uint32, P(C.c_uint32)]
    L.mmee_set_stream.argtypes = [C.c_void_p]
    L.mmee_shutdown.argtypes = []
    L.mmee_shutdown.restype = None
    L.mmee_strerror.argtypes = [C.c_int]
    L.mmee_strerror.restype = C.c_char_p
    for name in ("mmee_space_size", "mmee_decode", "mmee_eval_batch", "mmee_search", "mmee_search_ex",
                 "mmee_search_multi", "mmee_search_many", "mmee_search_noalloc", "mmee_offline_stats", "mmee_offline_rows", "mmee_set_stream",
                 "mmee_chain_space_size", "mmee_chain_decode", "mmee_chain_eval_batch",
                 "mmee_chain_search_multi", "mmee_chain_search_many", "mmee_pareto", "mmee_chain_pareto",
                 "mmee_front_bs_da", "mmee_chain_front_bs_da"):
        getattr(L, name).restype = C.c_int
    return L


_lib = _load()


def _strerror(code: int) -> str:
    return _lib.mmee_strerror(code).decode()


def _check(code: int, where: str, allow=()):
    if code != OK and code not in allow:
        raise MmeeError(code, where)
    return code


def workload(cfg) -> Workload:
    if isinstance(cfg, Workload):
        return cfg
    return Workload(cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["word_bytes"],
                    cfg["tiling_mode"], cfg["c_softmax"], 0)


def chain(cfg) -> Chain:
    if isinstance(cfg, Chain):
        return cfg
    return Chain(cfg["batch"], cfg["I"], cfg["K"], cfg["L"], cfg["J"], cfg["word_bytes"],
                 cfg["tiling_mode"], cfg["c_softmax"])


def hw(cfg) -> Hw:
    if isinstance(cfg, Hw):
        return cfg
    return Hw(cfg["pe_rows"], cfg["pe_cols"], cfg["n_arrays"], cfg["rf_bytes"], cfg["gb_bytes"],
              cfg["e_dram"], cfg["e_gb"], cfg["e_rf"], cfg["e_mac"], cfg["dram_bw"], cfg["gb_bw"])


def mmee_space_size(w, h) -> int:
    out = C.c_uint64()
    _check(_lib.mmee_space_size(C.byref(workload(w)), C.byref(hw(h)), C.byref(out)), "mmee_space_size")
    return out.value


def mmee_energy_regrouped(w, h, flags: int = SEARCH_PRUNED) -> bool:
    out = C.c_int()
    _check(_lib.mmee_energy_regrouped(C.byref(workload(w)), C.byref(hw(h)), flags, C.byref(out)),
           "mmee_energy_regrouped")
    return bool(out.value)


def mmee_chain_energy_regrouped(c, h, flags: int = SEARCH_PRUNED) -> bool:
    out = C.c_int()
    _check(_lib.mmee_chain_energy_regrouped(C.byref(chain(c)), C.byref(hw(h)), flags, C.byref(out)),
           "mmee_chain_energy_regrouped")
    return bool(out.value)


def mmee_decode(w, h, indices):
    idx = np.ascontiguousarray(indices, dtype=np.uint64)
    out = (Mapping * len(idx))()
    _check(_lib.mmee_decode(C.byref(workload(w)), C.byref(hw(h)),
                            idx.ctypes.data_as(C.POINTER(C.c_uint64)), len(idx), out), "mmee_decode")
    return list(out)


def mmee_eval_batch(w, h, first_idx: int, n: int, out=None):
    """Costs of n consecutive candidates.  out=None: returns a numpy record array (host);
    out=<int>: a device pointer to n 64-byte records, filled in place (nothing is copied back)."""
    if out is None:
        host = np.zeros(n, dtype=COST_DTYPE)
        _check(_lib.mmee_eval_batch(C.byref(workload(w)), C.byref(hw(h)), first_idx, n,
                                    host.ctypes.data), "mmee_eval_batch")
        return host
    _check(_lib.mmee_eval_batch(C.byref(workload(w)), C.byref(hw(h)), first_idx, n, C.c_void_p(int(out))),
           "mmee_eval_batch")
    return None


def mmee_search(w, h, objective: int) -> Result:
    r = Result()
    _check(_lib.mmee_search(C.byref(workload(w)), C.byref(hw(h)), objective, C.byref(r)), "mmee_search")
    return r


def mmee_search_ex(w, h, objective: int, flags: int = SEARCH_PRUNED, allow_infeasible: bool = False):
    r = Result()
    code = _check(_lib.mmee_search_ex(C.byref(workload(w)), C.byref(hw(h)), objective, flags, C.byref(r)),
                  "mmee_search_ex", allow=(ENOFEASIBLE,) if allow_infeasible else ())
    return (code, r) if allow_infeasible else r


def mmee_search_noalloc(w, h, objective: int, flags: int, out_dev: int) -> None:
    """Enqueue one search that allocates nothing; out_dev is a device pointer to one Result record,
    valid after the caller has synchronised the library's stream."""
    _check(_lib.mmee_search_noalloc(C.byref(workload(w)), C.byref(hw(h)), objective, flags,
                                    C.c_void_p(int(out_dev))), "mmee_search_noalloc")


def mmee_search_multi(w, h, objectives, flags: int = SEARCH_PRUNED):
    n = len(objectives)
    objs = (C.c_int * n)(*objectives)
    out = (Result * n)()
    _check(_lib.mmee_search_multi(C.byref(workload(w)), C.byref(hw(h)), objs, n, flags, out), "mmee_search_multi")
    return list(out)


class ManyPoints:
    """The argument arrays of mmee_search_many, marshalled once for repeated calls."""

    def __init__(self, points):
        n = self.n = len(points)
        self.ws = (Workload * n)(*[workload(p[0]) for p in points])
        self.hs = (Hw * n)(*[hw(p[1]) for p in points])
        self.objs = (C.c_int * n)(*[p[2] for p in points])
        self.out = (Result * n)()
        self.codes = (C.c_int * n)()


def mmee_search_many(points, flags: int = SEARCH_PRUNED):
    """points: sequence of (workload, hw, objective), or a ManyPoints made from one (its result
    arrays are then reused by the next call).  Returns (results, codes)."""
    m = points if isinstance(points, ManyPoints) else ManyPoints(points)
    _check(_lib.mmee_search_many(m.ws, m.hs, m.objs, m.n, flags, m.out, m.codes), "mmee_search_many", allow=(ENOFEASIBLE,))
    if m is points:
        return m.out, m.codes                   # the arrays themselves: valid until the next call with this ManyPoints
    return list(m.out), list(m.codes)


def mmee_chain_space_size(c, h) -> int:
    out = C.c_uint64()
    _check(_lib.mmee_chain_space_size(C.byref(chain(c)), C.byref(hw(h)), C.byref(out)), "mmee_chain_space_size")
    return out.value


def mmee_chain_decode(c, h, indices):
    idx = np.ascontiguousarray(indices, dtype=np.uint64)
    out = (Mapping * len(idx))()
    _check(_lib.mmee_chain_decode(C.byref(chain(c)), C.byref(hw(h)),
                                  idx.ctypes.data_as(C.POINTER(C.c_uint64)), len(idx), out), "mmee_chain_decode")
    return list(out)


def mmee_chain_eval_batch(c, h, first_idx: int, n: int, out=None):
    if out is None:
        host = np.zeros(n, dtype=COST_DTYPE)
        _check(_lib.mmee_chain_eval_batch(C.byref(chain(c)), C.byref(hw(h)), first_idx, n,
                                          host.ctypes.data), "mmee_chain_eval_batch")
        return host
    _check(_lib.mmee_chain_eval_batch(C.byref(chain(c)), C.byref(hw(h)), first_idx, n, C.c_void_p(int(out))),
           "mmee_chain_eval_batch")
    return None


def mmee_chain_search_multi(c, h, objectives, flags: int = SEARCH_PRUNED):
    n = len(objectives)
    objs = (C.c_int * n)(*objectives)
    out = (Result * n)()
    _check(_lib.mmee_chain_search_multi(C.byref(chain(c)), C.byref(hw(h)), objs, n, flags, out),
           "mmee_chain_search_multi")
    return list(out)


def mmee_chain_search_many(points, flags: int = SEARCH_PRUNED):
    """points: sequence of (chain, hw, objective).  Returns (results, codes)."""
    n = len(points)
    cs = (Chain * n)(*[chain(p[0]) for p in points])
    hs = (Hw * n)(*[hw(p[1]) for p in points])
    objs = (C.c_int * n)(*[p[2] for p in points])
    out = (Result * n)()
    codes = (C.c_int * n)()
    _check(_lib.mmee_chain_search_many(cs, hs, objs, n, flags, out, codes), "mmee_chain_search_many",
           allow=(ENOFEASIBLE,))
    return list(out), list(codes)


def _pareto(fn, name, problem, h, flags, capacity):
    out = (Result * capacity)()
    n = C.c_uint32()
    code = _check(fn(C.byref(problem), C.byref(hw(h)), flags, out, capacity, C.byref(n)), name,
                  allow=(ENOFEASIBLE, EOVERFLOW))
    return code, list(out[:n.value])


def mmee_pareto(w, h, flags: int = SEARCH_PRUNED, capacity: int = 256):
    """Energy-latency Pareto front by ascending latency.  Returns (code, [Result])."""
    return _pareto(_lib.mmee_pareto, "mmee_pareto", workload(w), h, flags, capacity)


def mmee_chain_pareto(c, h, flags: int = SEARCH_PRUNED, capacity: int = 256):
    return _pareto(_lib.mmee_chain_pareto, "mmee_chain_pareto", chain(c), h, flags, capacity)


def mmee_front_bs_da(w, h, flags: int = SEARCH_PRUNED, capacity: int = 1024):
    """DRAM access versus buffer size front by ascending buffer size.  Returns (code, [Result])."""
    return _pareto(_lib.mmee_front_bs_da, "mmee_front_bs_da", workload(w), h, flags, capacity)


def mmee_chain_front_bs_da(c, h, flags: int = SEARCH_PRUNED, capacity: int = 1024):
    return _pareto(_lib.mmee_chain_front_bs_da, "mmee_chain_front_bs_da", chain(c), h, flags, capacity)


def mmee_offline_stats() -> RowStats:
    s = RowStats()
    _check(_lib.mmee_offline_stats(C.byref(s)), "mmee_offline_stats")
    return s


def mmee_offline_rows(group: int, which: int = 1):
    """Row numbers (inside group g = r + 2 f) that denote a dataflow (which=0) or survive pruning (which=1)."""
    out = (C.c_uint32 * 15000)()
    n = C.c_uint32()
    _check(_lib.mmee_offline_rows(group, which, out, 15000, C.byref(n)), "mmee_offline_rows")
    return list(out[:n.value])


def mmee_set_stream(stream_ptr: int | None):
    _check(_lib.mmee_set_stream(C.c_void_p(stream_ptr or 0)), "mmee_set_stream")


def mmee_shutdown():
    _lib.mmee_shutdown()
