"""ctypes access to the CPU oracle and the loop-nest simulator.

TEST INFRASTRUCTURE: only tests, the smoke check and the CPU-baseline leg of
the benchmark import this package.  It never imports the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboracle.so")
SOURCES = [os.path.join(_HERE, "oracle.c"), os.path.join(_HERE, "sim.c"), os.path.join(_HERE, "offline.c")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add contraction)."""
    if not force and os.path.exists(LIB_PATH):
        newest = max(os.path.getmtime(s) for s in SOURCES)
        if os.path.getmtime(LIB_PATH) >= newest:
            return LIB_PATH
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-Wall", "-Wextra", "-o", LIB_PATH] + SOURCES + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB_PATH


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


class Detail(C.Structure):
    _fields_ = [("bs", C.c_uint64 * 5), ("loads", C.c_uint64 * 6), ("da", C.c_uint64 * 5),
                ("tau", C.c_uint32 * 5), ("bs_op1", C.c_uint64), ("bs_op2", C.c_uint64),
                ("br_tile1", C.c_uint64), ("br_tile2", C.c_uint64),
                ("cyc_tile1", C.c_uint64), ("cyc_tile2", C.c_uint64),
                ("rho", C.c_uint64), ("softmax_elems", C.c_uint64),
                ("prefix_len", C.c_uint32), ("n1_len", C.c_uint32), ("n2_len", C.c_uint32),
                ("prefix", C.c_uint8 * 4), ("n1", C.c_uint8 * 4), ("n2", C.c_uint8 * 4)]


class SimResult(C.Structure):
    _fields_ = [("da", C.c_uint64 * 5), ("max_occupancy", C.c_uint64),
                ("max_reserved", C.c_uint64), ("max_reserved_touch", C.c_uint64),
                ("footprint", C.c_uint64 * 5), ("n_regions", C.c_uint64),
                ("macs1", C.c_uint64), ("macs2", C.c_uint64), ("softmax_elems", C.c_uint64),
                ("stages1", C.c_uint64), ("stages2", C.c_uint64), ("n_stages", C.c_uint64),
                ("occ_trace", C.c_uint32 * 64),
                ("psum_violation", C.c_int32), ("coverage_error", C.c_int32)]


OBJ_ENERGY, OBJ_LATENCY, OBJ_LATENCY_THEN_ENERGY, OBJ_EDP = 0, 1, 2, 3
N_OBJ = 4

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(LIB_PATH)
        P = C.POINTER
        L.orc_from_attention.argtypes = [P(Workload), P(Chain)]
        L.orc_space_size.argtypes = [P(Chain), P(Hw), P(C.c_uint64)]
        L.orc_decode.argtypes = [P(Chain), P(Hw), C.c_uint64, P(Mapping)]
        L.orc_eval.argtypes = [P(Chain), P(Hw), C.c_uint64, P(Mapping), P(Cost), P(Detail)]
        L.orc_eval_mapping.argtypes = [P(Chain), P(Hw), P(Mapping), P(Cost), P(Detail)]
        L.orc_eval_batch.argtypes = [P(Chain), P(Hw), C.c_uint64, C.c_uint64, C.c_void_p]
        L.orc_search_range.argtypes = [P(Chain), P(Hw), C.c_int, C.c_uint64, C.c_uint64,
                                       P(C.c_uint64), P(Cost), P(C.c_uint64), P(C.c_int)]
        L.orc_search.argtypes = [P(Chain), P(Hw), C.c_int,
                                 P(C.c_uint64), P(Cost), P(C.c_uint64), P(C.c_int)]
        L.orc_search_all.argtypes = [P(Chain), P(Hw), C.c_uint64, C.c_uint64,
                                     C.c_uint64 * 4, Cost * 4, P(C.c_uint64), P(C.c_int)]
        L.orc_pareto.argtypes = [P(Chain), P(Hw), C.c_uint64, C.c_uint64, C.c_uint32,
                                 P(C.c_uint64), P(Cost), P(C.c_uint32)]
        L.orc_front.argtypes = [P(Chain), P(Hw), C.c_int, C.c_uint64, C.c_uint64, C.c_uint32,
                                P(C.c_uint64), P(Cost), P(C.c_uint32)]
        L.sim_run.argtypes = [C.c_uint32 * 4, C.c_uint32 * 4, C.c_uint8 * 4, C.c_uint8 * 4,
                              C.c_int, C.c_int, P(SimResult)]
        L.sim_tile_matmul.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_int,
                                      C.c_uint32, C.c_uint32, C.c_uint32,
                                      P(C.c_uint64), P(C.c_uint64), P(C.c_uint64)]
        L.orc_offline_rows.argtypes = [C.c_int, C.c_int, P(C.c_uint32), P(C.c_uint32), P(C.c_uint32),
                                       P(C.c_uint32), P(C.c_uint32)]
        L.orc_offline_rows.restype = C.c_int
        for name in ("orc_from_attention", "orc_space_size", "orc_decode", "orc_eval", "orc_eval_mapping",
                     "orc_eval_batch", "orc_search_range", "orc_search", "orc_search_all", "orc_pareto", "orc_front", "sim_run",
                     "sim_tile_matmul"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def workload(cfg: dict) -> Chain:
    """Attention shape (B, H, N, d) or free chain shape (batch, I, K, L, J) -> the oracle's chain."""
    if "I" in cfg:
        return Chain(cfg["batch"], cfg["I"], cfg["K"], cfg["L"], cfg["J"], cfg["word_bytes"],
                     cfg["tiling_mode"], cfg["c_softmax"])
    a = Workload(cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["word_bytes"],
                 cfg["tiling_mode"], cfg["c_softmax"], 0)
    c = Chain()
    if lib().orc_from_attention(C.byref(a), C.byref(c)):
        raise ValueError("orc_from_attention failed")
    return c


def hw(cfg: dict) -> Hw:
    return Hw(cfg["pe_rows"], cfg["pe_cols"], cfg["n_arrays"], cfg["rf_bytes"], cfg["gb_bytes"],
              cfg["e_dram"], cfg["e_gb"], cfg["e_rf"], cfg["e_mac"], cfg["dram_bw"], cfg["gb_bw"])


def space_size(w: Chain, h: Hw) -> int:
    out = C.c_uint64()
    rc = lib().orc_space_size(C.byref(w), C.byref(h), C.byref(out))
    if rc:
        raise ValueError(f"orc_space_size rc={rc}")
    return out.value


def evaluate(w: Chain, h: Hw, idx: int):
    m, c, d = Mapping(), Cost(), Detail()
    rc = lib().orc_eval(C.byref(w), C.byref(h), idx, C.byref(m), C.byref(c), C.byref(d))
    if rc:
        raise ValueError(f"orc_eval rc={rc}")
    return m, c, d


def evaluate_mapping(w: Chain, h: Hw, m: Mapping):
    c, d = Cost(), Detail()
    rc = lib().orc_eval_mapping(C.byref(w), C.byref(h), C.byref(m), C.byref(c), C.byref(d))
    if rc:
        raise ValueError(f"orc_eval_mapping rc={rc}")
    return c, d


def eval_batch(w: Chain, h: Hw, first_idx: int, n: int):
    """Returns a numpy structured array of n cost records."""
    import numpy as np
    out = np.zeros(n, dtype=COST_DTYPE)
    rc = lib().orc_eval_batch(C.byref(w), C.byref(h), first_idx, n, out.ctypes.data)
    if rc:
        raise ValueError(f"orc_eval_batch rc={rc}")
    return out


def search(w: Chain, h: Hw, objective: int, first_idx: int | None = None, n: int | None = None):
    """Exhaustive search.  Returns (rc, best_idx, Cost, n_valid, threads)."""
    bi, c, nv, th = C.c_uint64(), Cost(), C.c_uint64(), C.c_int()
    if first_idx is None:
        rc = lib().orc_search(C.byref(w), C.byref(h), objective, C.byref(bi), C.byref(c),
                              C.byref(nv), C.byref(th))
    else:
        rc = lib().orc_search_range(C.byref(w), C.byref(h), objective, first_idx, n,
                                    C.byref(bi), C.byref(c), C.byref(nv), C.byref(th))
    return rc, bi.value, c, nv.value, th.value


def search_all(w: Chain, h: Hw, first_idx: int | None = None, n: int | None = None):
    """One exhaustive pass, all four objectives.  Returns (rc, [idx]*4, [Cost]*4, n_valid, threads)."""
    if first_idx is None:
        first_idx, n = 0, space_size(w, h)
    bi, bc, nv, th = (C.c_uint64 * 4)(), (Cost * 4)(), C.c_uint64(), C.c_int()
    rc = lib().orc_search_all(C.byref(w), C.byref(h), first_idx, n, bi, bc, C.byref(nv), C.byref(th))
    return rc, list(bi), list(bc), nv.value, th.value


def pareto(w: Chain, h: Hw, capacity: int = 1024, first_idx: int | None = None, n: int | None = None):
    """Energy-latency Pareto front.  Returns (rc, [idx], [Cost]) by ascending latency."""
    if first_idx is None:
        first_idx, n = 0, space_size(w, h)
    idx, cost, cnt = (C.c_uint64 * capacity)(), (Cost * capacity)(), C.c_uint32()
    rc = lib().orc_pareto(C.byref(w), C.byref(h), first_idx, n, capacity, idx, cost, C.byref(cnt))
    return rc, list(idx[:cnt.value]), list(cost[:cnt.value])


def front_bs_da(w: Chain, h: Hw, capacity: int = 1024, first_idx: int | None = None, n: int | None = None):
    """DRAM access versus buffer size front over all dataflows.  Returns (rc, [idx], [Cost]) by
    ascending buffer size."""
    if first_idx is None:
        first_idx, n = 0, space_size(w, h)
    idx, cost, cnt = (C.c_uint64 * capacity)(), (Cost * capacity)(), C.c_uint32()
    rc = lib().orc_front(C.byref(w), C.byref(h), 1, first_idx, n, capacity, idx, cost, C.byref(cnt))
    return rc, list(idx[:cnt.value]), list(cost[:cnt.value])


def offline_rows(r: int, f: int):
    """Offline symbolic pruning of group (r, f): (rows that denote a dataflow, surviving rows,
    dominator of every removed row or None), row numbers inside the group."""
    valid, kept, dom = (C.c_uint32 * 15000)(), (C.c_uint32 * 15000)(), (C.c_uint32 * 15000)()
    nv, nk = C.c_uint32(), C.c_uint32()
    rc = lib().orc_offline_rows(r, f, valid, C.byref(nv), kept, C.byref(nk), dom)
    if rc:
        raise ValueError(f"orc_offline_rows rc={rc}")
    return list(valid[:nv.value]), list(kept[:nk.value]), [None if d == 0xFFFFFFFF else d for d in dom]


def simulate(xG, xD, order, level, recompute: int, fused: int) -> SimResult:
    r = SimResult()
    rc = lib().sim_run((C.c_uint32 * 4)(*xG), (C.c_uint32 * 4)(*xD), (C.c_uint8 * 4)(*order),
                       (C.c_uint8 * 4)(*level), recompute, fused, C.byref(r))
    if rc:
        raise ValueError(f"sim_run rc={rc}")
    return r


def sim_tile_matmul(m, r, n, mode, R, Cc, g):
    w, cy, mac = C.c_uint64(), C.c_uint64(), C.c_uint64()
    rc = lib().sim_tile_matmul(m, r, n, mode, R, Cc, g, C.byref(w), C.byref(cy), C.byref(mac))
    if rc:
        raise ValueError(f"sim_tile_matmul rc={rc}")
    return w.value, cy.value, mac.value


def _cost_dtype():
    import numpy as np
    return np.dtype([("bs_words", "<u8"), ("da_words", "<u8"), ("br_words", "<u8"),
                     ("mac_total", "<u8"), ("comp_cycles", "<u8"),
                     ("energy_pj", "<f8"), ("latency_cycles", "<f8"),
                     ("valid", "<u4"), ("reason", "<u4")])


COST_DTYPE = _cost_dtype()
