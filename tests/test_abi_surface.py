"""The C-ABI library loads and exports every symbol that include/mmee.h declares.
No compute call is made here (no GPU needed); host-only entry points are exercised."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mmee.h")
LIB = os.path.join(ROOT, "paper_2604_03446_amd", "libmmee.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmee_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_problem_statement():
    names = declared_functions()
    for required in ("mmee_space_size", "mmee_eval_batch", "mmee_search"):
        assert required in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_mirrors_the_header():
    import paper_2604_03446_amd as M
    for name in declared_functions():
        if name == "mmee_strerror":
            continue
        assert callable(getattr(M, name)), name
    assert ctypes.sizeof(M.Cost) == 64
    assert ctypes.sizeof(M.Mapping) == 56


def test_host_only_calls():
    import paper_2604_03446_amd as M
    from inputs import CONFIGS
    sizes = {k: M.mmee_space_size(c["workload"], c["hw"]) for k, c in CONFIGS.items()}
    assert sizes == {"tiny": 952560000, "bert": 2646000000, "prefill": 4976640000, "long": 6773760000}
    with pytest.raises(M.MmeeError) as e:
        M.mmee_space_size(dict(CONFIGS["tiny"]["workload"], d=0), CONFIGS["tiny"]["hw"])
    assert e.value.code == M.EINVAL
    # a workload whose counts would not stay exact integers in fp64 is refused, not approximated
    with pytest.raises(M.MmeeError):
        M.mmee_space_size(dict(CONFIGS["tiny"]["workload"], N=1 << 20, d=1 << 10, H=1 << 10), CONFIGS["tiny"]["hw"])


def test_host_factorisation_matches_naive_divisor_counts():
    """The online tiling enumeration (integer factorisation of every extent) is host logic:
    the space size must be the product of the divisor counts times 540000, in both tiling modes."""
    import paper_2604_03446_amd as M
    hw = dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=1 << 20,
              e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=64.0, gb_bw=256.0)

    def nd(x, mode):
        return sum(1 for g in range(1, x + 1) if x % g == 0 and (mode == 1 or g & (g - 1) == 0))

    for I, K, L, J in [(1, 1, 1, 1), (97, 2, 3, 5), (360, 48, 1000, 7), (720, 36, 49, 1024), (5040, 1, 2, 3)]:
        for mode in (0, 1):
            c = dict(batch=1, I=I, K=K, L=L, J=J, word_bytes=2, tiling_mode=mode, c_softmax=0)
            assert M.mmee_chain_space_size(c, hw) == nd(I, mode) * nd(K, mode) * nd(L, mode) * nd(J, mode) * 540000
    # attention is the chain I = L = N, K = J = d
    w = dict(B=2, H=3, N=360, d=48, word_bytes=2, tiling_mode=1, c_softmax=10)
    assert M.mmee_space_size(w, hw) == (nd(360, 1) * nd(48, 1)) ** 2 * 540000
    # an extent with more divisors than the tables hold is refused
    with pytest.raises(M.MmeeError):
        M.mmee_chain_space_size(dict(batch=1, I=1441440, K=1, L=1, J=1, word_bytes=2, tiling_mode=1, c_softmax=0), hw)


def test_energy_regrouping_is_offered_only_where_it_is_exact():
    """The search may add the energy as a row part plus a tiling part only when no rounding can
    occur: whole-number energies per access and a total below 2^53.  The size test rests on the
    bounds DRAM words <= 8 P, DRAM + buffer<->RF words <= 14 P, RF accesses <= 6 P and
    MACs + c_softmax * softmax elements <= (2 + c_softmax) P per instance, P = I*K*L*J; the oracle's
    maxima over whole small spaces (one unit energy at a time) must respect them."""
    import numpy as np
    import oracle as O
    import paper_2604_03446_amd as M
    from inputs import CONFIGS, sweep_hw
    reg = {k: M.mmee_energy_regrouped(c["workload"], c["hw"]) for k, c in CONFIGS.items()}
    assert reg == {"tiny": True, "bert": True, "prefill": True, "long": False}   # long: up to 2^56 pJ
    bert = CONFIGS["bert"]
    assert not M.mmee_energy_regrouped(bert["workload"], bert["hw"], M.SEARCH_ORDERED_SUM)
    assert not M.mmee_energy_regrouped(bert["workload"], dict(bert["hw"], e_gb=6.5))
    assert not M.mmee_energy_regrouped(bert["workload"], dict(bert["hw"], dram_bw=48.0))
    assert not M.mmee_energy_regrouped(bert["workload"], dict(bert["hw"], n_arrays=3))
    assert M.mmee_energy_regrouped(bert["workload"], dict(bert["hw"], e_dram=8.0e4))
    assert not M.mmee_energy_regrouped(bert["workload"], dict(bert["hw"], e_dram=9.0e4))
    assert not any(M.mmee_energy_regrouped(bert["workload"], h) for h in sweep_hw()[:8])  # fractional e_dram

    small = [dict(B=1, H=2, N=8, d=2, word_bytes=2, tiling_mode=1, c_softmax=10),
             dict(B=1, H=1, N=12, d=6, word_bytes=2, tiling_mode=0, c_softmax=3)]
    base_hw = dict(pe_rows=2, pe_cols=4, n_arrays=1, rf_bytes=32, gb_bytes=1 << 30,
                   e_dram=0.0, e_gb=0.0, e_rf=0.0, e_mac=0.0, dram_bw=2.0, gb_bw=64.0)
    for w in small:
        P = w["B"] * w["H"] * w["N"] * w["d"] * w["N"] * w["d"]
        ow = O.workload(w)
        for unit, coef in (("e_dram", 8), ("e_gb", 14), ("e_rf", 6), ("e_mac", 2 + w["c_softmax"])):
            oh = O.hw({**base_hw, unit: 1.0})
            S, worst = O.space_size(ow, oh), 0.0
            for first in range(0, S, 1 << 22):
                rec = O.eval_batch(ow, oh, first, min(1 << 22, S - first))
                e = rec["energy_pj"][rec["reason"] != 1]        # every index that denotes a dataflow
                worst = max(worst, float(e.max()))
                assert np.all(e == np.floor(e))
            assert 0 < worst <= coef * P, (w, unit, worst, coef * P)
