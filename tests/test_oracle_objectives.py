"""Pins for the oracle's reductions beyond a single minimum: the energy-delay product
objective (Sec. VII-K) and the energy-latency Pareto front (Sec. VI-A, Sec. VII-E), each against
its textbook definition evaluated with numpy on spaces small enough to hold in memory."""
import numpy as np
import pytest

import oracle as O

# (workload, hw, first index row, number of index rows): windows of a few million candidates;
# a minimum or a front over a window is defined exactly like one over the whole space
CASES = [
    dict(w=dict(B=1, H=1, N=16, d=4, word_bytes=2, tiling_mode=1, c_softmax=10),
         h=dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=16, gb_bytes=300,
                e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=1.0, gb_bw=2.0),
         rows=(270000, 30000)),               # fused, r = 0 and 1, first stationary pair
    dict(w=dict(B=1, H=1, N=16, d=4, word_bytes=2, tiling_mode=1, c_softmax=10),
         h=dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=16, gb_bytes=300,
                e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=1.0, gb_bw=2.0),
         rows=(300000, 15000)),
    dict(w=dict(B=1, H=2, N=8, d=2, word_bytes=2, tiling_mode=1, c_softmax=10),
         h=dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=96,
                e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=2.0, gb_bw=64.0),
         rows=(0, 100000)),                   # unfused rows, several stationary pairs
    dict(w=dict(batch=2, I=12, K=3, L=8, J=6, word_bytes=2, tiling_mode=1, c_softmax=0),
         h=dict(pe_rows=2, pe_cols=2, n_arrays=1, rf_bytes=12, gb_bytes=260,
                e_dram=60.0, e_gb=9.0, e_rf=2.0, e_mac=1.0, dram_bw=0.75, gb_bw=3.0),
         rows=(270000 + 4 * 30000, 30000)),
]
_cache = {}


def all_costs(k):
    if k not in _cache:
        case = CASES[k]
        w, h = O.workload(case["w"]), O.hw(case["h"])
        T = O.space_size(w, h) // 540000
        first, n = case["rows"][0] * T, case["rows"][1] * T
        c = O.eval_batch(w, h, first, n)
        ok = c["valid"] == 1
        E = np.where(ok, c["energy_pj"], np.inf)
        L = np.where(ok, c["latency_cycles"], np.inf)
        _cache[k] = (w, h, first, n, E, L)
    return _cache[k]


@pytest.mark.parametrize("k", range(len(CASES)))
def test_edp_objective_is_argmin_of_energy_times_latency(k):
    w, h, first, n, E, L = all_costs(k)
    with np.errstate(invalid="ignore"):
        edp = np.where(np.isfinite(E), E * L, np.inf)
    best = int(np.lexsort((np.arange(n), edp))[0])
    rc, idx, cost, _, _ = O.search_all(w, h, first, n)
    assert rc == 0 and idx[O.OBJ_EDP] == first + best
    assert cost[O.OBJ_EDP].energy_pj * cost[O.OBJ_EDP].latency_cycles == edp[best]
    rc1, i1, c1, _, _ = O.search(w, h, O.OBJ_EDP, first, n)
    assert rc1 == 0 and i1 == first + best
    # the product can only be as good as the two single-metric optima allow
    assert edp[best] >= E.min() * L.min()


def front_by_definition(E, L):
    """Sort by (latency, energy, index) and keep each point whose energy is strictly below
    everything before it: exactly the non-dominated set, lowest index among duplicates."""
    order = np.lexsort((np.arange(len(E)), E, L))
    out, best = [], np.inf
    for i in order:
        if not np.isfinite(L[i]):
            break
        if E[i] < best:
            out.append(int(i))
            best = E[i]
    return out


@pytest.mark.parametrize("k", range(len(CASES)))
def test_pareto_front_matches_the_definition(k):
    w, h, first, n, E, L = all_costs(k)
    want = front_by_definition(E, L)
    rc, idx, cost = O.pareto(w, h, 1024, first, n)
    assert rc == 0 and [i - first for i in idx] == want
    for i, c in zip(want, cost):
        assert c.energy_pj == E[i] and c.latency_cycles == L[i]
    # no candidate at all dominates a front point, and every candidate is covered by one
    fe, fl = E[want], L[want]
    for e, l in zip(fe, fl):
        assert not np.any((E <= e) & (L <= l) & ((E < e) | (L < l)))
    rng = np.random.default_rng(0)
    for i in rng.integers(0, n, 2000):
        if np.isfinite(E[i]):
            assert np.any((fe <= E[i]) & (fl <= L[i]))
    # its two ends are the single-objective optima
    rc, sidx, scost, _, _ = O.search_all(w, h, first, n)
    assert cost[0].latency_cycles == scost[O.OBJ_LATENCY].latency_cycles
    assert cost[-1].energy_pj == scost[O.OBJ_ENERGY].energy_pj
    assert idx[0] == sidx[O.OBJ_LATENCY_THEN_ENERGY]


@pytest.mark.parametrize("k", range(len(CASES)))
def test_dram_access_versus_buffer_size_front_matches_the_definition(k):
    """Sec. VII-C plots minimum DRAM access against buffer size requirement: the non-dominated
    (buffer size, DRAM access) pairs over every dataflow, whatever the buffer capacity."""
    case = CASES[k]
    w, h = O.workload(case["w"]), O.hw(case["h"])
    T = O.space_size(w, h) // 540000
    first, n = case["rows"][0] * T, case["rows"][1] * T
    c = O.eval_batch(w, h, first, n)
    real = c["reason"] != 1
    BS = np.where(real, c["bs_words"].astype(np.float64), np.inf)
    DA = np.where(real, c["da_words"].astype(np.float64), np.inf)
    want = front_by_definition(DA, BS)            # ascending buffer size, strictly falling traffic
    rc, idx, cost = O.front_bs_da(w, h, 1024, first, n)
    assert rc == 0 and [i - first for i in idx] == want
    assert len(want) >= 3
    for i, cc in zip(want, cost):
        assert cc.bs_words == BS[i] and cc.da_words == DA[i]
    bs = [cc.bs_words for cc in cost]
    da = [cc.da_words for cc in cost]
    assert bs == sorted(bs) and da == sorted(da, reverse=True)
    # the far end is the compulsory traffic: every matrix moved once
    X = case["w"]
    I, K, L, J = (X["I"], X["K"], X["L"], X["J"]) if "I" in X else (X["N"], X["d"], X["N"], X["d"])
    if case["rows"][0] >= 270000:                 # fused rows: C never touches DRAM
        assert da[-1] == I * K + K * L + L * J + I * J


def test_pareto_front_has_several_points_somewhere():
    w, h, first, n, E, L = all_costs(0)
    assert len(front_by_definition(E, L)) >= 3


def test_pareto_reports_infeasible_and_overflow():
    case = CASES[2]
    w = O.workload(case["w"])
    rc, idx, _ = O.pareto(w, O.hw(dict(case["h"], gb_bytes=4)), 16, 0, 300000)
    assert rc == -3 and idx == []
    w0, h0, first, n, _, _ = all_costs(0)
    rc, idx, _ = O.pareto(w0, h0, 2, first, n)
    assert rc == -5
