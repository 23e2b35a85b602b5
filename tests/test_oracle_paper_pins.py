"""Pins of the CPU oracle against what the paper prints.

Each test reads its expected values from a cited fixture under tests/golden/
(or states the cited sentence it checks) and never from the oracle itself.
"""
import itertools
import math
import os

import pytest

import oracle as O
from inputs import CONFIGS, SplitMix64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
DIMS = "iklj"


def read_fixture(name):
    kv = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip().split()
    return kv


def level_digit(name):
    # L3 is the tile itself, every further layer spans one more inter-tile loop
    return int(name[1:]) - 3


def all_tilings(N, d, mode=1):
    X = [N, d, N, d]
    divs = []
    for x in X:
        ds = [g for g in range(1, x + 1) if x % g == 0 and (mode == 1 or g & (g - 1) == 0)]
        divs.append(ds)
    for xg in itertools.product(*divs):
        yield list(xg), [X[q] // xg[q] for q in range(4)]


def monomial(q, xD, xG):
    b = list(xD) + list(xG)
    return math.prod(b[t] ** int(q[t]) for t in range(8))


HW = dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=1 << 40,
          e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=64.0, gb_bw=256.0)


def wl(N, d, H=1, B=1, c_softmax=10, mode=1):
    return dict(B=B, H=H, N=N, d=d, word_bytes=2, tiling_mode=mode, c_softmax=c_softmax)


def fig11_mapping(fx, xG, xD, r=0, s1=0, s2=0, f=1):
    order = [DIMS.index(c) for c in fx["order_outer_to_inner"]]
    level = [level_digit(fx["level_" + x][0]) for x in "ABDE"]
    m = O.Mapping()
    for q in range(4):
        m.xG[q], m.xD[q], m.order[q], m.level[q] = xG[q], xD[q], order[q], level[q]
    m.recompute, m.stat1, m.stat2, m.fused = r, s1, s2, f
    return m


def test_fig11_buffer_size_and_dram_access_closed_forms():
    """Sec. V-B (BS_A, Eq. 3) and Sec. V-C (Eq. 5, Eq. 6) for the example of Fig. 11."""
    fx = read_fixture("fig11_buffer_dram_example.txt")
    assert fx["b"] == "i_D k_D l_D j_D i_G k_G l_G j_G".split()
    w, h = O.workload(wl(12, 6)), O.hw(HW)
    n = 0
    for xG, xD in all_tilings(12, 6):
        m = fig11_mapping(fx, xG, xD)
        c, d = O.evaluate_mapping(w, h, m)
        assert d.bs[0] == monomial(fx["q_BS_A"], xD, xG)          # BS_A = k_D i_G k_G
        assert d.da[0] == monomial(fx["q_DA_A"], xD, xG)          # Eq. (5)
        assert d.da[0] == 12 * 6                                  # "the total size of matrix A"
        assert d.da[3] == monomial(fx["q_DA_D"], xD, xG)          # Eq. (6)
        assert d.da[3] == xD[0] * 12 * 6                          # "i_D copies of matrix D"
        assert d.tau[3] == int(fx["tau_D"][0]) and d.tau[4] == int(fx["tau_E"][0])
        assert d.bs_op1 == d.bs[0] + d.bs[1] + d.bs[2] + d.bs[4]  # Eq. (3)
        assert d.da[2] == 0                                       # DA_C = 0 (Sec. V-C)
        assert c.bs_words == max(d.bs_op1, d.bs_op2)              # Eq. (4)
        assert c.da_words == d.da[0] + d.da[1] + d.da[3] + d.da[4]  # Eq. (7)
        n += 1
    assert n == 6 * 4 * 6 * 4


def test_fig11_index_digits_agree_with_explicit_mapping():
    """The candidate index that encodes the Fig. 11 example decodes to that example."""
    fx = read_fixture("fig11_buffer_dram_example.txt")
    order = tuple(DIMS.index(c) for c in fx["order_outer_to_inner"])
    rank = sorted(itertools.permutations(range(4))).index(order)
    level = [level_digit(fx["level_" + x][0]) for x in "ABDE"]
    w, h = O.workload(wl(12, 6)), O.hw(HW)
    T = 6 * 4 * 6 * 4
    row = level[0] + 5 * (level[1] + 5 * (level[2] + 5 * (level[3] + 5 * (rank + 24 * (0 + 2 * (0 + 3 * (0 + 3 * 1)))))))
    for t in (0, 7, T - 1):
        m, c, d = O.evaluate(w, h, t + T * row)
        assert tuple(m.order) == order and list(m.level) == level
        assert (m.recompute, m.stat1, m.stat2, m.fused) == (0, 0, 0, 1)
        assert d.bs[0] == m.xD[1] * m.xG[0] * m.xG[1]


def test_fig10_unrolled_example_stage_sequence():
    """Sec. IV-B: ten stages, occupancy 3 -> 4 -> 3 tiles over the first three."""
    fx = read_fixture("fig10_unrolled_example.txt")
    fx11 = read_fixture("fig11_buffer_dram_example.txt")
    order = [DIMS.index(c) for c in fx11["order_outer_to_inner"]]
    level = [level_digit(fx11["level_" + x][0]) for x in "ABDE"]
    # unit tiles; k2 and j2 run 1..2; two C tiles (c1, c2) along l
    xG, xD = [1, 1, 1, 1], [1, 2, 2, 2]
    s = O.simulate(xG, xD, order, level, 0, 1)
    assert s.n_stages == int(fx["n_stages"][0])
    assert list(s.occ_trace[:3]) == [int(v) for v in fx["occupancy_stage_1_2_3"]]
    assert s.psum_violation == 0 and s.coverage_error == 0
    assert s.max_occupancy == 6          # a1 a2 c d e1 e2
    # the oracle's reservation for the same mapping equals the simulated peak, both for the
    # example itself (a chain with I = 1, K = L = J = 2) and for an attention shape (I = L)
    # with the same structure (i_G = 2: one tile row of two elements)
    for xG_, shape in (([1, 1, 1, 1], dict(batch=1, I=1, K=2, L=2, J=2, word_bytes=2, tiling_mode=1, c_softmax=10)),
                       ([2, 1, 1, 1], wl(2, 2))):
        s2 = O.simulate(xG_, xD, order, level, 0, 1)
        w, h = O.workload(shape), O.hw(HW)
        m = O.Mapping()
        for q in range(4):
            m.xG[q], m.xD[q], m.order[q], m.level[q] = xG_[q], xD[q], order[q], level[q]
        m.fused = 1
        c, d = O.evaluate_mapping(w, h, m)
        assert c.bs_words == s2.max_occupancy == (6 if xG_[0] == 1 else 4 + 1 + 2 + 4)
        assert list(d.da) == list(s2.da)


@pytest.mark.parametrize("N,d", [(8, 4), (12, 6)])
def test_mac_and_softmax_counts(N, d):
    """Sec. V-D: MACs = N_op1 + N_op2, or j_D N_op1 + N_op2 with recomputation;
    softmax energy c_softmax*i*l (times j_D with recomputation)."""
    hwd = dict(HW, e_dram=0.0, e_gb=0.0, e_rf=0.0, e_mac=1.0)
    h = O.hw(hwd)
    w10, w0 = O.workload(wl(N, d, H=3, c_softmax=10)), O.workload(wl(N, d, H=3, c_softmax=0))
    n_op1, n_op2 = N * d * N, N * d * N
    order_ok = [0, 2, 3, 1]      # j outside k: a C tile is rebuilt for every j
    for xG, xD in all_tilings(N, d):
        for r in (0, 1):
            m = O.Mapping()
            for q in range(4):
                m.xG[q], m.xD[q], m.order[q], m.level[q] = xG[q], xD[q], order_ok[q], 0
            m.recompute, m.fused = r, 1
            c10, _ = O.evaluate_mapping(w10, h, m)
            c0, _ = O.evaluate_mapping(w0, h, m)
            jD = xD[3]
            assert c10.mac_total == (jD if r else 1) * n_op1 + n_op2
            # with only e_mac = 1 the energy is the MAC count plus the softmax term, over 3 heads
            assert c0.energy_pj == 3 * c0.mac_total
            assert c10.energy_pj - c0.energy_pj == 3 * 10 * N * N * (jD if r else 1)
            # useful work never changes
            assert c10.mac_total - ((jD - 1) * n_op1 if r else 0) == 2 * N * N * d


def test_table2_bert_base_compute_bound_latency():
    """Table II, BERT-Base on Accel. 1: the printed latencies equal 12*2*N^2*64 MACs
    on 4 arrays of 1024 PEs at 1 GHz, i.e. the model's fully utilised compute term."""
    rows = []
    with open(os.path.join(GOLDEN, "table2_bert_base_accel1.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                n, ms = line.split()
                rows.append((int(n), float(ms)))
    assert [n for n, _ in rows] == [512, 4096, 16384]
    hwd = dict(pe_rows=32, pe_cols=32, n_arrays=4, rf_bytes=512, gb_bytes=1 << 20,
               e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=60.0, gb_bw=0.0)
    h = O.hw(hwd)
    for N, ms in rows:
        w = O.workload(wl(N, 64, H=12, mode=0))
        S = O.space_size(w, h)
        rng = SplitMix64(N)
        best = math.inf
        for _ in range(40000):
            _, c, _ = O.evaluate(w, h, rng.next() % S)
            if c.valid:
                best = min(best, c.latency_cycles)
        # 1 GHz: cycles / 1e6 = ms; the table prints two decimals
        assert round(best / 1e6, 2) == pytest.approx(ms, abs=0.0051)
        assert best == 12 * 2 * N * N * 64 / 4096


def test_single_tile_special_case():
    """x_D = 1 everywhere: one stage per operator, every matrix moved exactly once,
    everything resident (textbook unblocked matmul chain)."""
    N, d = 16, 8
    w, h = O.workload(wl(N, d)), O.hw(HW)
    for order in itertools.permutations(range(4)):
        for level in itertools.product(range(5), repeat=4):
            m = O.Mapping()
            for q in range(4):
                m.xG[q], m.xD[q], m.order[q], m.level[q] = [N, d, N, d][q], 1, order[q], level[q]
            m.fused = 1
            c, dt = O.evaluate_mapping(w, h, m)
            assert c.da_words == 4 * N * d
            assert list(dt.bs) == [N * d, d * N, N * N, N * d, N * d]
            assert c.mac_total == 2 * N * N * d


def test_energy_terms_isolated():
    """Sec. V-D: energy = DRAM<->buffer + buffer<->RF + compute; each unit-cost
    probe must return the matching access count (counts are pinned by the simulator)."""
    cfg = CONFIGS["tiny"]
    w = O.workload(dict(cfg["workload"], H=3, B=2))
    S = O.space_size(w, O.hw(cfg["hw"]))
    rng = SplitMix64(99)
    idxs = [rng.next() % S for _ in range(3000)]
    zero = dict(cfg["hw"], gb_bytes=1 << 40, e_dram=0.0, e_gb=0.0, e_rf=0.0, e_mac=0.0)
    probes = {k: O.hw({**zero, k: 1.0}) for k in ("e_dram", "e_gb", "e_rf", "e_mac")}
    seen = 0
    for idx in idxs:
        m, c, d = O.evaluate(w, probes["e_dram"], idx)
        if not c.valid:
            assert c.reason == 1
            continue
        seen += 1
        BH = 6
        assert c.energy_pj == BH * c.da_words
        assert O.evaluate(w, probes["e_gb"], idx)[1].energy_pj == BH * (c.da_words + c.br_words)
        assert O.evaluate(w, probes["e_rf"], idx)[1].energy_pj == BH * 3 * c.mac_total
        assert O.evaluate(w, probes["e_mac"], idx)[1].energy_pj == BH * (c.mac_total + 10 * d.softmax_elems)
    assert seen > 1000


def test_latency_is_max_of_streams():
    """Sec. V-D: latency = max(DRAM latency, compute latency) with full pipelining
    (plus the buffer<->RF stream when a buffer bandwidth is given)."""
    cfg = CONFIGS["tiny"]
    w = O.workload(dict(cfg["workload"], H=4))
    base = dict(cfg["hw"], gb_bytes=1 << 40)
    S = O.space_size(w, O.hw(base))
    rng = SplitMix64(5)
    hits = [0, 0, 0]
    for _ in range(3000):
        idx = rng.next() % S
        for dram_bw, gb_bw in ((64.0, 256.0), (0.5, 0.0), (0.0, 0.25), (1024.0, 8.0)):
            hw_ = O.hw(dict(base, n_arrays=2, dram_bw=dram_bw, gb_bw=gb_bw))
            _, c, _ = O.evaluate(w, hw_, idx)
            if not c.valid:
                continue
            streams = [float(c.comp_cycles),
                       c.da_words * 2 / dram_bw if dram_bw else 0.0,
                       c.br_words * 2 / gb_bw if gb_bw else 0.0]
            assert c.latency_cycles == pytest.approx(4 / 2 * max(streams), rel=1e-15)
            hits[streams.index(max(streams))] += 1
    assert all(hits)


def test_invariants_on_all_configs():
    """DRAM traffic is at least the compulsory traffic of Q, K, V and O; useful MACs are
    2*N^2*d per head; DA_C = 0 when fused; capacity mask is BS*word_bytes <= buffer bytes."""
    for name, cfg in CONFIGS.items():
        w, h = O.workload(cfg["workload"]), O.hw(cfg["hw"])
        N, d = cfg["workload"]["N"], cfg["workload"]["d"]
        S = O.space_size(w, h)
        rng = SplitMix64(hash(name) & 0xFFFF)
        nvalid = 0
        for _ in range(4000):
            m, c, dt = O.evaluate(w, h, rng.next() % S)
            if c.reason == 1:
                assert c.valid == 0 and math.isinf(c.energy_pj) and math.isinf(c.latency_cycles)
                assert m.recompute == 1
                continue
            assert c.da_words >= 4 * N * d
            rho = m.xD[3] if m.recompute else 1
            assert c.mac_total == (rho + 1) * N * N * d
            if m.fused:
                assert dt.da[2] == 0
            over = c.bs_words * 2 > cfg["hw"]["gb_bytes"]
            assert (c.valid == 0 and c.reason == 2) if over else (c.valid == 1 and c.reason == 0)
            nvalid += c.valid
        assert nvalid > 0


def test_two_gemm_and_conv_chain_shapes():
    """Sec. VII-J, Table V: two GEMMs [I,K,L,J] and convolution chains turned into GEMMs by im2col.
    The model is the same; only the four loop extents are free."""
    from inputs import CHAINS
    assert [CHAINS["mlp"]["workload"][k] for k in "IKLJ"] == [768, 64, 384, 64]
    assert [CHAINS["ffn"]["workload"][k] for k in "IKLJ"] == [2048, 768, 3072, 768]
    assert [CHAINS["cc1"]["workload"][k] for k in "IKLJ"] == [112 * 112, 64 * 9, 192, 128]
    assert [CHAINS["cc2"]["workload"][k] for k in "IKLJ"] == [56 * 56, 64, 64, 64]
    for name, cfg in CHAINS.items():
        w, h = O.workload(cfg["workload"]), O.hw(cfg["hw"])
        I, K, L, J = (cfg["workload"][k] for k in "IKLJ")
        S = O.space_size(w, h)
        rng = SplitMix64(len(name))
        seen = 0
        for _ in range(3000):
            m, c, dt = O.evaluate(w, h, rng.next() % S)
            assert [m.xG[q] * m.xD[q] for q in range(4)] == [I, K, L, J]
            if c.reason == 1:
                continue
            seen += 1
            rho = m.xD[3] if m.recompute else 1
            assert c.mac_total == rho * I * K * L + I * L * J
            assert c.da_words >= I * K + K * L + L * J + I * J      # every matrix moves at least once
            assert dt.softmax_elems == rho * I * L
        assert seen > 1000


def test_space_sizes():
    """Tilings come from integer factorisation of each dimension (Sec. VI-A); the
    loop-order / level / recompute / stationary / fusion choices number 540000."""
    expect = {"tiny": 7 * 6 * 7 * 6, "bert": 10 * 7 * 10 * 7, "prefill": 12 * 8 * 12 * 8, "long": 14 * 8 * 14 * 8}
    for name, T in expect.items():
        cfg = CONFIGS[name]
        assert O.space_size(O.workload(cfg["workload"]), O.hw(cfg["hw"])) == T * 540000
    # non-power-of-two shape: the two tiling modes differ
    h = O.hw(HW)
    assert O.space_size(O.workload(wl(48, 24, mode=1)), h) == (10 * 8) ** 2 * 540000
    assert O.space_size(O.workload(wl(48, 24, mode=0)), h) == (5 * 4) ** 2 * 540000
