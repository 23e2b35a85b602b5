"""GPU parity for free two-GEMM / convolution-chain shapes (Sec. VII-J, Table V):
the same kernels, four independent loop extents, non-power-of-two divisors."""
import json
import os

import numpy as np
import pytest

import oracle as O
from inputs import CHAINS, SplitMix64
from test_gpu_parity import INT_FIELDS, OBJ_NAMES, assert_costs_equal, check_result_against_oracle, windows

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def M():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2604_03446_amd as mod
    return mod


@pytest.mark.parametrize("name", sorted(CHAINS))
def test_chain_eval_batch_windows(M, name):
    cfg = CHAINS[name]
    w, h = cfg["workload"], cfg["hw"]
    ow, oh = O.workload(w), O.hw(h)
    S = O.space_size(ow, oh)
    assert M.mmee_chain_space_size(w, h) == S
    T = S // 540000
    for first, n in list(windows(S, 23, [1, 65, 100003, 2 * T + 31])) + [(0, 50000), (S - 50001, 50001)]:
        got = M.mmee_chain_eval_batch(w, h, first, n)
        want = O.eval_batch(ow, oh, first, n)
        assert_costs_equal(got, want, (name, first, n))
    rng = SplitMix64(9)
    idx = [0, S - 1] + [rng.next() % S for _ in range(300)]
    for i, m in zip(idx, M.mmee_chain_decode(w, h, idx)):
        om, _, _ = O.evaluate(ow, oh, i)
        assert (list(m.xG), list(m.xD), list(m.order), list(m.level)) == \
            (list(om.xG), list(om.xD), list(om.order), list(om.level))


SMALL_CHAINS = [
    (dict(batch=3, I=6, K=4, L=10, J=3, word_bytes=2, tiling_mode=1, c_softmax=0),
     dict(pe_rows=2, pe_cols=4, n_arrays=2, rf_bytes=16, gb_bytes=150,
          e_dram=180.0, e_gb=6.5, e_rf=1.0, e_mac=0.75, dram_bw=4.0, gb_bw=8.0)),
    (dict(batch=1, I=9, K=8, L=2, J=15, word_bytes=4, tiling_mode=1, c_softmax=7),
     dict(pe_rows=3, pe_cols=5, n_arrays=3, rf_bytes=40, gb_bytes=1000,
          e_dram=210.0, e_gb=5.0, e_rf=2.0, e_mac=1.0, dram_bw=6.0, gb_bw=0.0)),
]


@pytest.mark.parametrize("case", range(len(SMALL_CHAINS)))
def test_chain_search_small_spaces_against_oracle_enumeration(M, case):
    w, h = SMALL_CHAINS[case]
    ow, oh = O.workload(w), O.hw(h)
    rc, idx, cost, n_valid, _ = O.search_all(ow, oh)
    assert rc == 0
    for flags in (M.SEARCH_EXHAUSTIVE, M.SEARCH_PRUNED):
        multi = M.mmee_chain_search_multi(w, h, [0, 1, 2], flags)
        for obj in (0, 1, 2):
            res = multi[obj]
            assert res.best.idx == idx[obj], (case, flags, obj)
            assert res.cost.energy_pj == cost[obj].energy_pj
            assert res.cost.latency_cycles == cost[obj].latency_cycles
            check_result_against_oracle(res, ow, oh)


def test_table5_shapes_against_stored_oracle_optima(M):
    with open(os.path.join(GOLDEN, "expected_optima.json")) as fh:
        exp = json.load(fh)
    points, names = [], []
    for name, cfg in sorted(CHAINS.items()):
        e = exp["chain_" + name]
        assert e["workload"] == cfg["workload"] and e["hw"] == cfg["hw"]
        for obj in (0, 1, 2):
            points.append((cfg["workload"], cfg["hw"], obj))
            names.append(name)
    for flags in (M.SEARCH_PRUNED, M.SEARCH_EXHAUSTIVE):
        results, codes = M.mmee_chain_search_many(points, flags)
        for (w, h, obj), res, code, name in zip(points, results, codes, names):
            want = exp["chain_" + name]["best"][OBJ_NAMES[obj]]
            assert code == 0 and res.best.idx == want["idx"], (name, obj, flags)
            assert res.cost.energy_pj == float.fromhex(want["energy_pj"])
            assert res.cost.latency_cycles == float.fromhex(want["latency_cycles"])
            for fld in INT_FIELDS:
                assert getattr(res.cost, fld) == want[fld]
            check_result_against_oracle(res, O.workload(w), O.hw(h))
