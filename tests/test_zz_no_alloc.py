"""mmee_search_noalloc (the entry point that allocates nothing) against mmee_search_ex, through the
C ABI: two calls in a row, the second on a smaller problem, then more keys and the exhaustive row
set; an oversized problem is refused.  Integer fields, index, energy and latency bit-exact."""
import ctypes as C

import pytest

from inputs import CONFIGS

pytestmark = pytest.mark.gpu

INT_FIELDS = ("bs_words", "da_words", "br_words", "mac_total", "comp_cycles", "valid", "reason")


@pytest.fixture(scope="module")
def M():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2604_03446_amd as mod
    return mod


def run_noalloc(M, w, h, objective, flags):
    import torch
    buf = torch.full((C.sizeof(M.Result),), 0xAB, dtype=torch.uint8, device="cuda")
    M.mmee_search_noalloc(w, h, objective, flags, buf.data_ptr())
    torch.cuda.synchronize()
    return M.Result.from_buffer_copy(buf.cpu().numpy().tobytes())


def assert_same(got, want, where):
    assert got.best.idx == want.best.idx, where
    for fld in ("xG", "xD", "order", "level"):
        assert list(getattr(got.best, fld)) == list(getattr(want.best, fld)), (where, fld)
    assert (got.best.recompute, got.best.stat1, got.best.stat2, got.best.fused) == \
        (want.best.recompute, want.best.stat1, want.best.stat2, want.best.fused), where
    for fld in INT_FIELDS:
        assert getattr(got.cost, fld) == getattr(want.cost, fld), (where, fld)
    assert got.cost.energy_pj == want.cost.energy_pj and got.cost.latency_cycles == want.cost.latency_cycles, where
    assert got.space == want.space and got.evaluated == want.evaluated, where


def test_noalloc_matches_search_ex_two_calls_in_a_row_second_smaller(M):
    big, small = CONFIGS["long"], CONFIGS["tiny"]
    first = run_noalloc(M, big["workload"], big["hw"], M.OBJ_ENERGY, M.SEARCH_PRUNED)
    second = run_noalloc(M, small["workload"], small["hw"], M.OBJ_ENERGY, M.SEARCH_PRUNED)
    assert_same(first, M.mmee_search_ex(big["workload"], big["hw"], M.OBJ_ENERGY, M.SEARCH_PRUNED), "long")
    assert_same(second, M.mmee_search_ex(small["workload"], small["hw"], M.OBJ_ENERGY, M.SEARCH_PRUNED), "tiny")


def test_noalloc_every_key_and_row_set(M):
    for name in ("bert", "tiny"):
        cfg = CONFIGS[name]
        w, h = cfg["workload"], cfg["hw"]
        for flags in (M.SEARCH_PRUNED, M.SEARCH_EXHAUSTIVE, M.SEARCH_PRUNED | M.SEARCH_ORDERED_SUM):
            for obj in range(4):
                assert_same(run_noalloc(M, w, h, obj, flags), M.mmee_search_ex(w, h, obj, flags), (name, flags, obj))


def test_noalloc_infeasible_and_too_big(M):
    cfg = CONFIGS["tiny"]
    got = run_noalloc(M, cfg["workload"], dict(cfg["hw"], gb_bytes=4), M.OBJ_LATENCY, M.SEARCH_PRUNED)
    assert got.cost.valid == 0
    # 240 * 240 tilings: beyond the fixed scratch, refused before anything is enqueued
    w = dict(B=1, H=1, N=720720, d=1, word_bytes=2, tiling_mode=1, c_softmax=10)
    with pytest.raises(M.MmeeError) as e:
        run_noalloc(M, w, cfg["hw"], M.OBJ_ENERGY, M.SEARCH_PRUNED)
    assert e.value.code == M.ETOOBIG and "57600" in str(e.value)
    # and the scratch still serves the next call
    assert_same(run_noalloc(M, cfg["workload"], cfg["hw"], M.OBJ_EDP, M.SEARCH_PRUNED),
                M.mmee_search_ex(cfg["workload"], cfg["hw"], M.OBJ_EDP, M.SEARCH_PRUNED), "after refusal")
