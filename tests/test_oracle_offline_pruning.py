"""Pins for the plain reference of the offline symbolic pruning (oracle/offline.c; Sec. VI-B, Eq. (12)).

The reference decides with divisibility on a prime-valued probe; these tests check what that
decision must mean, numerically and on whole spaces, without using the probe:
every removed row has an earlier row that is no worse in buffer size and DRAM access on real
tilings of real shapes; searching only the surviving rows finds the optimum of the whole space,
index ties included; and a survivor is never beaten that way by an earlier row.
"""
import itertools

import numpy as np
import pytest

import oracle as O
from inputs import SplitMix64

HW = dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=1 << 40,
          e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=64.0, gb_bw=256.0)
GROUPS = [(0, 0), (1, 0), (0, 1), (1, 1)]          # (r, f), group number g = r + 2 f
PERMS = sorted(itertools.permutations(range(4)))

_rows = {}


def rows_of(r, f):
    if (r, f) not in _rows:
        _rows[(r, f)] = O.offline_rows(r, f)
    return _rows[(r, f)]


def mapping_of(row, r, f, xG, xD):
    m = O.Mapping()
    x = row
    for y in range(4):
        m.level[y] = x % 5
        x //= 5
    for q in range(4):
        m.order[q] = PERMS[x][q]
        m.xG[q], m.xD[q] = xG[q], xD[q]
    m.recompute, m.fused = r, f
    return m


def test_counts_per_group():
    """Recomputation needs a fused intermediate and j outside k: half of the orders."""
    counts = {g: (len(rows_of(*g)[0]), len(rows_of(*g)[1])) for g in GROUPS}
    assert [counts[g][0] for g in GROUPS] == [15000, 0, 15000, 7500]
    for g in GROUPS:
        valid, kept, dom = rows_of(*g)
        assert set(kept) <= set(valid) and kept == sorted(kept)
        assert all((dom[v] is None) == (v in set(kept)) for v in valid)
        assert all(dom[v] < v for v in valid if dom[v] is not None)
    print("survivors per group", {g: counts[g][1] for g in GROUPS})


def test_every_removed_row_has_an_earlier_row_no_worse_on_real_tilings():
    """Eq. (12)'s premise, checked with numbers: BS_u <= BS_v and DA_u <= DA_v for the row u
    that removes v, on seeded tilings of several shapes (boundaries of 1 included)."""
    rng = SplitMix64(0x0FF11E)
    shapes = [([48, 24, 48, 24], None), ([64, 32, 64, 32], None), ([12, 6, 30, 7], None)]
    probes = []
    for X, _ in shapes:
        for _ in range(3):
            xG = []
            for q in range(4):
                divs = [g for g in range(1, X[q] + 1) if X[q] % g == 0]
                xG.append(divs[rng.next() % len(divs)])
            probes.append((X, xG, [X[q] // xG[q] for q in range(4)]))
    hw = O.hw(HW)
    checked = 0
    for r, f in GROUPS:
        valid, kept, dom = rows_of(r, f)
        removed = [v for v in valid if dom[v] is not None]
        for v in removed[:: max(1, len(removed) // 1500)]:
            X, xG, xD = probes[(v + checked) % len(probes)]
            w = O.workload(dict(batch=1, I=X[0], K=X[1], L=X[2], J=X[3], word_bytes=2, tiling_mode=1, c_softmax=10))
            cu, _ = O.evaluate_mapping(w, hw, mapping_of(dom[v], r, f, xG, xD))
            cv, _ = O.evaluate_mapping(w, hw, mapping_of(v, r, f, xG, xD))
            assert cu.reason != 1 and cv.reason != 1
            assert cu.bs_words <= cv.bs_words and cu.da_words <= cv.da_words, (r, f, v, dom[v], xG)
            checked += 1
    assert checked > 4000


SMALL = [
    (dict(B=1, H=2, N=8, d=2, word_bytes=2, tiling_mode=1, c_softmax=10),
     dict(HW, gb_bytes=96, dram_bw=2.0, gb_bw=64.0)),
    (dict(B=1, H=1, N=6, d=3, word_bytes=2, tiling_mode=1, c_softmax=10),
     dict(pe_rows=2, pe_cols=4, n_arrays=1, rf_bytes=32, gb_bytes=120,
          e_dram=150.0, e_gb=7.0, e_rf=1.5, e_mac=0.5, dram_bw=3.0, gb_bw=16.0)),
    (dict(B=1, H=1, N=16, d=2, word_bytes=2, tiling_mode=0, c_softmax=10),
     dict(HW, gb_bytes=1 << 20, dram_bw=0.25, gb_bw=0.0)),
]


@pytest.mark.parametrize("case", range(len(SMALL)))
def test_searching_the_survivors_finds_the_optimum_of_the_whole_space(case):
    """Sec. VI-C: pruning retains every optimal solution.  Here with index ties: the lowest-index
    optimum of each objective lies in a surviving row.  The space is walked in blocks of one
    (r, s1, s2, f) digit combination = 15000 rows x all tilings."""
    wcfg, hcfg = SMALL[case]
    w, h = O.workload(wcfg), O.hw(hcfg)
    S = O.space_size(w, h)
    T = S // 540000
    n = 15000 * T
    in_group = np.arange(n) // T                     # levels and order digits of a block's candidates
    best_full, best_kept = [None] * 4, [None] * 4
    n_kept_total = 0
    for block in range(36):
        r, f = block % 2, block // 18
        c = O.eval_batch(w, h, block * n, n)
        ok = c["valid"] == 1
        E = np.where(ok, c["energy_pj"], np.inf)
        L = np.where(ok, c["latency_cycles"], np.inf)
        with np.errstate(invalid="ignore"):
            P = np.where(ok, E * L, np.inf)
        kept = np.zeros(15000, dtype=bool)
        kept[rows_of(r, f)[1]] = True
        sub = np.flatnonzero(kept[in_group])
        n_kept_total += len(sub)
        idx = np.arange(n)
        for o, keys in enumerate(((idx, E), (idx, L), (idx, E, L), (idx, P))):
            a = np.lexsort(keys)[0]
            cand = tuple(float(k[a]) for k in reversed(keys[1:])) + (block * n + int(a),)
            if np.isfinite(cand[0]) and (best_full[o] is None or cand < best_full[o]):
                best_full[o] = cand
            if len(sub):
                b = sub[np.lexsort(tuple(k[sub] for k in keys))[0]]
                cand = tuple(float(k[b]) for k in reversed(keys[1:])) + (block * n + int(b),)
                if np.isfinite(cand[0]) and (best_kept[o] is None or cand < best_kept[o]):
                    best_kept[o] = cand
    assert 0 < n_kept_total < S / 50
    assert all(v is not None for v in best_full) and best_kept == best_full
    rc, oidx, _, _, _ = O.search_all(w, h)
    assert rc == 0 and [v[-1] for v in best_full] == list(oidx)
    # and the two fronts are made of survivors only
    for rc_idx in (O.pareto(w, h), O.front_bs_da(w, h)):
        assert rc_idx[0] == 0
        for i in rc_idx[1]:
            row = i // T
            assert row % 15000 in set(rows_of((row // 15000) % 2, row // 270000)[1])


def test_no_survivor_is_beaten_by_an_earlier_row_everywhere():
    """Completeness against brute force: for every survivor v and every earlier row u of its group
    there is a tiling (of a shape whose boundaries are all different) where u is worse than v in
    buffer size or in DRAM access per operand -- otherwise v should have been removed."""
    X = [30, 42, 66, 70]
    tilings = [([X[q] // d[q] for q in range(4)], list(d)) for d in
               ((2, 3, 6, 5), (5, 2, 3, 7), (3, 7, 2, 2), (1, 1, 1, 1), (6, 6, 11, 10), (15, 21, 33, 35))]
    w, hw = O.workload(dict(batch=1, I=X[0], K=X[1], L=X[2], J=X[3], word_bytes=2, tiling_mode=1, c_softmax=10)), O.hw(HW)
    for r, f in GROUPS:
        valid, kept, _ = rows_of(r, f)
        if not valid:
            continue
        terms = {}
        for v in valid:
            per = []
            for xG, xD in tilings:
                _, d = O.evaluate_mapping(w, hw, mapping_of(v, r, f, xG, xD))
                per.append(list(d.bs) + [int(t) for t in d.tau] + [d.da[0], d.da[1], d.da[3], d.da[4], d.loads[2], d.loads[5]])
            terms[v] = np.array(per, dtype=np.int64)
        allv = np.array(valid)
        stack = np.stack([terms[v] for v in valid])             # rows x tilings x terms
        for v in kept:
            earlier = stack[allv < v]
            if len(earlier) == 0:
                continue
            no_worse_everywhere = (earlier <= terms[v][None]).all(axis=(1, 2))
            assert not no_worse_everywhere.any(), (r, f, v)
