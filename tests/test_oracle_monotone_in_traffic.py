"""A property of the model (Sec. V) that the batched pruned search rests on, checked on the oracle
over whole small spaces: with tiling, recomputation choice, fusion choice and the two stationary
modes fixed, a candidate's energy, latency and energy-delay product never decrease when its DRAM
access grows, and whether it fits the buffer does not depend on the stationary modes.  The rows
(loop order x buffering levels) that fit therefore attain the minimum of every objective at a
row of least DRAM access -- with rounding as it is, in the oracle's own order of operations.
"""
import numpy as np
import pytest

import oracle as O

CASES = [
    # whole-number energies, power-of-two bandwidths, a buffer that cuts the space
    (dict(B=1, H=2, N=8, d=2, word_bytes=2, tiling_mode=1, c_softmax=10),
     dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=96,
          e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=2.0, gb_bw=64.0)),
    # fractional energies, other bandwidths and array count, ragged folds
    (dict(B=2, H=3, N=6, d=3, word_bytes=2, tiling_mode=1, c_softmax=3),
     dict(pe_rows=3, pe_cols=2, n_arrays=3, rf_bytes=10, gb_bytes=120,
          e_dram=187.3125, e_gb=6.75, e_rf=1.5, e_mac=0.25, dram_bw=3.0, gb_bw=5.0)),
    # latency bound by DRAM for many rows, by compute for others
    (dict(B=1, H=1, N=12, d=2, word_bytes=4, tiling_mode=1, c_softmax=0),
     dict(pe_rows=2, pe_cols=8, n_arrays=1, rf_bytes=48, gb_bytes=1 << 12,
          e_dram=100.0, e_gb=7.0, e_rf=0.0, e_mac=2.0, dram_bw=0.5, gb_bw=0.0)),
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_every_objective_is_monotone_in_dram_access(case):
    w, h = CASES[case]
    ow, oh = O.workload(w), O.hw(h)
    S = O.space_size(ow, oh)
    T = S // 540000
    block = 15000 * T                         # the rows of one (r, s1, s2, f) choice, every tiling
    fits = {}                                 # (r, f) -> which (row, tiling) fit, from the first mode pair seen
    checked = strict = 0
    for hi in range(36):                      # hi = r + 2 s1 + 6 s2 + 18 f
        r, f = hi & 1, hi // 18
        c = O.eval_batch(ow, oh, hi * block, block).reshape(15000, T)
        valid = c["valid"] == 1
        if (r, f) in fits:
            assert (valid == fits[(r, f)]).all()            # the stationary modes never decide feasibility
        else:
            fits[(r, f)] = valid
        da = np.where(valid, c["da_words"].astype(np.float64), np.inf)
        order = np.argsort(da, axis=0, kind="stable")
        da_s = np.take_along_axis(da, order, axis=0)
        both = np.isfinite(da_s[1:]) & np.isfinite(da_s[:-1])
        en = np.take_along_axis(c["energy_pj"], order, axis=0)
        lat = np.take_along_axis(c["latency_cycles"], order, axis=0)
        for key in (en, lat, en * lat):
            assert (key[1:][both] >= key[:-1][both]).all(), (case, hi)
        # the pair (latency, energy) in lexicographic order
        worse = (lat[1:] > lat[:-1]) | ((lat[1:] == lat[:-1]) & (en[1:] >= en[:-1]))
        assert worse[both].all(), (case, hi)
        # hence: the minimum over the rows that fit is the value at a row of least DRAM access
        any_fit = valid.any(axis=0)
        for key in (c["energy_pj"], c["latency_cycles"]):
            least = np.where(valid, key, np.inf).min(axis=0)
            at_least_da = np.take_along_axis(key, order[:1], axis=0)[0]
            assert (least[any_fit] == at_least_da[any_fit]).all(), (case, hi)
        checked += int(both.sum())
        strict += int((en[1:][both] > en[:-1][both]).sum())
    assert checked > 100000 and strict > 0
