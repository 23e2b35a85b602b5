"""The register file is a live capacity in the model: a PE keeps g = rf_bytes / word / 2 stationary
words (Sec. II-B hardware; Sec. V-D buffer<->register-file traffic under a stationary mode), so a
larger file folds the stationary operand fewer times and moves fewer words between buffer and
array.  Checked on the fold-by-fold enumeration and on whole small spaces of the oracle."""
import oracle as O

W = dict(B=1, H=2, N=16, d=8, word_bytes=2, tiling_mode=1, c_softmax=10)
HW = dict(pe_rows=4, pe_cols=4, n_arrays=1, rf_bytes=64, gb_bytes=2048,
          e_dram=200.0, e_gb=6.0, e_rf=1.0, e_mac=1.0, dram_bw=8.0, gb_bw=4.0)


def test_fold_enumeration_words_fall_with_the_stationary_words_per_pe():
    for mode in range(3):
        for (m, r, n, R, C) in ((24, 10, 36, 4, 4), (7, 5, 9, 3, 4), (64, 64, 64, 16, 16)):
            words = [O.sim_tile_matmul(m, r, n, mode, R, C, g)[0] for g in range(1, 40)]
            cycles = {O.sim_tile_matmul(m, r, n, mode, R, C, g)[1] for g in range(1, 40)}
            assert all(a >= b for a, b in zip(words, words[1:])) and words[0] > words[-1]
            assert len(cycles) == 1                      # the file changes traffic, not the schedule
            # once a PE row holds a whole row of the stationary operand nothing is fetched twice
            u, v, t = ((r, n, m), (m, r, n), (m, n, r))[mode]
            g_all = -(-v // C)
            assert words[g_all - 1] == words[-1] == u * v + t * u + t * v * -(-u // R)


def test_optimum_moves_with_the_register_file():
    ow = O.workload(W)
    seen = []
    for rf in (6, 8, 16, 64, 1024):
        oh = O.hw(dict(HW, rf_bytes=rf))
        rc, idx, cost, n_valid, _ = O.search_all(ow, oh)
        assert rc == 0 and n_valid > 0
        seen.append((idx[0], cost[0].energy_pj, cost[1].latency_cycles))
    energies = [s[1] for s in seen]
    latencies = [s[2] for s in seen]
    assert all(a >= b for a, b in zip(energies, energies[1:])) and energies[0] > energies[-1]
    assert all(a >= b for a, b in zip(latencies, latencies[1:])) and latencies[0] > latencies[-1]
    assert seen[0][0] != seen[-1][0]                     # another mapping wins
    assert seen[-2][:2] == seen[-1][:2]                  # beyond the tiles' width a larger file changes nothing
