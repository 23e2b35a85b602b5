/* The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): every entry
 * point once on small inputs, including the edges of its index ranges.  Built and run by
 * tests/test_oracle_sanitizers.py; exits 0 when nothing was reported and the results agree with
 * each other. */
#include <stdio.h>
#include <stdlib.h>
#include "../../oracle/oracle.c"
#include "../../oracle/sim.c"

int orc_offline_rows(int r, int f, uint32_t *valid_out, uint32_t *n_valid, uint32_t *kept_out, uint32_t *n_kept,
                     uint32_t *dominator_out);

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(void)
{
    orc_workload a = {1, 2, 12, 6, 2, 1, 10, 0};
    orc_hw hw = {3, 5, 2, 14, 400, 187.5, 6.25, 1.0, 0.5, 3.0, 5.0};
    orc_chain w;
    CHECK(orc_from_attention(&a, &w) == 0);
    uint64_t S = 0;
    CHECK(orc_space_size(&w, &hw, &S) == 0 && S == 576ull * 540000ull);

    /* windows at both ends of the space and one out of range */
    enum { WIN = 4096 };
    orc_cost *costs = (orc_cost *)malloc(sizeof(orc_cost) * WIN);
    CHECK(costs);
    CHECK(orc_eval_batch(&w, &hw, 0, WIN, costs) == 0);
    CHECK(orc_eval_batch(&w, &hw, S - WIN, WIN, costs) == 0);
    CHECK(orc_eval_batch(&w, &hw, S - WIN + 1, WIN, costs) != 0);
    orc_mapping m;
    orc_cost c;
    orc_detail d;
    CHECK(orc_decode(&w, &hw, S - 1, &m) == 0 && m.idx == S - 1);
    CHECK(orc_decode(&w, &hw, S, &m) != 0);
    CHECK(orc_eval(&w, &hw, S - 1, &m, &c, &d) == 0);
    CHECK(c.valid == costs[WIN - 1].valid && c.da_words == costs[WIN - 1].da_words);

    /* a search over a slice, one key at a time and all keys in one pass */
    const uint64_t first = 1234567, n = 3000000;
    uint64_t idx4[N_OBJ], nv = 0;
    orc_cost cost4[N_OBJ];
    int threads = 0;
    CHECK(orc_search_all(&w, &hw, first, n, idx4, cost4, &nv, &threads) == 0 && nv > 0 && threads >= 1);
    for (int o = 0; o < N_OBJ; ++o) {
        uint64_t bi = 0, nv1 = 0;
        CHECK(orc_search_range(&w, &hw, o, first, n, &bi, &c, &nv1, &threads) == 0);
        CHECK(bi == idx4[o] && nv1 == nv && c.energy_pj == cost4[o].energy_pj && c.latency_cycles == cost4[o].latency_cycles);
    }
    CHECK(orc_search_all(&w, &hw, S - 10, 11, idx4, cost4, &nv, &threads) != 0);

    /* both fronts over the slice */
    enum { CAP = 512 };
    uint64_t *fidx = (uint64_t *)malloc(sizeof(uint64_t) * CAP);
    orc_cost *fcost = (orc_cost *)malloc(sizeof(orc_cost) * CAP);
    uint32_t nf = 0;
    CHECK(fidx && fcost);
    for (int kind = 0; kind < 2; ++kind) {
        CHECK(orc_front(&w, &hw, kind, first, n, CAP, fidx, fcost, &nf) == 0 && nf >= 1 && nf <= CAP);
        for (uint32_t k = 1; k < nf; ++k)
            CHECK(kind == 0 ? fcost[k].latency_cycles > fcost[k - 1].latency_cycles : fcost[k].bs_words > fcost[k - 1].bs_words);
    }

    /* the stage-by-stage simulator and the fold enumeration */
    const uint32_t xG[4] = {2, 3, 1, 3}, xD[4] = {3, 1, 6, 1};
    for (int perm = 0; perm < 24; perm += 5)
        for (int lev = 0; lev < 625; lev += 37)
            for (int rf = 0; rf < 3; ++rf) {
                orc_mapping mm;
                memset(&mm, 0, sizeof(mm));
                CHECK(orc_decode(&w, &hw, (uint64_t)(lev + 625 * perm) * 576, &mm) == 0);
                sim_result s;
                const int r = rf == 1, f = rf != 2;
                int rc = sim_run(xG, xD, mm.order, mm.level, r, f, &s);
                CHECK(rc == 0 || r);        /* recomputation is no dataflow for some orders */
                if (rc == 0) CHECK(s.psum_violation == 0 && s.coverage_error == 0);
            }
    uint64_t words = 0, cycles = 0, macs = 0;
    for (int mode = 0; mode < 3; ++mode) {
        CHECK(sim_tile_matmul(7, 5, 9, mode, 3, 4, 2, &words, &cycles, &macs) == 0);
        CHECK(macs == 7ull * 5 * 9);
    }

    /* the plain reference of the offline pruning */
    uint32_t *valid = (uint32_t *)malloc(4 * 15000), *kept = (uint32_t *)malloc(4 * 15000), *dom = (uint32_t *)malloc(4 * 15000);
    CHECK(valid && kept && dom);
    static const uint32_t want_kept[4] = {86, 0, 74, 110};
    for (int g = 0; g < 4; ++g) {
        uint32_t n_valid = 0, n_kept = 0;
        CHECK(orc_offline_rows(g & 1, g >> 1, valid, &n_valid, kept, &n_kept, dom) == 0);
        CHECK(n_kept == want_kept[g] && n_kept <= n_valid && n_valid <= 15000);
    }
    free(valid); free(kept); free(dom); free(fidx); free(fcost); free(costs);
    printf("oracle under sanitizers: ok\n");
    return 0;
}
