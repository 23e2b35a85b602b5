/* A plain C program that uses the library through include/mmee.h only: no Python, no torch.
 * Prints one line per call in a fixed format that tests/test_gpu_c_client.py compares with the
 * oracle.  Usage: abi_client B H N d word tiling_mode c_softmax pe_rows pe_cols n_arrays rf gb
 *                            e_dram e_gb e_rf e_mac dram_bw gb_bw first_idx n */
#include <inttypes.h>
#include <stdio.h>
#include <stdlib.h>

#include "mmee.h"

int main(int argc, char **argv)
{
    if (argc != 21) { fprintf(stderr, "expected 20 arguments\n"); return 2; }
    mmee_workload w = {0};
    mmee_hw h = {0};
    w.B = (uint32_t)atol(argv[1]); w.H = (uint32_t)atol(argv[2]); w.N = (uint32_t)atol(argv[3]);
    w.d = (uint32_t)atol(argv[4]); w.word_bytes = (uint32_t)atol(argv[5]);
    w.tiling_mode = (uint32_t)atol(argv[6]); w.c_softmax = (uint32_t)atol(argv[7]);
    h.pe_rows = (uint32_t)atol(argv[8]); h.pe_cols = (uint32_t)atol(argv[9]); h.n_arrays = (uint32_t)atol(argv[10]);
    h.rf_bytes = (uint32_t)atol(argv[11]); h.gb_bytes = (uint64_t)atoll(argv[12]);
    h.e_dram = atof(argv[13]); h.e_gb = atof(argv[14]); h.e_rf = atof(argv[15]); h.e_mac = atof(argv[16]);
    h.dram_bw = atof(argv[17]); h.gb_bw = atof(argv[18]);
    const uint64_t first = (uint64_t)atoll(argv[19]), n = (uint64_t)atoll(argv[20]);

    uint64_t space = 0;
    int rc = mmee_space_size(&w, &h, &space);
    if (rc) { fprintf(stderr, "mmee_space_size: %s\n", mmee_strerror(rc)); return 1; }
    printf("space %" PRIu64 "\n", space);

    mmee_cost *costs = (mmee_cost *)malloc(sizeof(mmee_cost) * n);
    if (!costs) return 1;
    rc = mmee_eval_batch(&w, &h, first, n, costs);
    if (rc) { fprintf(stderr, "mmee_eval_batch: %s\n", mmee_strerror(rc)); return 1; }
    for (uint64_t a = 0; a < n; ++a)
        printf("cost %" PRIu64 " %" PRIu64 " %" PRIu64 " %" PRIu64 " %" PRIu64 " %" PRIu64 " %a %a %u %u\n", first + a,
               costs[a].bs_words, costs[a].da_words, costs[a].br_words, costs[a].mac_total, costs[a].comp_cycles,
               costs[a].energy_pj, costs[a].latency_cycles, costs[a].valid, costs[a].reason);
    free(costs);

    for (int objective = 0; objective < 4; ++objective) {
        mmee_result pruned, full;
        rc = mmee_search(&w, &h, objective, &pruned);
        if (rc) { fprintf(stderr, "mmee_search: %s\n", mmee_strerror(rc)); return 1; }
        rc = mmee_search_ex(&w, &h, objective, MMEE_SEARCH_EXHAUSTIVE, &full);
        if (rc) { fprintf(stderr, "mmee_search_ex: %s\n", mmee_strerror(rc)); return 1; }
        if (pruned.best.idx != full.best.idx) { fprintf(stderr, "pruned and exhaustive disagree\n"); return 1; }
        printf("best %d %" PRIu64 " %a %a xG %u %u %u %u order %u%u%u%u level %u%u%u%u r %u s %u %u f %u\n", objective,
               full.best.idx, full.cost.energy_pj, full.cost.latency_cycles, full.best.xG[0], full.best.xG[1],
               full.best.xG[2], full.best.xG[3], full.best.order[0], full.best.order[1], full.best.order[2],
               full.best.order[3], full.best.level[0], full.best.level[1], full.best.level[2], full.best.level[3],
               full.best.recompute, full.best.stat1, full.best.stat2, full.best.fused);
    }
    mmee_shutdown();
    return 0;
}
