/*
 * Offline symbolic pruning, plain reference -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Sec. VI-B prunes (loop order, buffering level) solutions inside a group by comparing
 * symbolic expressions of buffer size and DRAM access, so that the outcome holds for every
 * workload and tiling.  Here the expressions are not written down a second time: the oracle's
 * own per-candidate walk (orc_eval_mapping in oracle.c) is run once per row on a probe whose
 * four inter-tile boundaries are the distinct primes 2, 3, 5, 7 and whose tiles are single
 * elements.  Every term of the model is a product of a subset of the boundaries, so the value
 * it takes on the probe spells out which boundaries it contains, and "term of u contains no
 * boundary that the same term of v lacks" is plain divisibility.
 *
 * Rule (Eq. (12), in the form that also protects ties between equal costs): inside a group
 * (same recomputation and fusion choice; the stationary modes never enter buffer size or DRAM
 * access) row v is removed when some row u with a LOWER row number is no larger in every term:
 * each BS_X, each retention indicator tau_X, each DA_X (for the unfused intermediate: the
 * spill count and the fetch count).  Every boundary is at least 1, so u is then no larger than
 * v in buffer size and DRAM access for every tiling, and u comes first in index order.
 * The comparison is the plain O(n^2) one, row against every earlier row.
 *
 * Row number inside a group = p_A + 5 p_B + 25 p_D + 125 p_E + 625 * order rank (the digits
 * of the candidate index below r).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* mirrors of oracle.c's public structs (same translation-unit-independent layout) */
typedef struct { uint32_t batch, I, K, L, J, word_bytes, tiling_mode, c_softmax; } off_chain;
typedef struct {
    uint32_t pe_rows, pe_cols, n_arrays, rf_bytes;
    uint64_t gb_bytes;
    double e_dram, e_gb, e_rf, e_mac, dram_bw, gb_bw;
} off_hw;
typedef struct {
    uint64_t idx;
    uint32_t xG[4], xD[4];
    uint8_t order[4], level[4];
    uint8_t recompute, stat1, stat2, fused;
} off_mapping;
typedef struct {
    uint64_t bs_words, da_words, br_words, mac_total, comp_cycles;
    double energy_pj, latency_cycles;
    uint32_t valid, reason;
} off_cost;
typedef struct {
    uint64_t bs[5], loads[6], da[5];
    uint32_t tau[5];
    uint64_t bs_op1, bs_op2, br_tile1, br_tile2, cyc_tile1, cyc_tile2, rho, softmax_elems;
    uint32_t prefix_len, n1_len, n2_len;
    uint8_t prefix[4], n1[4], n2[4];
} off_detail;

int orc_eval_mapping(const off_chain *w, const off_hw *hw, const off_mapping *m, off_cost *c, off_detail *d);

#define OFF_ROWS 15000      /* 5^4 levels x 24 orders */
#define OFF_TERMS 16

typedef struct {
    int is_dataflow;
    uint64_t term[OFF_TERMS];   /* BS_A..BS_E, tau_A..tau_E (as 1 or 2), DA_A, DA_B, DA_D, DA_E, C spills, C fetches */
} off_row;

static void order_of_rank(unsigned rank, uint8_t ord[4])
{
    /* the rank-th permutation of (i,k,l,j) = (0,1,2,3) in lexicographic order, by counting */
    unsigned seen = 0;
    for (uint8_t a = 0; a < 4; ++a)
        for (uint8_t b = 0; b < 4; ++b)
            for (uint8_t c = 0; c < 4; ++c)
                for (uint8_t d = 0; d < 4; ++d) {
                    if (a == b || a == c || a == d || b == c || b == d || c == d) continue;
                    if (seen++ == rank) { ord[0] = a; ord[1] = b; ord[2] = c; ord[3] = d; return; }
                }
}

static int probe_row(unsigned row, int r, int f, off_row *out)
{
    static const uint32_t PRIME[4] = {2, 3, 5, 7};
    off_chain w = {1, 2, 3, 5, 7, 1, 1, 0};
    off_hw hw;
    memset(&hw, 0, sizeof(hw));
    hw.pe_rows = hw.pe_cols = hw.n_arrays = 1;
    hw.rf_bytes = 64;
    hw.gb_bytes = 1ull << 40;
    hw.e_dram = hw.e_gb = hw.e_rf = hw.e_mac = 1.0;
    off_mapping m;
    memset(&m, 0, sizeof(m));
    for (int q = 0; q < 4; ++q) { m.xG[q] = 1; m.xD[q] = PRIME[q]; }
    unsigned x = row;
    for (int y = 0; y < 4; ++y) { m.level[y] = (uint8_t)(x % 5); x /= 5; }
    order_of_rank(x, m.order);
    m.recompute = (uint8_t)r; m.fused = (uint8_t)f;
    off_cost c;
    off_detail d;
    if (orc_eval_mapping(&w, &hw, &m, &c, &d)) return -1;
    memset(out, 0, sizeof(*out));
    out->is_dataflow = c.reason != 1;
    if (!out->is_dataflow) return 0;
    for (int X = 0; X < 5; ++X) {
        out->term[X] = d.bs[X];
        out->term[5 + X] = d.tau[X] ? 2 : 1;
    }
    out->term[10] = d.da[0]; out->term[11] = d.da[1]; out->term[12] = d.da[3]; out->term[13] = d.da[4];
    /* unfused C: how often a tile is spilled by Op1 and fetched by Op2 (fused: no DRAM traffic) */
    out->term[14] = f ? 1 : d.loads[2];
    out->term[15] = f ? 1 : d.loads[5];
    return 0;
}

static int no_larger(const off_row *u, const off_row *v)
{
    for (int t = 0; t < OFF_TERMS; ++t)
        if (v->term[t] % u->term[t]) return 0;
    return 1;
}

/* Rows of group (r, f) that denote a dataflow, and those of them that survive the pruning, as
 * ascending row numbers.  valid_out / kept_out hold up to 15000 entries each (may be NULL).
 * dominator_out (15000 entries, may be NULL): for a removed row the lowest row that removes it,
 * 0xFFFFFFFF for every other row. */
int orc_offline_rows(int r, int f, uint32_t *valid_out, uint32_t *n_valid, uint32_t *kept_out, uint32_t *n_kept,
                     uint32_t *dominator_out)
{
    if (r < 0 || r > 1 || f < 0 || f > 1 || !n_valid || !n_kept) return -1;
    off_row *rows = (off_row *)malloc(sizeof(off_row) * OFF_ROWS);
    if (!rows) return -1;
    for (unsigned row = 0; row < OFF_ROWS; ++row)
        if (probe_row(row, r, f, &rows[row])) { free(rows); return -1; }
    uint32_t nv = 0, nk = 0;
    if (dominator_out) memset(dominator_out, 0xFF, sizeof(uint32_t) * OFF_ROWS);
    for (unsigned v = 0; v < OFF_ROWS; ++v) {
        if (!rows[v].is_dataflow) continue;
        if (valid_out) valid_out[nv] = v;
        ++nv;
        int removed = 0;
        for (unsigned u = 0; u < v && !removed; ++u)
            if (rows[u].is_dataflow && no_larger(&rows[u], &rows[v])) {
                removed = 1;
                if (dominator_out) dominator_out[v] = u;
            }
        if (!removed) {
            if (kept_out) kept_out[nk] = v;
            ++nk;
        }
    }
    free(rows);
    *n_valid = nv; *n_kept = nk;
    return 0;
}
