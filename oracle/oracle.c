/*
 * MMEE oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, candidate-by-candidate CPU evaluation of the analytical
 * model of "Fast Cross-Operator Optimization of Attention Dataflow" (MMEE).
 * There is no matrix encoding, no table sharing between candidates and no
 * pruning here: every candidate index is decoded, its loop nest is walked
 * with ordinary loops and ifs, and the cost is formed from scratch.
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * call this file; the product path never does, and this file shares no code
 * with it.
 *
 * Notation (Sec. III-A, Sec. IV-A):
 *   Op1: C[i,l] = sum_k A[i,k] B[k,l]   (producer, Q K^T)
 *   Op2: E[i,j] = sum_l C[i,l] D[l,j]   (consumer, P V)
 *   dims are numbered i=0, k=1, l=2, j=3;  X = x_D * x_G  (inter-tile count
 *   times intra-tile size, Sec. IV-A "Loop Boundary").
 *
 * Parity pins (see tests): the closed forms printed in Sec. V-B/V-C for the
 * Fig. 11 example (buffer-size and DRAM-access estimation), the MAC and softmax counts of Sec. V-D, the compute-bound
 * latencies of Table II, the single-tile special case, and a stage-by-stage
 * loop-nest simulator (sim.c).  The GB<->RF traffic term and the unfused
 * variant are pinned by brute force (fold-by-fold enumeration of a tile matmul on
 * the PE array; the simulator's DRAM counts with C staged through DRAM).  The
 * paper prints neither a formula nor a value for these two, so what they are
 * pinned to is this build's reading of its description, not a number of the paper.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    uint32_t B, H, N, d;
    uint32_t word_bytes;
    uint32_t tiling_mode;   /* 0: power-of-two divisors, 1: all divisors */
    uint32_t c_softmax;
    uint32_t reserved;
} orc_workload;

/* Two chained matrix multiplications of free shape (Sec. VII-J: two GEMMs, or a
 * convolution chain after im2col): Op1 is I x K x L, Op2 is I x L x J, `batch`
 * independent instances.  Attention is the case I = L = N, K = J = d, batch = B*H. */
typedef struct {
    uint32_t batch, I, K, L, J;
    uint32_t word_bytes, tiling_mode, c_softmax;
} orc_chain;

typedef struct {
    uint32_t pe_rows, pe_cols, n_arrays, rf_bytes;
    uint64_t gb_bytes;
    double e_dram, e_gb, e_rf, e_mac;
    double dram_bw, gb_bw;
} orc_hw;

typedef struct {
    uint64_t idx;
    uint32_t xG[4], xD[4];      /* i,k,l,j */
    uint8_t order[4];           /* inter-tile loops, outer -> inner */
    uint8_t level[4];           /* p_A, p_B, p_D, p_E */
    uint8_t recompute, stat1, stat2, fused;
} orc_mapping;

typedef struct {
    uint64_t bs_words, da_words, br_words, mac_total, comp_cycles;
    double energy_pj, latency_cycles;
    uint32_t valid, reason;     /* reason: 0 ok, 1 not a dataflow, 2 over capacity */
} orc_cost;

/* Per-operand terms, exposed so that tests can pin them one by one. */
typedef struct {
    uint64_t bs[5];     /* BS_A, BS_B, BS_C, BS_D, BS_E (words)          */
    uint64_t loads[6];  /* A, B, C-as-Op1-output, D, E, C-as-Op2-input    */
    uint64_t da[5];     /* DA_A, DA_B, DA_C, DA_D, DA_E (words)          */
    uint32_t tau[5];    /* retention indicator (tau_C is always 0)        */
    uint64_t bs_op1, bs_op2;
    uint64_t br_tile1, br_tile2, cyc_tile1, cyc_tile2;
    uint64_t rho, softmax_elems;
    uint32_t prefix_len, n1_len, n2_len;
    uint8_t prefix[4], n1[4], n2[4];
} orc_detail;

enum { DIM_I = 0, DIM_K = 1, DIM_L = 2, DIM_J = 3 };
enum { OPD_A = 0, OPD_B = 1, OPD_C = 2, OPD_D = 3, OPD_E = 4 };
enum { OBJ_ENERGY = 0, OBJ_LATENCY = 1, OBJ_LATENCY_THEN_ENERGY = 2, OBJ_EDP = 3, N_OBJ = 4 };

/* Own dimensions of each operand (Sec. V-A, the paragraph on an operand's dimensions). */
static const int OWN[5][2] = {
    {DIM_I, DIM_K}, {DIM_K, DIM_L}, {DIM_I, DIM_L}, {DIM_L, DIM_J}, {DIM_I, DIM_J}};

/* ------------------------------------------------------------------ */
/* tiling enumeration: integer factorisation X = x_D * x_G (Sec. VI-A) */

static int list_divisors(uint32_t X, uint32_t mode, uint32_t *out, int cap)
{
    int n = 0;
    for (uint32_t g = 1; g <= X; ++g) {
        if (X % g) continue;
        if (mode == 0 && (g & (g - 1))) continue;   /* keep powers of two only */
        if (n < cap) out[n] = g;
        ++n;
    }
    return n;
}

#define MAXDIV 1536

typedef struct {
    uint32_t X[4];
    uint32_t ndiv[4];
    uint32_t div[4][MAXDIV];
    uint64_t n_tilings;
} tiling_space;

static int make_space(const orc_chain *w, tiling_space *ts)
{
    ts->X[DIM_I] = w->I; ts->X[DIM_K] = w->K; ts->X[DIM_L] = w->L; ts->X[DIM_J] = w->J;
    ts->n_tilings = 1;
    for (int q = 0; q < 4; ++q) {
        int n = list_divisors(ts->X[q], w->tiling_mode, ts->div[q], MAXDIV);
        if (n <= 0 || n > MAXDIV) return -1;
        ts->ndiv[q] = (uint32_t)n;
        ts->n_tilings *= (uint64_t)n;
    }
    return 0;
}

#define ROWS_PER_TILING 540000ull   /* 5^4 levels * 24 orders * 2 * 3 * 3 * 2 */

static int check_args(const orc_chain *w, const orc_hw *hw)
{
    if (!w || !hw) return -1;
    if (!w->batch || !w->I || !w->K || !w->L || !w->J || !w->word_bytes) return -1;
    if (w->tiling_mode > 1) return -1;
    if (!hw->pe_rows || !hw->pe_cols || !hw->n_arrays) return -1;
    if (hw->rf_bytes < 3 * w->word_bytes) return -1;
    if (!(hw->e_dram >= 0) || !(hw->e_gb >= 0) || !(hw->e_rf >= 0) || !(hw->e_mac >= 0)) return -1;
    if (!(hw->dram_bw >= 0) || !(hw->gb_bw >= 0)) return -1;
    return 0;
}

/* Attention as a chain (Sec. III-A): A = Q, B = K^T, D = V, E = O per head. */
int orc_from_attention(const orc_workload *a, orc_chain *c)
{
    if (!a || !c) return -1;
    if ((uint64_t)a->B * a->H > 0xffffffffull) return -1;
    c->batch = a->B * a->H;
    c->I = a->N; c->K = a->d; c->L = a->N; c->J = a->d;
    c->word_bytes = a->word_bytes; c->tiling_mode = a->tiling_mode; c->c_softmax = a->c_softmax;
    return 0;
}

int orc_space_size(const orc_chain *w, const orc_hw *hw, uint64_t *out)
{
    tiling_space ts;
    if (check_args(w, hw) || !out) return -1;
    if (make_space(w, &ts)) return -1;
    *out = ts.n_tilings * ROWS_PER_TILING;
    return 0;
}

/* ------------------------------------------------------------------ */
/* index -> candidate tuple.  Digits, least significant first:
 *   t_i t_k t_l t_j | p_A p_B p_D p_E | order rank | r | s1 | s2 | f       */

static void unrank_order(unsigned rank, uint8_t ord[4])
{
    /* lexicographic rank of the outer->inner sequence over i<k<l<j */
    int avail[4] = {0, 1, 2, 3};
    int n = 4;
    unsigned fact[4] = {6, 2, 1, 1};
    for (int a = 0; a < 4; ++a) {
        unsigned pick = rank / fact[a];
        rank %= fact[a];
        ord[a] = (uint8_t)avail[pick];
        for (int b = (int)pick; b < n - 1; ++b) avail[b] = avail[b + 1];
        --n;
    }
}

static int decode_idx(const tiling_space *ts, uint64_t idx, orc_mapping *m)
{
    if (idx >= ts->n_tilings * ROWS_PER_TILING) return -2;
    m->idx = idx;
    for (int q = 0; q < 4; ++q) {
        uint32_t t = (uint32_t)(idx % ts->ndiv[q]);
        idx /= ts->ndiv[q];
        m->xG[q] = ts->div[q][t];
        m->xD[q] = ts->X[q] / m->xG[q];
    }
    for (int x = 0; x < 4; ++x) { m->level[x] = (uint8_t)(idx % 5); idx /= 5; }
    unrank_order((unsigned)(idx % 24), m->order); idx /= 24;
    m->recompute = (uint8_t)(idx % 2); idx /= 2;
    m->stat1 = (uint8_t)(idx % 3); idx /= 3;
    m->stat2 = (uint8_t)(idx % 3); idx /= 3;
    m->fused = (uint8_t)(idx % 2);
    return 0;
}

int orc_decode(const orc_chain *w, const orc_hw *hw, uint64_t idx, orc_mapping *out)
{
    tiling_space ts;
    if (check_args(w, hw) || !out) return -1;
    if (make_space(w, &ts)) return -1;
    return decode_idx(&ts, idx, out);
}

/* ------------------------------------------------------------------ */
/* the model for one candidate                                         */

static uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

/* Number of times the buffered block of an operand is (re)filled.
 * nest: the operand's operator loop nest, outer -> inner.
 * The blocker is the innermost loop outside the buffering level whose
 * iteration changes the buffered data (Sec. V-A "Blocker").
 *  - blocker is one of the loops that both operators share and the operand is
 *    not retained: the operator switch evicts it once per iteration of the
 *    shared loops (the Scenario 2 situation of Sec. V-C: the boundary of the
 *    loop that forces the switch is not a factor);
 *  - otherwise Scenario 1: blocker boundary times every loop above it.      */
static uint64_t refills(const uint8_t *nest, int nlen, const int own[2], int level,
                        int tau, const int pos[4], const int in_prefix[4],
                        const uint8_t *prefix, int prefix_len, const uint32_t xD[4])
{
    int b = -1;
    for (int a = nlen - 1; a >= 0; --a) {
        int q = nest[a];
        if ((q == own[0] || q == own[1]) && pos[q] >= level) { b = a; break; }
    }
    if (b < 0) return 1;
    uint64_t n = 1;
    if (!tau && in_prefix[nest[b]]) {
        for (int a = 0; a < prefix_len; ++a) n *= xD[prefix[a]];
    } else {
        for (int a = 0; a <= b; ++a) n *= xD[nest[a]];
    }
    return n;
}

/* GB<->RF words and cycles of one tile-level matmul m x r x n on an R x C
 * array under a stationary mode (0 WS, 1 IS, 2 OS).  The mode fixes which two
 * dims are spread over rows/columns (u, v) and which is streamed in time (t). */
static void tile_matmul(uint64_t m, uint64_t r, uint64_t n, int mode,
                        uint64_t R, uint64_t C, uint64_t g,
                        uint64_t *words, uint64_t *cycles)
{
    uint64_t u, v, t;
    if (mode == 0)      { u = r; v = n; t = m; }   /* weight stationary */
    else if (mode == 1) { u = m; v = r; t = n; }   /* input stationary  */
    else                { u = m; v = n; t = r; }   /* output stationary */
    uint64_t stationary = u * v;
    uint64_t stream_tu = t * u * ceil_div(v, C * g);
    uint64_t stream_tv = t * v * ceil_div(u, R);
    *words = stationary + stream_tu + stream_tv;
    *cycles = ceil_div(u, R) * ceil_div(v, C) * t;
}

static void eval_mapping(const orc_chain *w, const orc_hw *hw, const tiling_space *ts,
                         const orc_mapping *m, orc_cost *c, orc_detail *dt)
{
    orc_detail local;
    if (!dt) dt = &local;
    memset(dt, 0, sizeof(*dt));
    memset(c, 0, sizeof(*c));

    const uint32_t *xG = m->xG, *xD = m->xD;
    const int r = m->recompute, f = m->fused;

    /* position of each inter-tile loop, 0 = innermost (Sec. IV-A) */
    int pos[4];
    for (int a = 0; a < 4; ++a) pos[m->order[a]] = 3 - a;

    /* Not a dataflow: recomputation asked for but the order never revisits a
     * C tile (k outside j), or recomputation of an intermediate that lives in
     * DRAM anyway. */
    if (r && (!f || pos[DIM_K] > pos[DIM_J])) {
        c->valid = 0; c->reason = 1;
        c->energy_pj = INFINITY; c->latency_cycles = INFINITY;
        return;
    }

    /* Region program (Sec. IV-B): loops shared by both operators lead; below
     * them the producer runs its remaining loops to completion (no partial
     * sums cross, Sec. III-C), softmax, then the consumer runs its own.      */
    int shared[4] = {1, 0, 1, r ? 1 : 0};
    int in_prefix[4] = {0, 0, 0, 0};
    int plen = 0;
    while (plen < 4 && shared[m->order[plen]]) { in_prefix[m->order[plen]] = 1; ++plen; }
    int n1 = 0, n2 = 0;
    for (int a = 0; a < 4; ++a) {
        int q = m->order[a];
        dt->prefix[a] = (a < plen) ? (uint8_t)q : 0;
        if (a < plen || q == DIM_I || q == DIM_K || q == DIM_L) dt->n1[n1++] = (uint8_t)q;
        if (a < plen || q == DIM_I || q == DIM_L || q == DIM_J) dt->n2[n2++] = (uint8_t)q;
    }
    dt->prefix_len = (uint32_t)plen; dt->n1_len = (uint32_t)n1; dt->n2_len = (uint32_t)n2;

    /* tile footprints */
    uint64_t tile[5];
    for (int x = 0; x < 5; ++x) tile[x] = (uint64_t)xG[OWN[x][0]] * xG[OWN[x][1]];

    /* Operand buffer size: product of the boundaries of its own dimensional
     * loops at and below its buffering level (Sec. V-B). */
    int level[5] = {m->level[0], m->level[1], 0, m->level[2], m->level[3]};
    for (int x = 0; x < 5; ++x) {
        if (x == OPD_C) continue;
        uint64_t bs = tile[x];
        for (int e = 0; e < 2; ++e) {
            int q = OWN[x][e];
            if (pos[q] < level[x]) bs *= xD[q];
        }
        dt->bs[x] = bs;
        dt->tau[x] = level[x] >= 1;   /* buffered at an inter-tile loop */
    }
    /* C never leaves the chip when fused, so it must hold every tile the
     * producer finishes before the consumer starts: all its own loops that are
     * not shared.  Unfused, C is staged one tile at a time. */
    {
        uint64_t bs = tile[OPD_C];
        if (f) {
            if (!in_prefix[DIM_I]) bs *= xD[DIM_I];
            if (!in_prefix[DIM_L]) bs *= xD[DIM_L];
        }
        dt->bs[OPD_C] = bs;
        dt->tau[OPD_C] = 0;
    }

    /* Operator and overall buffer size, Eq. (1), (2), (4). */
    dt->bs_op1 = dt->bs[OPD_A] + dt->bs[OPD_B] + dt->bs[OPD_C]
               + dt->tau[OPD_D] * dt->bs[OPD_D] + dt->tau[OPD_E] * dt->bs[OPD_E];
    dt->bs_op2 = dt->bs[OPD_C] + dt->bs[OPD_D] + dt->bs[OPD_E]
               + dt->tau[OPD_A] * dt->bs[OPD_A] + dt->tau[OPD_B] * dt->bs[OPD_B];
    uint64_t BS = dt->bs_op1 > dt->bs_op2 ? dt->bs_op1 : dt->bs_op2;

    /* DRAM access per operand = buffer size x number of refills (Sec. V-C). */
    dt->loads[0] = refills(dt->n1, n1, OWN[OPD_A], level[OPD_A], (int)dt->tau[OPD_A], pos, in_prefix, dt->prefix, plen, xD);
    dt->loads[1] = refills(dt->n1, n1, OWN[OPD_B], level[OPD_B], (int)dt->tau[OPD_B], pos, in_prefix, dt->prefix, plen, xD);
    dt->loads[3] = refills(dt->n2, n2, OWN[OPD_D], level[OPD_D], (int)dt->tau[OPD_D], pos, in_prefix, dt->prefix, plen, xD);
    dt->loads[4] = refills(dt->n2, n2, OWN[OPD_E], level[OPD_E], (int)dt->tau[OPD_E], pos, in_prefix, dt->prefix, plen, xD);
    dt->da[OPD_A] = dt->bs[OPD_A] * dt->loads[0];
    dt->da[OPD_B] = dt->bs[OPD_B] * dt->loads[1];
    dt->da[OPD_D] = dt->bs[OPD_D] * dt->loads[3];
    dt->da[OPD_E] = dt->bs[OPD_E] * dt->loads[4];
    if (f) {
        dt->da[OPD_C] = 0;                    /* DA_C = 0, Sec. V-C */
    } else {
        /* Unfused: C is a tile-level DRAM operand of both operators, plus one
         * stand-alone softmax pass that reads S and writes P. */
        dt->loads[2] = refills(dt->n1, n1, OWN[OPD_C], 0, 0, pos, in_prefix, dt->prefix, plen, xD);
        dt->loads[5] = refills(dt->n2, n2, OWN[OPD_C], 0, 0, pos, in_prefix, dt->prefix, plen, xD);
        uint64_t IL = (uint64_t)ts->X[DIM_I] * ts->X[DIM_L];
        dt->da[OPD_C] = tile[OPD_C] * dt->loads[2] + tile[OPD_C] * dt->loads[5] + 2 * IL;
    }
    uint64_t DA = dt->da[OPD_A] + dt->da[OPD_B] + dt->da[OPD_D] + dt->da[OPD_E] + dt->da[OPD_C];  /* Eq. (7) */

    /* Recomputation multiplies the producer's work by j_D (Sec. V-D). */
    uint64_t rho = r ? xD[DIM_J] : 1;
    dt->rho = rho;
    uint64_t I = ts->X[DIM_I], K = ts->X[DIM_K], L = ts->X[DIM_L], J = ts->X[DIM_J];
    uint64_t MAC = rho * I * K * L + I * L * J;
    uint64_t SM = rho * I * L;
    dt->softmax_elems = SM;

    /* Buffer <-> register-file traffic and compute cycles, per stationary mode. */
    uint64_t R = hw->pe_rows, Cc = hw->pe_cols;
    uint64_t g = (uint64_t)hw->rf_bytes / w->word_bytes / 2;
    tile_matmul(xG[DIM_I], xG[DIM_K], xG[DIM_L], m->stat1, R, Cc, g, &dt->br_tile1, &dt->cyc_tile1);
    tile_matmul(xG[DIM_I], xG[DIM_L], xG[DIM_J], m->stat2, R, Cc, g, &dt->br_tile2, &dt->cyc_tile2);
    uint64_t stages1 = rho * xD[DIM_I] * xD[DIM_K] * xD[DIM_L];
    uint64_t stages2 = (uint64_t)xD[DIM_I] * xD[DIM_L] * xD[DIM_J];
    uint64_t BR = stages1 * dt->br_tile1 + stages2 * dt->br_tile2;
    uint64_t comp = stages1 * dt->cyc_tile1 + stages2 * dt->cyc_tile2;

    c->bs_words = BS; c->da_words = DA; c->br_words = BR;
    c->mac_total = MAC; c->comp_cycles = comp;

    /* capacity constraint */
    if (BS * (uint64_t)w->word_bytes > hw->gb_bytes) {
        c->valid = 0; c->reason = 2;
        c->energy_pj = INFINITY; c->latency_cycles = INFINITY;
        return;
    }

    /* Energy: DRAM<->buffer, buffer<->RF, RF<->MAC and compute (Sec. V-D);
     * softmax costs c_softmax per element of C produced.  All heads. */
    uint64_t BH = w->batch;
    uint64_t T_dram = BH * DA;
    uint64_t T_gb = BH * (DA + BR);
    uint64_t T_rf = BH * 3 * MAC;
    uint64_t T_mac = BH * (MAC + (uint64_t)w->c_softmax * SM);
    double e = hw->e_dram * (double)T_dram;
    e = e + hw->e_gb * (double)T_gb;
    e = e + hw->e_rf * (double)T_rf;
    e = e + hw->e_mac * (double)T_mac;
    c->energy_pj = e;

    /* Latency: load/compute/store fully pipelined, so the slowest of the
     * three streams sets the pace (Sec. V-D); softmax hides behind the tile
     * pipeline.  Heads are spread over the arrays. */
    double t_comp = (double)comp;
    double t_dram = hw->dram_bw > 0 ? (double)(DA * (uint64_t)w->word_bytes) / hw->dram_bw : 0.0;
    double t_gb = hw->gb_bw > 0 ? (double)(BR * (uint64_t)w->word_bytes) / hw->gb_bw : 0.0;
    double per_head = fmax(fmax(t_comp, t_dram), t_gb);
    c->latency_cycles = ((double)BH / (double)hw->n_arrays) * per_head;
    c->valid = 1; c->reason = 0;
}

int orc_eval(const orc_chain *w, const orc_hw *hw, uint64_t idx,
             orc_mapping *map_out, orc_cost *cost_out, orc_detail *detail_out)
{
    tiling_space ts;
    orc_mapping m;
    orc_cost c;
    if (check_args(w, hw)) return -1;
    if (make_space(w, &ts)) return -1;
    int rc = decode_idx(&ts, idx, &m);
    if (rc) return rc;
    eval_mapping(w, hw, &ts, &m, &c, detail_out);
    if (map_out) *map_out = m;
    if (cost_out) *cost_out = c;
    return 0;
}

/* Evaluate an explicit tuple (used by tests that build the Fig. 11 example
 * directly from its description instead of from an index). */
int orc_eval_mapping(const orc_chain *w, const orc_hw *hw, const orc_mapping *m,
                     orc_cost *cost_out, orc_detail *detail_out)
{
    tiling_space ts;
    orc_cost c;
    if (check_args(w, hw) || !m) return -1;
    if (make_space(w, &ts)) return -1;
    for (int q = 0; q < 4; ++q)
        if (!m->xG[q] || (uint64_t)m->xG[q] * m->xD[q] != ts.X[q]) return -1;
    eval_mapping(w, hw, &ts, m, &c, detail_out);
    if (cost_out) *cost_out = c;
    return 0;
}

int orc_eval_batch(const orc_chain *w, const orc_hw *hw, uint64_t first_idx,
                   uint64_t n, orc_cost *out)
{
    tiling_space ts;
    if (check_args(w, hw) || (n && !out)) return -1;
    if (make_space(w, &ts)) return -1;
    uint64_t S = ts.n_tilings * ROWS_PER_TILING;
    if (first_idx > S || n > S - first_idx) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < (int64_t)n; ++a) {
        orc_mapping m;
        decode_idx(&ts, first_idx + (uint64_t)a, &m);
        eval_mapping(w, hw, &ts, &m, &out[a], 0);
    }
    return 0;
}

/* lexicographic objective key, lowest index wins ties */
static int better(int objective, const orc_cost *a, uint64_t ia, const orc_cost *b, uint64_t ib)
{
    double pa, pb, sa = 0, sb = 0;
    if (objective == OBJ_ENERGY) { pa = a->energy_pj; pb = b->energy_pj; }
    else if (objective == OBJ_EDP) {       /* energy-delay product (Sec. VII-K) */
        pa = a->energy_pj * a->latency_cycles; pb = b->energy_pj * b->latency_cycles;
    }
    else { pa = a->latency_cycles; pb = b->latency_cycles; }
    if (objective == OBJ_LATENCY_THEN_ENERGY) { sa = a->energy_pj; sb = b->energy_pj; }
    if (pa != pb) return pa < pb;
    if (sa != sb) return sa < sb;
    return ia < ib;
}

/* Exhaustive search over [first_idx, first_idx + n): evaluate every candidate,
 * keep the minimum.  Returns 0, -3 when no candidate in the range is feasible. */
int orc_search_range(const orc_chain *w, const orc_hw *hw, int objective,
                     uint64_t first_idx, uint64_t n,
                     uint64_t *best_idx, orc_cost *best_cost, uint64_t *n_valid, int *threads_used)
{
    tiling_space ts;
    if (check_args(w, hw) || !best_idx || !best_cost) return -1;
    if (objective < 0 || objective >= N_OBJ) return -1;
    if (make_space(w, &ts)) return -1;
    uint64_t S = ts.n_tilings * ROWS_PER_TILING;
    if (first_idx > S || n > S - first_idx) return -2;

    int have = 0;
    uint64_t gidx = 0, gvalid = 0;
    orc_cost gcost;
    memset(&gcost, 0, sizeof(gcost));
    int nthreads = 1;
    const uint64_t CH = 1u << 16;
    int64_t nchunks = (int64_t)((n + CH - 1) / CH);
#pragma omp parallel
    {
        int lhave = 0;
        uint64_t lidx = 0, lvalid = 0;
        orc_cost lcost;
        memset(&lcost, 0, sizeof(lcost));
#ifdef _OPENMP
#pragma omp single
        nthreads = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1)
        for (int64_t ch = 0; ch < nchunks; ++ch) {
            uint64_t lo = first_idx + (uint64_t)ch * CH;
            uint64_t hi = lo + CH;
            if (hi > first_idx + n) hi = first_idx + n;
            for (uint64_t idx = lo; idx < hi; ++idx) {
                orc_mapping m;
                orc_cost c;
                decode_idx(&ts, idx, &m);
                eval_mapping(w, hw, &ts, &m, &c, 0);
                if (!c.valid) continue;
                ++lvalid;
                if (!lhave || better(objective, &c, idx, &lcost, lidx)) { lhave = 1; lcost = c; lidx = idx; }
            }
        }
#pragma omp critical
        {
            gvalid += lvalid;
            if (lhave && (!have || better(objective, &lcost, lidx, &gcost, gidx))) { have = 1; gcost = lcost; gidx = lidx; }
        }
    }
    if (threads_used) *threads_used = nthreads;
    if (n_valid) *n_valid = gvalid;
    if (!have) { best_cost->valid = 0; return -3; }
    *best_idx = gidx; *best_cost = gcost;
    return 0;
}

/* One pass over [first_idx, first_idx + n) keeping the minimum for each of the
 * four objectives at once (slot = objective code). */
int orc_search_all(const orc_chain *w, const orc_hw *hw, uint64_t first_idx, uint64_t n,
                   uint64_t best_idx[N_OBJ], orc_cost best_cost[N_OBJ], uint64_t *n_valid, int *threads_used)
{
    tiling_space ts;
    if (check_args(w, hw) || !best_idx || !best_cost) return -1;
    if (make_space(w, &ts)) return -1;
    uint64_t S = ts.n_tilings * ROWS_PER_TILING;
    if (first_idx > S || n > S - first_idx) return -2;
    int have = 0, nthreads = 1;
    uint64_t gidx[N_OBJ] = {0, 0, 0, 0}, gvalid = 0;
    orc_cost gcost[N_OBJ];
    memset(gcost, 0, sizeof(gcost));
    const uint64_t CH = 1u << 16;
    int64_t nchunks = (int64_t)((n + CH - 1) / CH);
#pragma omp parallel
    {
        int lhave = 0;
        uint64_t lidx[N_OBJ] = {0, 0, 0, 0}, lvalid = 0;
        orc_cost lcost[N_OBJ];
        memset(lcost, 0, sizeof(lcost));
#ifdef _OPENMP
#pragma omp single
        nthreads = omp_get_num_threads();
#endif
#pragma omp for schedule(dynamic, 1)
        for (int64_t ch = 0; ch < nchunks; ++ch) {
            uint64_t lo = first_idx + (uint64_t)ch * CH;
            uint64_t hi = lo + CH;
            if (hi > first_idx + n) hi = first_idx + n;
            for (uint64_t idx = lo; idx < hi; ++idx) {
                orc_mapping m;
                orc_cost c;
                decode_idx(&ts, idx, &m);
                eval_mapping(w, hw, &ts, &m, &c, 0);
                if (!c.valid) continue;
                ++lvalid;
                for (int o = 0; o < N_OBJ; ++o)
                    if (!lhave || better(o, &c, idx, &lcost[o], lidx[o])) { lcost[o] = c; lidx[o] = idx; }
                lhave = 1;
            }
        }
#pragma omp critical
        {
            gvalid += lvalid;
            if (lhave) {
                for (int o = 0; o < N_OBJ; ++o)
                    if (!have || better(o, &lcost[o], lidx[o], &gcost[o], gidx[o])) { gcost[o] = lcost[o]; gidx[o] = lidx[o]; }
                have = 1;
            }
        }
    }
    if (threads_used) *threads_used = nthreads;
    if (n_valid) *n_valid = gvalid;
    if (!have) { for (int o = 0; o < N_OBJ; ++o) best_cost[o].valid = 0; return -3; }
    for (int o = 0; o < N_OBJ; ++o) { best_idx[o] = gidx[o]; best_cost[o] = gcost[o]; }
    return 0;
}

/* Energy-latency Pareto front (Sec. VI-A, Sec. VII-E): the feasible candidates that no other
 * candidate beats in both metrics.  Among candidates with identical (energy, latency) the lowest
 * index stands for all.  Points come out by ascending latency (so descending energy).
 * One plain pass: every candidate is checked against the current front.
 * Returns 0, -3 when nothing is feasible, -5 when the front outgrows `capacity`. */
typedef struct { double e, l; uint64_t idx; } front_pt;

static int front_insert(front_pt *f, int *n, int cap, double e, double l, uint64_t idx)
{
    /* dominated by (or equal to, with a lower index than) a point already there? */
    for (int a = 0; a < *n; ++a) {
        if (f[a].e <= e && f[a].l <= l) {
            if (f[a].e == e && f[a].l == l) { if (idx < f[a].idx) f[a].idx = idx; }
            return 0;
        }
    }
    /* it stays: drop what it dominates */
    int m = 0;
    for (int a = 0; a < *n; ++a)
        if (!(e <= f[a].e && l <= f[a].l)) f[m++] = f[a];
    if (m >= cap) return -5;
    f[m].e = e; f[m].l = l; f[m].idx = idx;
    *n = m + 1;
    return 0;
}

/* kind 0: (energy, latency) over the feasible candidates, listed by ascending latency.
 * kind 1: (DRAM access, buffer size requirement) over every candidate that denotes a dataflow,
 *         whatever the buffer capacity (the DRAM-access-versus-buffer-size curve of Sec. VII-C),
 *         listed by ascending buffer size. */
int orc_front(const orc_chain *w, const orc_hw *hw, int kind, uint64_t first_idx, uint64_t n, uint32_t capacity,
              uint64_t *idx_out, orc_cost *cost_out, uint32_t *n_out)
{
    tiling_space ts;
    if (check_args(w, hw) || !idx_out || !cost_out || !n_out || !capacity || capacity > 4096) return -1;
    if (kind < 0 || kind > 1) return -1;
    if (make_space(w, &ts)) return -1;
    uint64_t S = ts.n_tilings * ROWS_PER_TILING;
    if (first_idx > S || n > S - first_idx) return -2;
    front_pt global[4096];
    int ng = 0, overflow = 0;
    const uint64_t CH = 1u << 16;
    int64_t nchunks = (int64_t)((n + CH - 1) / CH);
#pragma omp parallel
    {
        front_pt local[4096];
        int nl = 0, bad = 0;
#pragma omp for schedule(dynamic, 1)
        for (int64_t ch = 0; ch < nchunks; ++ch) {
            uint64_t lo = first_idx + (uint64_t)ch * CH;
            uint64_t hi = lo + CH;
            if (hi > first_idx + n) hi = first_idx + n;
            for (uint64_t idx = lo; idx < hi; ++idx) {
                orc_mapping m;
                orc_cost c;
                decode_idx(&ts, idx, &m);
                eval_mapping(w, hw, &ts, &m, &c, 0);
                if (kind == 0) {
                    if (!c.valid) continue;
                    if (front_insert(local, &nl, 4096, c.energy_pj, c.latency_cycles, idx)) bad = 1;
                } else {
                    if (c.reason == 1) continue;
                    if (front_insert(local, &nl, 4096, (double)c.da_words, (double)c.bs_words, idx)) bad = 1;
                }
            }
        }
#pragma omp critical
        {
            if (bad) overflow = 1;
            for (int a = 0; a < nl; ++a)
                if (front_insert(global, &ng, 4096, local[a].e, local[a].l, local[a].idx)) overflow = 1;
        }
    }
    if (overflow || (uint32_t)ng > capacity) return -5;
    if (!ng) { *n_out = 0; return -3; }
    /* ascending latency (kind 0) / buffer size (kind 1) */
    for (int a = 1; a < ng; ++a) {
        front_pt key = global[a];
        int b = a - 1;
        while (b >= 0 && global[b].l > key.l) { global[b + 1] = global[b]; --b; }
        global[b + 1] = key;
    }
    for (int a = 0; a < ng; ++a) {
        orc_mapping m;
        idx_out[a] = global[a].idx;
        decode_idx(&ts, global[a].idx, &m);
        eval_mapping(w, hw, &ts, &m, &cost_out[a], 0);
    }
    *n_out = (uint32_t)ng;
    return 0;
}

int orc_pareto(const orc_chain *w, const orc_hw *hw, uint64_t first_idx, uint64_t n, uint32_t capacity,
               uint64_t *idx_out, orc_cost *cost_out, uint32_t *n_out)
{
    return orc_front(w, hw, 0, first_idx, n, capacity, idx_out, cost_out, n_out);
}

int orc_search(const orc_chain *w, const orc_hw *hw, int objective,
               uint64_t *best_idx, orc_cost *best_cost, uint64_t *n_valid, int *threads_used)
{
    uint64_t S;
    int rc = orc_space_size(w, hw, &S);
    if (rc) return rc;
    return orc_search_range(w, hw, objective, 0, S, best_idx, best_cost, n_valid, threads_used);
}
