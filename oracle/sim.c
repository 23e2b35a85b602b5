/*
 * Brute-force loop-nest simulator -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Executes a fused (or unfused) two-operator dataflow stage by stage on a
 * tiny shape and counts what actually happens: which tiles sit in the on-chip
 * buffer, how many words cross the DRAM boundary, how many MACs run.  It uses
 * no closed form of the analytical model; it exists to pin the oracle's
 * closed forms (oracle.c), with which it shares no code.
 *
 * One compute stage = the multiplication of one pair of tiles (Sec. III-B,
 * Fig. 5).  Data moves at tile granularity.  A buffered block of an operand
 * is the set of its tiles spanned by its own inter-tile loops below the
 * buffering level; it is filled tile by tile as the tiles are first used and
 * is thrown away when a stage needs a tile outside it (Sec. IV-B, buffer-utilisation chart of Fig. 10).
 * Operands whose buffering level is the tile itself are released when the
 * other operator takes over; operands buffered at an inter-tile loop are
 * retained (Sec. III-D, Sec. IV-A "Buffering Level").
 *
 * Three occupancy counts come out.  `max_occupancy` counts the words really
 * resident at each stage (blocks fill tile by tile, as in the chart of Fig. 10).
 * The two reservation counts follow the rule of Sec. IV-A that an operand
 * buffered at an inter-tile loop gets a space equal to its footprint, allocated
 * and retained: the footprint of such an operand is MEASURED as the largest fill
 * its block ever reaches during the run (no closed form), and that space counts
 * in full either from the start to the end of the run (`max_reserved`, static
 * allocation) or from the block's first use on (`max_reserved_touch`).  Operands
 * at tile level and the intermediate C count as they are resident in all three.
 */
#include <stdint.h>
#include <string.h>

enum { SI = 0, SK = 1, SL = 2, SJ = 3 };
#define SIM_MAX_D 16            /* largest inter-tile count per dimension */
#define SIM_TRACE 64

typedef struct {
    uint64_t da[5];             /* words moved DRAM<->buffer for A,B,C,D,E */
    uint64_t max_occupancy;     /* peak words resident over all stages     */
    uint64_t max_reserved;      /* peak with retained operands' measured footprints reserved throughout */
    uint64_t max_reserved_touch;/* the same, each footprint reserved from its block's first use on      */
    uint64_t footprint[5];      /* largest fill of each operand's block (A,B,C,D,E), words              */
    uint64_t n_regions;         /* iterations of the loops shared by both operators                      */
    uint64_t macs1, macs2;      /* MACs executed by Op1 and Op2            */
    uint64_t softmax_elems;     /* elements of C sent through softmax      */
    uint64_t stages1, stages2;  /* tile-pair multiplications               */
    uint64_t n_stages;          /* all stages incl. softmax                */
    uint32_t occ_trace[SIM_TRACE];  /* occupancy in tiles*tile_words per stage (first 64) */
    int32_t psum_violation;     /* consumer saw an unfinished C tile       */
    int32_t coverage_error;     /* some (i,l,j) product missing or doubled */
} sim_result;

typedef struct {
    int d0, d1;                 /* own dims                                */
    int level;                  /* buffering level: # innermost loops spanned */
    int in_tag[2];              /* own dim e is part of the block tag      */
    int resident;
    int tag[2];
    uint8_t have[SIM_MAX_D][SIM_MAX_D];
    uint64_t tile_words;
    uint64_t occ;               /* words currently resident                */
    uint64_t peak;              /* largest occ so far                      */
    uint64_t moved;             /* words moved over the DRAM boundary      */
} sim_operand;

static void opd_init(sim_operand *o, int d0, int d1, int level, const int pos[4], uint64_t tile_words)
{
    memset(o, 0, sizeof(*o));
    o->d0 = d0; o->d1 = d1; o->level = level; o->tile_words = tile_words;
    o->in_tag[0] = pos[d0] >= level;
    o->in_tag[1] = pos[d1] >= level;
}

static void opd_drop(sim_operand *o)
{
    o->resident = 0; o->occ = 0;
    memset(o->have, 0, sizeof(o->have));
}

static void opd_touch(sim_operand *o, const int v[4])
{
    int c0 = v[o->d0], c1 = v[o->d1];
    int t0 = o->in_tag[0] ? c0 : 0, t1 = o->in_tag[1] ? c1 : 0;
    if (!o->resident || o->tag[0] != t0 || o->tag[1] != t1) {
        opd_drop(o);
        o->resident = 1; o->tag[0] = t0; o->tag[1] = t1;
    }
    if (!o->have[c0][c1]) {
        o->have[c0][c1] = 1;
        o->occ += o->tile_words;
        o->moved += o->tile_words;
        if (o->occ > o->peak) o->peak = o->occ;
    }
}

/* advance an odometer over loops[0..n) (outer -> inner); returns 0 when done */
static int odo_next(const uint8_t *loops, int n, const uint32_t xD[4], int v[4])
{
    for (int a = n - 1; a >= 0; --a) {
        int q = loops[a];
        if (++v[q] < (int)xD[q]) return 1;
        v[q] = 0;
    }
    return 0;
}

/* One execution of the stage program.  reserve = NULL: plain run.  Otherwise reserve[A,B,C,D,E]
 * holds the footprints measured by an earlier run and the two reservation counts are taken. */
static int sim_pass(const uint32_t xG[4], const uint32_t xD[4], const uint8_t order[4],
                    const uint8_t level[4] /* A,B,D,E */, int recompute, int fused,
                    const uint64_t *reserve, sim_result *out)
{
    memset(out, 0, sizeof(*out));
    for (int q = 0; q < 4; ++q)
        if (xD[q] == 0 || xD[q] > SIM_MAX_D || xG[q] == 0) return -1;
    if (recompute && !fused) return -1;

    int pos[4];
    for (int a = 0; a < 4; ++a) pos[order[a]] = 3 - a;

    /* split the loop sequence: leading loops that both operators iterate,
     * then each operator's private remainder */
    uint8_t pre[4], prod[4], cons[4];
    int npre = 0, nprod = 0, ncons = 0, lead = 1;
    for (int a = 0; a < 4; ++a) {
        int q = order[a];
        int both = (q == SI || q == SL || (recompute && q == SJ));
        if (lead && both) { pre[npre++] = (uint8_t)q; continue; }
        lead = 0;
        if (q != SJ) prod[nprod++] = (uint8_t)q;
        if (q != SK) cons[ncons++] = (uint8_t)q;
    }

    uint64_t tA = (uint64_t)xG[SI] * xG[SK], tB = (uint64_t)xG[SK] * xG[SL];
    uint64_t tC = (uint64_t)xG[SI] * xG[SL], tD = (uint64_t)xG[SL] * xG[SJ];
    uint64_t tE = (uint64_t)xG[SI] * xG[SJ];

    sim_operand A, B, D, E, Cw, Cr;
    opd_init(&A, SI, SK, level[0], pos, tA);
    opd_init(&B, SK, SL, level[1], pos, tB);
    opd_init(&D, SL, SJ, level[2], pos, tD);
    opd_init(&E, SI, SJ, level[3], pos, tE);
    opd_init(&Cw, SI, SL, 0, pos, tC);      /* unfused only: C spilled by Op1 */
    opd_init(&Cr, SI, SL, 0, pos, tC);      /* unfused only: C fetched by Op2 */

    /* on-chip C tiles of the current region (fused) and their k-progress */
    static _Thread_local uint8_t c_live[SIM_MAX_D][SIM_MAX_D];
    static _Thread_local uint16_t c_acc[SIM_MAX_D][SIM_MAX_D];
    /* how often each (i,l,j) tile product was executed */
    static _Thread_local uint16_t done[SIM_MAX_D][SIM_MAX_D][SIM_MAX_D];
    memset(done, 0, sizeof(done));
    uint64_t c_occ = 0;

    uint64_t n_stage = 0, max_occ = 0, max_res = 0, max_touch = 0, c_peak = 0, n_regions = 0;
    sim_operand *ext[4] = {&A, &B, &D, &E};
    const int ext_slot[4] = {0, 1, 3, 4};
#define RECORD_STAGE() do { \
        uint64_t occ_ = A.occ + B.occ + D.occ + E.occ + Cw.occ + Cr.occ + c_occ; \
        if (occ_ > max_occ) max_occ = occ_; \
        if (c_occ > c_peak) c_peak = c_occ; \
        if (n_stage < SIM_TRACE) out->occ_trace[n_stage] = (uint32_t)occ_; \
        if (reserve) { \
            /* tile-level operands and C as they are resident; retained operands by footprint */ \
            uint64_t dyn_ = Cw.occ + Cr.occ + c_occ, all_ = 0, touched_ = 0; \
            for (int x_ = 0; x_ < 4; ++x_) { \
                if (ext[x_]->level == 0) dyn_ += ext[x_]->occ; \
                else { all_ += reserve[ext_slot[x_]]; if (ext[x_]->resident) touched_ += reserve[ext_slot[x_]]; } \
            } \
            if (all_ + dyn_ > max_res) max_res = all_ + dyn_; \
            if (touched_ + dyn_ > max_touch) max_touch = touched_ + dyn_; \
        } \
        ++n_stage; } while (0)

    int v[4] = {0, 0, 0, 0};
    int first_region = 1;
    do {    /* iterations of the shared leading loops */
        ++n_regions;
        /* ---- the producer takes over ---- */
        if (!first_region) {
            if (level[2] == 0) opd_drop(&D);
            if (level[3] == 0) opd_drop(&E);
            opd_drop(&Cr);
        }
        first_region = 0;
        memset(c_live, 0, sizeof(c_live));
        memset(c_acc, 0, sizeof(c_acc));
        c_occ = 0;
        uint64_t region_c_tiles = 0;
        for (int a = 0; a < nprod; ++a) v[prod[a]] = 0;
        do {
            opd_touch(&A, v);
            opd_touch(&B, v);
            if (fused) {
                if (!c_live[v[SI]][v[SL]]) { c_live[v[SI]][v[SL]] = 1; c_occ += tC; ++region_c_tiles; }
            } else {
                if (!c_live[v[SI]][v[SL]]) { c_live[v[SI]][v[SL]] = 1; ++region_c_tiles; }
                opd_touch(&Cw, v);
            }
            ++c_acc[v[SI]][v[SL]];
            out->macs1 += (uint64_t)xG[SI] * xG[SK] * xG[SL];
            ++out->stages1;
            RECORD_STAGE();
        } while (odo_next(prod, nprod, xD, v));

        /* ---- hand-over: softmax on the finished C tiles ---- */
        if (level[0] == 0) opd_drop(&A);
        if (level[1] == 0) opd_drop(&B);
        opd_drop(&Cw);
        out->softmax_elems += region_c_tiles * tC;
        RECORD_STAGE();

        /* ---- the consumer takes over ---- */
        for (int a = 0; a < ncons; ++a) v[cons[a]] = 0;
        do {
            if (!c_live[v[SI]][v[SL]] || c_acc[v[SI]][v[SL]] != xD[SK]) out->psum_violation = 1;
            if (!fused) opd_touch(&Cr, v);
            opd_touch(&D, v);
            opd_touch(&E, v);
            ++done[v[SI]][v[SL]][v[SJ]];
            out->macs2 += (uint64_t)xG[SI] * xG[SL] * xG[SJ];
            ++out->stages2;
            RECORD_STAGE();
        } while (odo_next(cons, ncons, xD, v));
        for (int a = 0; a < ncons; ++a) v[cons[a]] = 0;
        for (int a = 0; a < nprod; ++a) v[prod[a]] = 0;
    } while (odo_next(pre, npre, xD, v));

    for (uint32_t i = 0; i < xD[SI]; ++i)
        for (uint32_t l = 0; l < xD[SL]; ++l)
            for (uint32_t j = 0; j < xD[SJ]; ++j)
                if (done[i][l][j] != 1) out->coverage_error = 1;

    out->da[0] = A.moved; out->da[1] = B.moved;
    out->da[3] = D.moved; out->da[4] = E.moved;
    if (fused) out->da[2] = 0;
    else {
        /* spill by Op1 + fetch by Op2 + the separate softmax pass (read S, write P) */
        uint64_t IL = (uint64_t)xG[SI] * xD[SI] * xG[SL] * xD[SL];
        out->da[2] = Cw.moved + Cr.moved + 2 * IL;
    }
    out->max_occupancy = max_occ;
    out->max_reserved = max_res;
    out->max_reserved_touch = max_touch;
    out->footprint[0] = A.peak; out->footprint[1] = B.peak;
    out->footprint[2] = fused ? c_peak : (Cw.peak > Cr.peak ? Cw.peak : Cr.peak);
    out->footprint[3] = D.peak; out->footprint[4] = E.peak;
    out->n_regions = n_regions;
    out->n_stages = n_stage;
    return 0;
}

int sim_run(const uint32_t xG[4], const uint32_t xD[4], const uint8_t order[4],
            const uint8_t level[4] /* A,B,D,E */, int recompute, int fused,
            sim_result *out)
{
    /* first run: what happens, and how large each operand's block gets */
    sim_result first;
    int rc = sim_pass(xG, xD, order, level, recompute, fused, 0, &first);
    if (rc) { memset(out, 0, sizeof(*out)); return rc; }
    /* second run of the same program with those footprints reserved */
    rc = sim_pass(xG, xD, order, level, recompute, fused, first.footprint, out);
    if (rc) return rc;
    /* the two runs are the same program: everything but the reservation counts agrees */
    if (out->max_occupancy != first.max_occupancy || out->n_stages != first.n_stages) return -2;
    for (int x = 0; x < 5; ++x)
        if (out->da[x] != first.da[x] || out->footprint[x] != first.footprint[x]) return -2;
    return 0;
}

/* One tile-level matmul m x r x n on an R x C array whose PEs each keep g
 * stationary words: enumerate every fold of the stationary operand onto the
 * array and count the words that cross the buffer<->register-file boundary and
 * the cycles spent.  mode: 0 weight-, 1 input-, 2 output-stationary. */
int sim_tile_matmul(uint32_t m, uint32_t r, uint32_t n, int mode,
                    uint32_t R, uint32_t C, uint32_t g,
                    uint64_t *words, uint64_t *cycles, uint64_t *macs)
{
    uint32_t u, v, t;
    if (!R || !C || !g) return -1;
    if (mode == 0)      { u = r; v = n; t = m; }
    else if (mode == 1) { u = m; v = r; t = n; }
    else if (mode == 2) { u = m; v = n; t = r; }
    else return -1;
    uint64_t w = 0, cyc = 0, mac = 0;
    for (uint32_t u0 = 0; u0 < u; u0 += R) {
        uint32_t cu = u - u0 < R ? u - u0 : R;                 /* rows in use */
        for (uint32_t v0 = 0; v0 < v; v0 += C * g) {
            uint32_t cv = v - v0 < C * g ? v - v0 : C * g;     /* stationary columns held */
            w += (uint64_t)cu * cv;                            /* pin the stationary chunk */
            for (uint32_t tt = 0; tt < t; ++tt) {
                w += cu;                                       /* one vector along the rows in */
                w += cv;                                       /* one vector along the columns in/out */
                mac += (uint64_t)cu * cv;
            }
            /* each PE column serves its g (or fewer) stationary words in turn */
            for (uint32_t c0 = 0; c0 < cv; c0 += C) cyc += t;
        }
    }
    *words = w; *cycles = cyc; *macs = mac;
    return 0;
}
