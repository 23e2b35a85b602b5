// Batched search over short row lists (the pruned rows of Sec. VI-B): many problems in one launch.
//
// The online stage of Sec. VI-A costs a few hundred surviving rows against a few thousand tilings
// per problem -- microseconds of arithmetic -- so a sweep over hardware designs and sequence lengths
// (Sec. VII-H, VII-I) is bound by launches and table traffic unless the problems share a launch.
// Here one work item is (problem, chunk of 64 tilings) and a block builds the chunk's slice of the
// boundary-side tables straight into LDS, from the problem's divisor lists: nothing per tiling ever
// touches HBM.  Lane = tiling, wave = a contiguous share of one group's row list, so a row's
// selectors are wave-uniform (scalar loads) and the per-tiling constants of the nine stationary
// combinations sit in registers for the whole item.  Each item leaves one (key, index) record per
// objective; the block that finishes a problem's last item reduces the problem's records and writes
// the winner's full cost record and mapping.
//
// Included once by mmee.hip, after kernels.h.
#pragma once
#include "kernels.h"

namespace mmee {

constexpr int BATCH_THREADS = 1024;
constexpr int BATCH_WAVES = BATCH_THREADS / 64;
constexpr int BATCH_TC = 64;                 // tilings per item = lanes of a wave
constexpr int BATCH_NCS = 20;                // constants per (tiling, r), as in layout.h

struct BatchProblem {                        // one problem, in device memory
    DivTable dv;
    ModelConst mc;
    uint32_t first_item;                     // its first work item in the launch
    uint32_t n_chunks;                       // its work items
    uint32_t slot;                           // where its N_OBJ final records go
    uint32_t pad_;
};

struct BatchArgs {
    const BatchProblem *prob;
    const uint32_t *first_items;             // [n_prob + 1] ascending, for the item -> problem search
    uint32_t n_prob, n_items;
    const uint4 *enc;                        // every encoded row (for the winner's record)
    const uint4 *row_enc;                    // the compacted lists, row id in .w
    uint32_t task_off[BATCH_WAVES];          // per wave: where its share of a list starts in row_enc,
    uint32_t task_cnt[BATCH_WAVES];          //           how many rows it holds,
    uint32_t task_g[BATCH_WAVES];            //           and the group g = r + 2 f they belong to
    Key *item_keys;                          // [n_items][N_OBJ]
    uint32_t *tickets;                       // [n_prob] items finished
    unsigned long long *hints;               // [n_prob][N_OBJ] lowest value seen so far (bits of a non-negative fp64)
    FinalRecord *final_out;                  // [result slot][N_OBJ]
};

// ---- the boundary side, one value at a time ---------------------------------------------------
// Every count of the model is an integer below 2^53 (the host refuses workloads where it is not),
// so products and sums of them are exact in fp64 whatever their order.

struct TilingF {                             // boundary vector of one tiling (Eq. (10)), as fp64
    double G[4], D[4];
};

__device__ __forceinline__ TilingF tiling_of(const DivTable &dv, uint32_t t)
{
    TilingF v;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t n = dv.ndiv[q];
        const uint32_t digit = t % n;
        t /= n;
        const uint32_t g = dv.div[q][digit];
        v.G[q] = (double)g;
        v.D[q] = (double)(dv.X[q] / g);
    }
    return v;
}

// tile_X * {1, d0, d1, d0 d1}; option 4 = the operand takes no space
__device__ __forceinline__ double footprint(double tile, double d0, double d1, uint32_t opt)
{
    const double v = tile * ((opt & 1) ? d0 : 1.0) * ((opt & 2) ? d1 : 1.0);
    return opt >= 4 ? 0.0 : v;
}

// entry `ent` of the per-tiling table (layout.h), bh = B*H for the scaled DRAM terms, 1 for the raw ones
__device__ __forceinline__ double table_entry(uint32_t ent, const TilingF &v, const double X[4], double bh)
{
    const double tA = v.G[DI] * v.G[DK], tB = v.G[DK] * v.G[DL], tC = v.G[DI] * v.G[DL], tD = v.G[DL] * v.G[DJ],
                 tE = v.G[DI] * v.G[DJ];
    if (ent < ENT_BS_DE) {                                   // BS_A[a] + BS_B[b]
        const uint32_t k = ent - ENT_BS_AB;
        return footprint(tA, v.D[DI], v.D[DK], k & 3) + footprint(tB, v.D[DK], v.D[DL], k >> 2);
    }
    if (ent < ENT_RET_DE) {                                  // BS_D[a] + BS_E[b]
        const uint32_t k = ent - ENT_BS_DE;
        return footprint(tD, v.D[DL], v.D[DJ], k & 3) + footprint(tE, v.D[DI], v.D[DJ], k >> 2);
    }
    if (ent < ENT_RET_AB) {                                  // tau_D BS_D[a] + tau_E BS_E[b]
        const uint32_t k = ent - ENT_RET_DE;
        return footprint(tD, v.D[DL], v.D[DJ], k % 5) + footprint(tE, v.D[DI], v.D[DJ], k / 5);
    }
    if (ent < ENT_BS_C) {                                    // tau_A BS_A[a] + tau_B BS_B[b]
        const uint32_t k = ent - ENT_RET_AB;
        return footprint(tA, v.D[DI], v.D[DK], k % 5) + footprint(tB, v.D[DK], v.D[DL], k / 5);
    }
    if (ent < ENT_DA_AB) return footprint(tC, v.D[DI], v.D[DL], ent - ENT_BS_C);
    if (ent < ENT_DA_DE) {                                   // |A| {1, l_D, j_D, l_D j_D} + |B| {1, i_D, j_D, i_D j_D}
        const uint32_t k = ent - ENT_DA_AB;
        return bh * (footprint(X[DI] * X[DK], v.D[DL], v.D[DJ], k & 3) + footprint(X[DK] * X[DL], v.D[DI], v.D[DJ], k >> 2));
    }
    if (ent < ENT_DA_C) {                                    // |D| {1, i_D, k_D, i_D k_D} + |E| {1, k_D, l_D, k_D l_D}
        const uint32_t k = ent - ENT_DA_DE;
        return bh * (footprint(X[DL] * X[DJ], v.D[DI], v.D[DK], k & 3) + footprint(X[DI] * X[DJ], v.D[DK], v.D[DL], k >> 2));
    }
    // unfused C: spilled by Op1, fetched by Op2, plus one softmax pass over S and P; option 4: fused, no traffic
    const uint32_t c = ent - ENT_DA_C;
    const double spill = (c & 1) ? v.D[DK] : 1.0, fetch = (c & 2) ? v.D[DJ] : 1.0;
    return c >= 4 ? 0.0 : bh * (X[DI] * X[DL]) * (spill + fetch + 2.0);
}

// ceil(a / b) for a 32-bit a; b may exceed 32 bits (then one fold suffices)
__device__ __forceinline__ double cdiv_f64(uint32_t a, uint64_t b) { return b > a ? 1.0 : (double)((a - 1u) / (uint32_t)b + 1u); }

// words crossing buffer<->RF and cycles of one tile matmul m x r x n; mode 0 WS, 1 IS, 2 OS
__device__ __forceinline__ void tile_cost_f64(uint32_t m, uint32_t r, uint32_t n, uint32_t mode, const ModelConst &mc,
                                              double &words, double &cycles)
{
    const uint32_t rows_dim = mode == 0 ? r : m;             // spread over PE rows
    const uint32_t cols_dim = mode == 1 ? r : n;             // spread over PE columns
    const double time_dim = (double)(mode == 0 ? m : (mode == 1 ? n : r));
    const double row_folds = cdiv_f64(rows_dim, mc.pe_rows);
    const double rd = (double)rows_dim, cd = (double)cols_dim;
    words = rd * cd + time_dim * rd * cdiv_f64(cols_dim, (uint64_t)mc.pe_cols * mc.g_words) + time_dim * cd * row_folds;
    cycles = row_folds * cdiv_f64(cols_dim, mc.pe_cols) * time_dim;
}

// what one stationary combination (s1, s2) and recomputation choice r contribute for one tiling
struct ComboTerms {
    double br, cyc, mac, sm;                 // buffer<->RF words, cycles, MACs, softmax elements (per instance)
    double lat_part;                         // c_lat * max(cycles, buffer<->RF time)
    double e_rf_part, e_mac_part;
};

__device__ __forceinline__ ComboTerms combo_terms(const TilingF &v, const double X[4], const ModelConst &mc, uint32_t r,
                                                  uint32_t s1, uint32_t s2)
{
    ComboTerms o;
    double br1, cy1, br2, cy2;
    tile_cost_f64((uint32_t)v.G[DI], (uint32_t)v.G[DK], (uint32_t)v.G[DL], s1, mc, br1, cy1);
    tile_cost_f64((uint32_t)v.G[DI], (uint32_t)v.G[DL], (uint32_t)v.G[DJ], s2, mc, br2, cy2);
    const double rho = r ? v.D[DJ] : 1.0;                    // producer repeated per j tile (Sec. V-D)
    const double st1 = rho * v.D[DI] * v.D[DK] * v.D[DL], st2 = v.D[DI] * v.D[DL] * v.D[DJ];
    o.br = st1 * br1 + st2 * br2;
    o.cyc = st1 * cy1 + st2 * cy2;
    o.mac = rho * X[DI] * X[DK] * X[DL] + X[DI] * X[DL] * X[DJ];
    o.sm = rho * X[DI] * X[DL];
    const double t_gb = mc.gb_bw > 0.0 ? (o.br * mc.word) / mc.gb_bw : 0.0;
    o.lat_part = mc.c_lat * fmax(o.cyc, t_gb);
    o.e_rf_part = mc.e_rf * (mc.BH * 3.0 * o.mac);
    o.e_mac_part = mc.e_mac * (mc.BH * (o.mac + (double)mc.c_softmax * o.sm));
    return o;
}

// One candidate, complete, from the problem description alone: the winner's cost record (Sec. V-D's
// order of the energy terms, as eval_candidate).
__device__ __forceinline__ void eval_candidate_direct(const uint4 *enc, const DivTable &dv, const ModelConst &mc, uint64_t idx,
                                                      mmee_cost &c)
{
    const uint32_t t = (uint32_t)(idx % mc.T), row = (uint32_t)(idx / mc.T);
    const uint32_t lo = row % 15000;
    uint32_t hi = row / 15000;
    const uint32_t r = hi & 1; hi >>= 1;
    const uint32_t s1 = hi % 3; hi /= 3;
    const uint32_t s2 = hi % 3, f = hi / 3;
    const uint4 e = enc[lo + ROWS_PER_GROUP * (r + 2 * f)];
    if (!(sel_of(e, ROW_FLAGS) & 1)) {
        c.bs_words = c.da_words = c.br_words = c.mac_total = c.comp_cycles = 0;
        c.energy_pj = pos_inf(); c.latency_cycles = pos_inf();
        c.valid = 0; c.reason = 1;
        return;
    }
    const TilingF v = tiling_of(dv, t);
    const double X[4] = {(double)dv.X[0], (double)dv.X[1], (double)dv.X[2], (double)dv.X[3]};
    double w[NSEL];
#pragma unroll
    for (int k = 0; k < NSEL; ++k) w[k] = table_entry(sel_of(e, k), v, X, 1.0);
    const ComboTerms ct = combo_terms(v, X, mc, r, s1, s2);
    const double bs = fmax(w[0] + w[2] + w[1], w[3] + w[2] + w[4]);     // Eq. (1), (2), (4)
    const double da = w[5] + w[6] + w[7];                                // Eq. (7)
    c.bs_words = (uint64_t)bs; c.da_words = (uint64_t)da; c.br_words = (uint64_t)ct.br;
    c.mac_total = (uint64_t)ct.mac; c.comp_cycles = (uint64_t)ct.cyc;
    if (bs > mc.cap_words) {
        c.energy_pj = pos_inf(); c.latency_cycles = pos_inf();
        c.valid = 0; c.reason = 2;
        return;
    }
    double en = mc.e_dram * (mc.BH * da);
    en = en + mc.e_gb * (mc.BH * (da + ct.br));
    en = en + ct.e_rf_part;
    en = en + ct.e_mac_part;
    double l_dram;
    if (mc.bw_pow2) l_dram = da * mc.eval_k;
    else l_dram = (da * mc.word) / mc.dram_bw;
    c.energy_pj = en;
    c.latency_cycles = fmax(mc.c_lat * l_dram, ct.lat_part);
    c.valid = 1; c.reason = 0;
}

// hints start at +inf, tickets at zero
__global__ void k_batch_init(uint32_t *tickets, unsigned long long *hints, uint32_t n_prob)
{
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a < n_prob) tickets[a] = 0;
    if (a < n_prob * N_OBJ) hints[a] = 0x7ff0000000000000ull;
}

// MASK, FAST, REGROUP as in k_search.  One block per work item.
template <int MASK, bool FAST, bool REGROUP>
__global__ __launch_bounds__(BATCH_THREADS) void k_search_batch(BatchArgs a)
{
    __shared__ double tab[NENT * BATCH_TC];                  // entry-major, lane = tiling: conflict-free as it is
    __shared__ double cst[2 * BATCH_NCS * BATCH_TC];         // [r][constant][tiling]
    __shared__ Key wave_best[N_OBJ][BATCH_WAVES];
    __shared__ uint32_t is_last;

    const double inf = pos_inf();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t item = blockIdx.x;

    // which problem: the last p with first_items[p] <= item
    ConstPtr<uint32_t> firsts = as_constant(a.first_items);
    uint32_t lo = 0, hi = a.n_prob;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (firsts[mid] <= item) lo = mid; else hi = mid;
    }
    const uint32_t p = lo;
    const BatchProblem *pr = a.prob + p;
    // the descriptors are read-only while the kernel runs: wave-uniform fields through scalar loads
    ModelConst mc;
    {
        ConstPtr<uint32_t> words = as_constant(reinterpret_cast<const uint32_t *>(&pr->mc));
        uint32_t buf[sizeof(ModelConst) / 4];
#pragma unroll
        for (uint32_t k = 0; k < sizeof(ModelConst) / 4; ++k) buf[k] = words[k];
        __builtin_memcpy(&mc, buf, sizeof(ModelConst));
    }
    ConstPtr<uint32_t> tail = as_constant(&pr->first_item);      // first_item, n_chunks, slot
    const uint32_t n_chunks = tail[1], slot = tail[2];
    const uint32_t t0 = (item - firsts[p]) * BATCH_TC;
    const uint32_t T = mc.T;
    const uint32_t nt = min((uint32_t)BATCH_TC, T - t0);

    // ---- build: this lane's tiling (beyond the chunk: its last tiling once more, masked out below)
    {
        const TilingF v = tiling_of(pr->dv, t0 + min(lane, nt - 1));
        const double X[4] = {(double)pr->dv.X[0], (double)pr->dv.X[1], (double)pr->dv.X[2], (double)pr->dv.X[3]};
        if (wave < 9) {
            // one stationary combination per wave, both recomputation choices
            const uint32_t s1 = wave % 3, s2 = wave / 3;
#pragma unroll
            for (uint32_t r = 0; r < 2; ++r) {
                const ComboTerms ct = combo_terms(v, X, mc, r, s1, s2);
                double *cs = cst + r * BATCH_NCS * BATCH_TC + lane;
                cs[wave * BATCH_TC] = REGROUP ? (mc.e_gb * (mc.BH * ct.br) + ct.e_rf_part) + ct.e_mac_part : mc.BH * ct.br;
                cs[(9 + wave) * BATCH_TC] = ct.lat_part;
                if (wave == 0) { cs[18 * BATCH_TC] = ct.e_rf_part; cs[19 * BATCH_TC] = ct.e_mac_part; }
            }
        } else {
            // the 123 table entries, shared out over the other seven waves
            constexpr uint32_t PER = (NENT + (BATCH_WAVES - 9) - 1) / (BATCH_WAVES - 9);
            const uint32_t e0 = (wave - 9) * PER, e1 = min(e0 + PER, (uint32_t)NENT);
            for (uint32_t ent = e0; ent < e1; ++ent) tab[ent * BATCH_TC + lane] = table_entry(ent, v, X, mc.BH);
        }
    }
    __syncthreads();

    // ---- cost: this wave's share of one group's rows against the chunk
    const uint32_t n_rows = a.task_cnt[wave], g = a.task_g[wave], r = g & 1;
    ConstPtr<uint32_t> rows32 = as_constant(reinterpret_cast<const uint32_t *>(a.row_enc + a.task_off[wave]));
    auto load_row = [&](uint32_t i) {
        uint4 e;
        e.x = rows32[4 * i]; e.y = rows32[4 * i + 1]; e.z = rows32[4 * i + 2]; e.w = rows32[4 * i + 3];
        return e;
    };
    const double cap = lane < nt ? mc.cap_words : -1.0;      // a lane beyond the chunk never passes the capacity test
    double gb[9], latc[9];
    {
        const double *cs = cst + r * BATCH_NCS * BATCH_TC + lane;
#pragma unroll
        for (int c = 0; c < 9; ++c) { gb[c] = cs[c * BATCH_TC]; latc[c] = cs[(9 + c) * BATCH_TC]; }
    }
    const double e_rf_part = REGROUP ? 0.0 : cst[(r * BATCH_NCS + 18) * BATCH_TC + lane];
    const double e_mac_part = REGROUP ? 0.0 : cst[(r * BATCH_NCS + 19) * BATCH_TC + lane];
    const double *col = tab + lane;

    double bestE[9], bestL[9], bestP[9], bestLE_l[9], bestLE_e[9];
    uint32_t codeLE[9];
#pragma unroll
    for (int c9 = 0; c9 < 9; ++c9) { bestE[c9] = bestL[c9] = bestP[c9] = bestLE_l[c9] = bestLE_e[c9] = inf; codeLE[c9] = 0; }

    // the row part of one (row, tiling): Eq. (1), (2), (4), capacity mask, B*H * Eq. (7)
    auto row_part = [&](const uint4 &e, double &dram_words, double &e_part, double &l_dram) {
        double w[NSEL];
#pragma unroll
        for (int k = 0; k < NSEL; ++k) w[k] = col[sel_of(e, k) * BATCH_TC];
        const bool ok = fmax(w[0] + w[2] + w[1], w[3] + w[2] + w[4]) <= cap;
        dram_words = w[5] + w[6] + w[7];
        e_part = (REGROUP ? mc.e_sum : mc.e_dram) * dram_words;
        if constexpr (FAST) l_dram = dram_words * mc.dram_k;
        else l_dram = mc.dram_bw > 0.0 ? mc.c_lat * (((dram_words / mc.BH) * mc.word) / mc.dram_bw) : 0.0;
        const double over = __hiloint2double(ok ? 0 : 0x7ff00000, 0);
        e_part = fmax(e_part, over);
        l_dram = fmax(l_dram, over);
        pin(e_part);
        pin(l_dram);
    };
    auto combo_cost = [&](double dram_words, double e_part, double l_dram, double gb_c, double latc_c, double &en, double &lat) {
        if constexpr (REGROUP) {
            en = e_part + gb_c;
        } else {
            const double gb_words = dram_words + gb_c;
            en = e_part + mc.e_gb * gb_words;
            en = en + e_rf_part;
            en = en + e_mac_part;
        }
        lat = fmax(l_dram, latc_c);
    };

    for (uint32_t i = 0; i < n_rows; ++i) {
        const uint4 e = load_row(i);
        double dram_words, e_part, l_dram;
        row_part(e, dram_words, e_part, l_dram);
#pragma unroll
        for (int c9 = 0; c9 < 9; ++c9) {
            double en, lat;
            combo_cost(dram_words, e_part, l_dram, gb[c9], latc[c9], en, lat);
            if constexpr (MASK & 1) bestE[c9] = fmin(bestE[c9], en);
            if constexpr (MASK & 2) bestL[c9] = fmin(bestL[c9], lat);
            if constexpr (MASK & 8) bestP[c9] = fmin(bestP[c9], en * lat);
            if constexpr (MASK & 4) {
                // rows come in index order: a strict < keeps the lowest index on ties
                const bool lt = (lat < bestLE_l[c9]) | ((lat == bestLE_l[c9]) & (en < bestLE_e[c9]));
                bestLE_l[c9] = lt ? lat : bestLE_l[c9];
                bestLE_e[c9] = lt ? en : bestLE_e[c9];
                codeLE[c9] = lt ? i : codeLE[c9];
            }
        }
    }

    // ---- this wave's record per key
    Key mine[N_OBJ];
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) { mine[o].p = inf; mine[o].s = 0.0; mine[o].idx = ~0ull; }
    if (n_rows) {
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) {
            if (!((MASK >> o) & 1) || o == 2) continue;
            // scalar keys: only minima were kept; the position is recovered where it can matter
            const double *best = o == 0 ? bestE : (o == 1 ? bestL : bestP);
            double mine_v = best[0];
#pragma unroll
            for (int c9 = 1; c9 < 9; ++c9) mine_v = fmin(mine_v, best[c9]);
            const double wave_v = uniform_f64(wave_min_f64(mine_v));
            if (!(wave_v < inf)) continue;
            // a value some other item has already reached or beaten strictly cannot win
            unsigned long long *hint = a.hints + (uint64_t)p * N_OBJ + o;
            const double seen = __longlong_as_double((long long)__hip_atomic_load(hint, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if (wave_v > seen) continue;
            // the lowest combination in which some tiling reaches the minimum
            uint32_t cstar = 9;
#pragma unroll
            for (int c9 = 8; c9 >= 0; --c9) cstar = best[c9] == wave_v ? (uint32_t)c9 : cstar;
            const uint32_t c_u = __builtin_amdgcn_readfirstlane(wave_min_u32(cstar));
            double gb_u = gb[0], latc_u = latc[0];
#pragma unroll
            for (int c9 = 1; c9 < 9; ++c9) {
                gb_u = c_u == (uint32_t)c9 ? gb[c9] : gb_u;
                latc_u = c_u == (uint32_t)c9 ? latc[c9] : latc_u;
            }
            // the first row (index order) in which a tiling reaches it, at its lowest such tiling
            for (uint32_t i = 0; i < n_rows; ++i) {
                const uint4 e = load_row(i);
                double dram_words, e_part, l_dram, en, lat;
                row_part(e, dram_words, e_part, l_dram);
                combo_cost(dram_words, e_part, l_dram, gb_u, latc_u, en, lat);
                const double val = o == 0 ? en : (o == 1 ? lat : en * lat);
                const unsigned long long hits = __ballot(val == wave_v);
                if (!hits) continue;
                const uint32_t index_row = index_row_base(e.w) + 30000u * (c_u % 3) + 90000u * (c_u / 3);
                mine[o].p = wave_v;
                mine[o].idx = (uint64_t)t0 + ((uint32_t)__ffsll((long long)hits) - 1u) + (uint64_t)T * index_row;
                break;
            }
            // (only a value that this wave's record really carries may turn other waves away)
            if (lane == 0 && mine[o].p == wave_v)
                __hip_atomic_fetch_min(hint, (unsigned long long)__double_as_longlong(wave_v), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        }
        if constexpr (MASK & 4) {
            Key k;
            k.p = inf; k.s = 0.0; k.idx = ~0ull;
#pragma unroll
            for (int c9 = 0; c9 < 9; ++c9) {
                // ascending combination = ascending index
                if (bestLE_l[c9] < k.p || (bestLE_l[c9] == k.p && bestLE_e[c9] < k.s)) {
                    const uint32_t dfrow = rows32[4 * codeLE[c9] + 3];
                    k.p = bestLE_l[c9];
                    k.s = bestLE_e[c9];
                    k.idx = (uint64_t)(t0 + lane) + (uint64_t)T * (index_row_base(dfrow) + 30000u * (c9 % 3) + 90000u * (c9 / 3));
                }
            }
            if (!(k.p < inf)) { k.s = 0.0; k.idx = ~0ull; }
            mine[2] = wave_min(k);
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o)
            if ((MASK >> o) & 1) wave_best[o][wave] = mine[o];
    }
    __syncthreads();

    // ---- the item's record, then the problem's ticket
    if (threadIdx.x == 0) {
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) {
            if (!((MASK >> o) & 1)) continue;
            Key k = wave_best[o][0];
            for (int wv = 1; wv < BATCH_WAVES; ++wv)
                if (key_less(wave_best[o][wv], k)) k = wave_best[o][wv];
            Key *dst = a.item_keys + (uint64_t)item * N_OBJ + o;
            __hip_atomic_store(&dst->idx, k.idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(reinterpret_cast<uint64_t *>(&dst->p), (uint64_t)__double_as_longlong(k.p), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(reinterpret_cast<uint64_t *>(&dst->s), (uint64_t)__double_as_longlong(k.s), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        __threadfence();
        const uint32_t ticket = __hip_atomic_fetch_add(a.tickets + p, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        is_last = ticket == n_chunks - 1;
    }
    __syncthreads();
    if (!is_last) return;

    // ---- the block that finished the problem's last item reduces the problem's records
    __threadfence();
    const uint32_t item0 = firsts[p];
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) {
        if (!((MASK >> o) & 1)) continue;
        Key k; k.p = inf; k.s = 0.0; k.idx = ~0ull;
        for (uint32_t b = threadIdx.x; b < n_chunks; b += BATCH_THREADS) {
            Key *src = a.item_keys + (uint64_t)(item0 + b) * N_OBJ + o;
            Key c;
            c.idx = __hip_atomic_load(&src->idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c.p = __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<uint64_t *>(&src->p), __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_AGENT));
            c.s = __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<uint64_t *>(&src->s), __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_AGENT));
            if (key_less(c, k)) k = c;
        }
        k = wave_min(k);
        if (lane == 0) wave_best[o][wave] = k;
    }
    __syncthreads();
    if (threadIdx.x < N_OBJ && ((MASK >> threadIdx.x) & 1)) {
        const int o = threadIdx.x;
        Key k = wave_best[o][0];
        for (int wv = 1; wv < BATCH_WAVES; ++wv)
            if (key_less(wave_best[o][wv], k)) k = wave_best[o][wv];
        FinalRecord *fr = a.final_out + (uint64_t)slot * N_OBJ + o;
        fr->key = k;
        mmee_cost c;
        mmee_mapping m;
        if (k.p < inf) {
            eval_candidate_direct(a.enc, pr->dv, mc, k.idx, c);
            decode_candidate(pr->dv, T, k.idx, m);
        } else {
            c.bs_words = c.da_words = c.br_words = c.mac_total = c.comp_cycles = 0;
            c.energy_pj = inf; c.latency_cycles = inf; c.valid = 0; c.reason = 0;
            for (int q = 0; q < 4; ++q) { m.xG[q] = m.xD[q] = 0; m.order[q] = m.level[q] = 0; }
            m.idx = ~0ull; m.recompute = m.stat1 = m.stat2 = m.fused = 0;
        }
        const uint64_t *cs = reinterpret_cast<const uint64_t *>(&c);
        for (int q = 0; q < 8; ++q) fr->cost[q] = cs[q];
        uint64_t mbuf[7] = {0, 0, 0, 0, 0, 0, 0};
        __builtin_memcpy(mbuf, &m, sizeof(mmee_mapping));
        for (int q = 0; q < 7; ++q) fr->map[q] = mbuf[q];
    }
}

}  // namespace mmee
