// Batched search over short row lists (the pruned rows of Sec. VI-B): many problems in one launch.
//
// The online stage of Sec. VI-A costs a few hundred surviving rows against a few thousand tilings
// per problem -- microseconds of arithmetic -- so a sweep over hardware designs and sequence lengths
// (Sec. VII-H, VII-I) is bound by launches and table traffic unless the problems share a launch.
// Here one work item is (problem, chunk of 64 tilings) and a block builds the chunk's slice of the
// boundary-side tables straight into LDS, from the problem's divisor lists: nothing per tiling ever
// touches HBM.  Lane = tiling, wave = a contiguous piece of one group's row list, so a row's table
// offsets are wave-uniform and the per-tiling constants of the nine stationary combinations sit in
// registers for the whole item.  Only the table entries that the rows refer to are staged (77 of 123
// for the pruned rows), which lets two 512-thread blocks share a CU; a row's offsets into the staged
// table and the entries' places in it reach the waves as scalar loads.  A block takes a contiguous range
// of items, waves carry their best (value, index) across the items of a problem, and each (block,
// problem) stretch leaves one record per key; k_batch_finish, launched behind the search, reduces a
// problem's records and writes the winner's full cost record and mapping.
//
// Included once by mmee.hip, after kernels.h.
#pragma once
#include "kernels.h"

namespace mmee {

constexpr int BATCH_THREADS = 512;           // two blocks per CU, four waves per SIMD
constexpr int BATCH_WAVES = BATCH_THREADS / 64;
constexpr int BATCH_TC = 64;                 // tilings per item = lanes of a wave
constexpr int BATCH_NCS = 20;                // constants per (tiling, r), as in layout.h
constexpr int BATCH_MAX_USED = 80;           // table entries the row lists may refer to (the pruned rows use 77)
constexpr int BATCH_MAX_ROWS = 288;          // rows the lists may hold (the pruned lists hold 270)
constexpr int BATCH_MAX_SPLIT = 4;           // blocks that may share the rows of one chunk (small launches)

constexpr int BATCH_INLINE_DIVS = 448;       // divisors (all four lists together) of a problem that rides in the kernel arguments

struct BatchProblemHead {
    ModelConst mc;
    uint32_t first_item;                     // its first work item in the launch
    uint32_t n_work;                         // its work items: chunks of 64 tilings x row shares
    uint32_t slot;                           // where its N_OBJ final records go
    uint32_t pad_;
    uint32_t X[4], ndiv[4];                  // extents and divisor counts of i, k, l, j
};

struct BatchProblem {                        // one problem, in device memory
    BatchProblemHead h;
    uint32_t list[4 * MAXDIV];               // the four divisor lists one after the other, ndiv[q] entries each
};

// A launch of one problem carries it inside the kernel arguments: no descriptor copy has to reach the
// device before the kernel may start.  Same layout as the front of a BatchProblem, then the launch's
// two-entry first-item table.
struct BatchInline {
    BatchProblemHead h;
    uint32_t list[BATCH_INLINE_DIVS];
    uint32_t firsts[2];
    uint32_t on, pad_;
};

struct BatchArgs {
    const BatchProblem *prob;
    const uint32_t *first_items;             // [n_prob + 1] ascending, for the item -> problem search
    uint32_t n_prob, n_items;
    const uint4 *enc;                        // every encoded row (for the winner's record)
    // the row lists, one after the other (group by group, ascending row number inside a group)
    const uint32_t *row_off;                 // [n_rows][8] byte offsets of a row's eight table values in the staged table
    const uint32_t *row_df;                  // [n_rows] the rows' numbers (levels/order + 15000 * (r + 2 f))
    const uint32_t *cmap;                    // [NENT] table entry -> its place in the staged table, 0xFFFF when no row refers to it
    uint32_t n_rows, n_used;
    // A chunk's rows are shared out over `split` work items (1 in a large launch; more when the launch
    // would otherwise leave most of the chip idle), and inside a work item over the waves of the block.
    uint32_t split, split_log2;                 // a power of two
    uint32_t task_lo[BATCH_MAX_SPLIT * BATCH_WAVES];     // per (share, wave): its first row in the lists,
    uint32_t task_cnt[BATCH_MAX_SPLIT * BATCH_WAVES];    //                    how many rows it takes,
    uint32_t task_g[BATCH_MAX_SPLIT * BATCH_WAVES];      //                    and the group g = r + 2 f they belong to
    Key *item_keys;                          // [n_items][N_OBJ]; written at the first item of every (block, problem) stretch
    uint32_t per_block;                      // items per block of the search launch (the finish kernel needs it)
    FinalRecord *final_out;                  // [result slot][N_OBJ]
    BatchInline inl;                         // inl.on: the launch's only problem is here, prob and first_items are unused
};

// Where a launch's problems and first-item table are: in device memory, or inside the kernel
// arguments themselves (which are ordinary read-only memory to the kernel).
__device__ __forceinline__ void batch_tables(const BatchArgs &a, const BatchProblem *&probs, ConstPtr<uint32_t> &firsts)
{
    probs = a.prob;
    firsts = as_constant(a.first_items);
    if (a.inl.on) {
        ConstPtr<char> args = (ConstPtr<char>)__builtin_amdgcn_kernarg_segment_ptr();
        probs = (const BatchProblem *)(args + offsetof(BatchArgs, inl));
        firsts = (ConstPtr<uint32_t>)(args + offsetof(BatchArgs, inl) + offsetof(BatchInline, firsts));
    }
}

// ---- the boundary side, one value at a time ---------------------------------------------------
// Every count of the model is an integer below 2^53 (the host refuses workloads where it is not),
// so products and sums of them are exact in fp64 whatever their order.

struct TilingF {                             // boundary vector of one tiling (Eq. (10)), as fp64
    double G[4], D[4];
};

// digit q of tiling t: the intra-tile size x_G and the inter-tile count x_D of dimension q
__device__ __forceinline__ void tiling_dim(const DivTable &dv, uint32_t t, int q, double &G, double &D)
{
    uint32_t radix = 1;
    for (int k = 0; k < q; ++k) radix *= dv.ndiv[k];
    const uint32_t g = dv.div[q][(t / radix) % dv.ndiv[q]];
    G = (double)g;
    D = (double)(dv.X[q] / g);
}

__device__ __forceinline__ TilingF tiling_of(const DivTable &dv, uint32_t t)
{
    TilingF v;
#pragma unroll
    for (int q = 0; q < 4; ++q) tiling_dim(dv, t, q, v.G[q], v.D[q]);
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

// ceil(a / b) for a whole number 1 <= a < 2^32 held in fp64, given 1 / b rounded once (ModelConst)
__device__ __forceinline__ double cdiv_f64(double a, double rcp_b) { return __builtin_floor((a - 0.5) * rcp_b) + 1.0; }

// words crossing buffer<->RF and cycles of one tile matmul m x r x n; mode 0 WS, 1 IS, 2 OS
__device__ __forceinline__ void tile_cost_f64(double m, double r, double n, uint32_t mode, const ModelConst &mc,
                                              double &words, double &cycles)
{
    const double rd = mode == 0 ? r : m;                     // spread over PE rows
    const double cd = mode == 1 ? r : n;                     // spread over PE columns
    const double time_dim = mode == 0 ? m : (mode == 1 ? n : r);
    const double row_folds = cdiv_f64(rd, mc.rcp_rows);
    words = rd * cd + time_dim * rd * cdiv_f64(cd, mc.rcp_cols_g) + time_dim * cd * row_folds;
    cycles = row_folds * cdiv_f64(cd, mc.rcp_cols) * time_dim;
}

// what one stationary combination (s1, s2) and recomputation choice r contribute for one tiling
struct ComboTerms {
    double br, cyc, mac, sm;                 // buffer<->RF words, cycles, MACs, softmax elements (per instance)
    double lat_part;                         // c_lat * max(cycles, buffer<->RF time)
    double e_rf_part, e_mac_part;
};

// ... from the two operators' tile costs (words and cycles of one tile matmul each)
__device__ __forceinline__ ComboTerms combo_terms_from(const TilingF &v, const double X[4], const ModelConst &mc, uint32_t r,
                                                       double br1, double cy1, double br2, double cy2)
{
    ComboTerms o;
    const double rho = r ? v.D[DJ] : 1.0;                    // producer repeated per j tile (Sec. V-D)
    const double st1 = rho * v.D[DI] * v.D[DK] * v.D[DL], st2 = v.D[DI] * v.D[DL] * v.D[DJ];
    o.br = st1 * br1 + st2 * br2;
    o.cyc = st1 * cy1 + st2 * cy2;
    o.mac = rho * X[DI] * X[DK] * X[DL] + X[DI] * X[DL] * X[DJ];
    o.sm = rho * X[DI] * X[DL];
    // a power-of-two bandwidth: the quotient is the product with one exactly representable constant
    const double t_gb = mc.gb_pow2 ? o.br * mc.gb_k : (mc.gb_bw > 0.0 ? (o.br * mc.word) / mc.gb_bw : 0.0);
    o.lat_part = mc.c_lat * fmax(o.cyc, t_gb);
    o.e_rf_part = mc.e_rf * (mc.BH * 3.0 * o.mac);
    o.e_mac_part = mc.e_mac * (mc.BH * (o.mac + (double)mc.c_softmax * o.sm));
    return o;
}

__device__ __forceinline__ ComboTerms combo_terms(const TilingF &v, const double X[4], const ModelConst &mc, uint32_t r,
                                                  uint32_t s1, uint32_t s2)
{
    double br1, cy1, br2, cy2;
    tile_cost_f64(v.G[DI], v.G[DK], v.G[DL], s1, mc, br1, cy1);
    tile_cost_f64(v.G[DI], v.G[DL], v.G[DJ], s2, mc, br2, cy2);
    return combo_terms_from(v, X, mc, r, br1, cy1, br2, cy2);
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

// The table entries of one kind, for this lane's tiling, into the staged table: x[a] + y[b] for every
// option pair (na x nb of them, entry number first + a + na * b), each at the place cmap gives it.
template <int NA, int NB>
__device__ __forceinline__ void stage_pair_sums(double *tab_lane, ConstPtr<uint32_t> cmap, int first, const double (&x)[5],
                                                const double (&y)[5])
{
    // the places are wave-uniform (scalar loads): an entry no row refers to costs a branch, nothing more
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            const uint32_t at = cmap[first + a + NA * b];
            if (at != 0xFFFFu) tab_lane[at * BATCH_TC] = x[a] + y[b];
        }
}

// footprints of one operand under its five options (4 = takes no space)
__device__ __forceinline__ void footprints(double (&o)[5], double tile, double d0, double d1)
{
    o[0] = tile; o[1] = tile * d0; o[2] = tile * d1; o[3] = tile * d0 * d1; o[4] = 0.0;
}

// MASK, FAST, REGROUP as in k_search.  Every block takes a contiguous range of the work items, so
// that it stays with one problem for many items: a wave keeps its running best (value, index) per key
// across the items of a problem and recovers a position only where it can matter; one record per
// (block, problem) leaves the block, at the slot of the first item of that stretch.
template <int MASK, bool FAST, bool REGROUP>
__global__ __launch_bounds__(BATCH_THREADS, 4) void k_search_batch(BatchArgs a)
{
    __shared__ double tab[BATCH_MAX_USED * BATCH_TC];        // entry-major, lane = tiling: conflict-free as it is
    __shared__ double cst[2 * BATCH_NCS * BATCH_TC];         // [r][constant][tiling]
    __shared__ double gd[8 * BATCH_TC];                      // the chunk's boundary vectors: G[0..3], D[0..3] per tiling
    __shared__ double tc[6 * 2 * BATCH_TC];                  // tile costs: [op * 3 + mode][words, cycles][tiling]
    __shared__ uint32_t div_lds[4 * MAXDIV];                 // the current problem's divisor lists
    __shared__ Key wave_best[N_OBJ][BATCH_WAVES];

    const double inf = pos_inf();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // A wave's rows and the table's entry places are the same for all its lanes: both come through
    // the constant address space (scalar loads), a row's eight offsets as one load, one row ahead of use.
    typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
    ConstPtr<u32x8> row_offs = (ConstPtr<u32x8>)a.row_off;
    ConstPtr<uint32_t> cmap_c = as_constant(a.cmap);

    const uint32_t item_lo = blockIdx.x * a.per_block, item_hi = min(item_lo + a.per_block, a.n_items);
    if (item_lo >= item_hi) return;
    // the first item's problem: the last p with first_items[p] <= item; later items move p on
    const BatchProblem *probs;
    ConstPtr<uint32_t> firsts;
    batch_tables(a, probs, firsts);
    uint32_t p;
    {
        uint32_t lo = 0, hi = a.n_prob;
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (firsts[mid] <= item_lo) lo = mid; else hi = mid;
        }
        p = lo;
    }
    ConstPtr<uint32_t> row_df = as_constant(a.row_df);
    const char *tab_bytes = reinterpret_cast<const char *>(tab) + lane * 8;

    // the wave's running best over the items of the current problem
    double run_p[N_OBJ], run_s[N_OBJ];                       // (primary, secondary) as in Key; secondary 0 for scalar keys
    uint64_t run_idx[N_OBJ];
    uint32_t run_c[N_OBJ], run_i[N_OBJ], run_t0[N_OBJ];      // its combination, its row (place in the row lists), its chunk
    auto reset_running = [&]() {
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) { run_p[o] = inf; run_s[o] = 0.0; run_idx[o] = ~0ull; run_c[o] = run_i[o] = run_t0[o] = 0; }
    };
    reset_running();
    uint32_t staged_p = 0xFFFFFFFFu;

    // one stretch = the block's items of one problem
    for (uint32_t seg_first = item_lo; seg_first < item_hi;) {
      while (firsts[p + 1] <= seg_first) ++p;
      const uint32_t seg_end = min(item_hi, firsts[p + 1]), seg_len = seg_end - seg_first;
      // The items of a stretch are visited with a stride of about 0.618 of its length (coprime to it):
      // costs tend to move steadily along the tiling index, and in such an order the running minimum
      // improves a logarithmic number of times instead of at every item, so positions are rarely recovered.
      uint32_t stride = max(1u, (uint32_t)(((uint64_t)seg_len * 40503u) >> 16));
      {
          auto gcd = [](uint32_t x, uint32_t y) { while (y) { const uint32_t z = x % y; x = y; y = z; } return x; };
          while (stride < seg_len && gcd(stride, seg_len) != 1) ++stride;
          if (stride >= seg_len) stride = 1;
      }
      uint32_t place = 0;                                    // (visit * stride) mod seg_len, kept by addition
      for (uint32_t visit = 0; visit < seg_len; ++visit, place = place + stride >= seg_len ? place + stride - seg_len : place + stride) {
        const uint32_t item = seg_first + place;
        const BatchProblem *pr = probs + p;
        // the descriptors are read-only while the kernel runs: wave-uniform fields through scalar loads
        ModelConst mc;
        {
            ConstPtr<uint32_t> words = as_constant(reinterpret_cast<const uint32_t *>(&pr->h.mc));
            uint32_t buf[sizeof(ModelConst) / 4];
#pragma unroll
            for (uint32_t k = 0; k < sizeof(ModelConst) / 4; ++k) buf[k] = words[k];
            __builtin_memcpy(&mc, buf, sizeof(ModelConst));
        }
        ConstPtr<uint32_t> tail = as_constant(&pr->h.first_item);
        const uint32_t work = item - tail[0];
        const uint32_t t0 = (work >> a.split_log2) * BATCH_TC;
        // this wave's piece of one group's rows, within the work item's share of the chunk's rows
        const uint32_t task = (work & (a.split - 1)) * BATCH_WAVES + wave;
        const uint32_t n_rows = a.task_cnt[task], row_lo = a.task_lo[task], r = a.task_g[task] & 1;
        const uint32_t T = mc.T;
        const uint32_t nt = min((uint32_t)BATCH_TC, T - t0);
        ConstPtr<uint32_t> dvw = as_constant(pr->h.X);       // X[4], ndiv[4]
        const uint32_t nd0 = dvw[4], nd1 = dvw[5], nd2 = dvw[6], nd3 = dvw[7];
        if (staged_p != p) {
            // a new problem: its divisor lists into LDS (the previous item's barriers have passed)
            const uint32_t n_list = nd0 + nd1 + nd2 + nd3;
            for (uint32_t k = threadIdx.x; k < n_list; k += BATCH_THREADS) div_lds[k] = pr->list[k];
            staged_p = p;
            __syncthreads();
        }

        // ---- decode: dimension q of every tiling of the chunk by wave q (beyond the chunk: its last
        // tiling once more, masked out below)
        if (wave < 4) {
            const uint32_t t = t0 + min(lane, nt - 1);
            const uint32_t radix = wave == 0 ? 1u : (wave == 1 ? nd0 : (wave == 2 ? nd0 * nd1 : nd0 * nd1 * nd2));
            const uint32_t nq = wave == 0 ? nd0 : (wave == 1 ? nd1 : (wave == 2 ? nd2 : nd3));
            const uint32_t list0 = wave == 0 ? 0u : (wave == 1 ? nd0 : (wave == 2 ? nd0 + nd1 : nd0 + nd1 + nd2));
            const uint32_t g = div_lds[list0 + (t / radix) % nq];
            gd[wave * BATCH_TC + lane] = (double)g;
            gd[(4 + wave) * BATCH_TC + lane] = (double)(dvw[wave] / g);
        }
        __syncthreads();

        // ---- build, first half: the six tile costs (one per wave) and the table entries the rows refer to
        TilingF v;
#pragma unroll
        for (int q = 0; q < 4; ++q) { v.G[q] = gd[q * BATCH_TC + lane]; v.D[q] = gd[(4 + q) * BATCH_TC + lane]; }
        const double X[4] = {(double)dvw[0], (double)dvw[1], (double)dvw[2], (double)dvw[3]};
        if (wave < 6) {
            double words, cycles;
            if (wave < 3) tile_cost_f64(v.G[DI], v.G[DK], v.G[DL], wave, mc, words, cycles);
            else tile_cost_f64(v.G[DI], v.G[DL], v.G[DJ], wave - 3, mc, words, cycles);
            tc[(wave * 2) * BATCH_TC + lane] = words;
            tc[(wave * 2 + 1) * BATCH_TC + lane] = cycles;
        }
        {
            // one kind of table entry per wave (layout.h); the two waves without a tile cost take the 25-entry kinds
            double *tab_lane = tab + lane;
            double x[5], y[5];
            switch (wave) {
            case 0:                                           // BS_A[a] + BS_B[b]
                footprints(x, v.G[DI] * v.G[DK], v.D[DI], v.D[DK]);
                footprints(y, v.G[DK] * v.G[DL], v.D[DK], v.D[DL]);
                stage_pair_sums<4, 4>(tab_lane, cmap_c, ENT_BS_AB, x, y);
                break;
            case 1:                                           // BS_D[a] + BS_E[b]
                footprints(x, v.G[DL] * v.G[DJ], v.D[DL], v.D[DJ]);
                footprints(y, v.G[DI] * v.G[DJ], v.D[DI], v.D[DJ]);
                stage_pair_sums<4, 4>(tab_lane, cmap_c, ENT_BS_DE, x, y);
                break;
            case 6:                                           // tau_D BS_D[a] + tau_E BS_E[b]
                footprints(x, v.G[DL] * v.G[DJ], v.D[DL], v.D[DJ]);
                footprints(y, v.G[DI] * v.G[DJ], v.D[DI], v.D[DJ]);
                stage_pair_sums<5, 5>(tab_lane, cmap_c, ENT_RET_DE, x, y);
                break;
            case 7:                                           // tau_A BS_A[a] + tau_B BS_B[b]
                footprints(x, v.G[DI] * v.G[DK], v.D[DI], v.D[DK]);
                footprints(y, v.G[DK] * v.G[DL], v.D[DK], v.D[DL]);
                stage_pair_sums<5, 5>(tab_lane, cmap_c, ENT_RET_AB, x, y);
                break;
            case 2: {                                         // BS_C[c]; B*H * DA_C[c]
                footprints(x, v.G[DI] * v.G[DL], v.D[DI], v.D[DL]);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t at = cmap_c[ENT_BS_C + c];
                    if (at != 0xFFFFu) tab_lane[at * BATCH_TC] = x[c];
                }
#pragma unroll
                for (int c = 0; c < 5; ++c) {
                    // unfused C: spilled by Op1, fetched by Op2, one softmax pass over S and P; option 4: fused
                    const double spill = (c & 1) ? v.D[DK] : 1.0, fetch = (c & 2) ? v.D[DJ] : 1.0;
                    const uint32_t at = cmap_c[ENT_DA_C + c];
                    if (at != 0xFFFFu) tab_lane[at * BATCH_TC] = c >= 4 ? 0.0 : mc.BH * (X[DI] * X[DL]) * (spill + fetch + 2.0);
                }
                break;
            }
            case 3:                                           // B*H * (|A| {1, l_D, j_D, l_D j_D} + |B| {1, i_D, j_D, i_D j_D})
                footprints(x, mc.BH * (X[DI] * X[DK]), v.D[DL], v.D[DJ]);
                footprints(y, mc.BH * (X[DK] * X[DL]), v.D[DI], v.D[DJ]);
                stage_pair_sums<4, 4>(tab_lane, cmap_c, ENT_DA_AB, x, y);
                break;
            case 4:                                           // B*H * (|D| {1, i_D, k_D, i_D k_D} + |E| {1, k_D, l_D, k_D l_D})
                footprints(x, mc.BH * (X[DL] * X[DJ]), v.D[DI], v.D[DK]);
                footprints(y, mc.BH * (X[DI] * X[DJ]), v.D[DK], v.D[DL]);
                stage_pair_sums<4, 4>(tab_lane, cmap_c, ENT_DA_DE, x, y);
                break;
            default: break;
            }
        }
        __syncthreads();
        // ---- build, second half: the 18 (recomputation, combination) constant pairs, shared out over the waves
        for (uint32_t job = wave; job < 18; job += BATCH_WAVES) {
            const uint32_t rr = job / 9, c9 = job % 9, s1 = c9 % 3, s2 = c9 / 3;
            const ComboTerms ct = combo_terms_from(v, X, mc, rr, tc[(s1 * 2) * BATCH_TC + lane], tc[(s1 * 2 + 1) * BATCH_TC + lane],
                                                   tc[((3 + s2) * 2) * BATCH_TC + lane], tc[((3 + s2) * 2 + 1) * BATCH_TC + lane]);
            double *cs = cst + rr * BATCH_NCS * BATCH_TC + lane;
            cs[c9 * BATCH_TC] = REGROUP ? (mc.e_gb * (mc.BH * ct.br) + ct.e_rf_part) + ct.e_mac_part : mc.BH * ct.br;
            cs[(9 + c9) * BATCH_TC] = ct.lat_part;
            if (c9 == 0) { cs[18 * BATCH_TC] = ct.e_rf_part; cs[19 * BATCH_TC] = ct.e_mac_part; }
        }
        __syncthreads();

        // ---- cost: this wave's rows against the chunk
        const double cap = lane < nt ? mc.cap_words : -1.0;  // a lane beyond the chunk never passes the capacity test
        double gb[9], latc[9];
        {
            const double *cs = cst + r * BATCH_NCS * BATCH_TC + lane;
#pragma unroll
            for (int c = 0; c < 9; ++c) { gb[c] = cs[c * BATCH_TC]; latc[c] = cs[(9 + c) * BATCH_TC]; }
        }
        const double e_rf_part = REGROUP ? 0.0 : cst[(r * BATCH_NCS + 18) * BATCH_TC + lane];
        const double e_mac_part = REGROUP ? 0.0 : cst[(r * BATCH_NCS + 19) * BATCH_TC + lane];

        // Every key is a monotone function of a candidate's DRAM traffic once tiling, recomputation choice
        // and stationary combination are fixed: DRAM energy and DRAM time grow with it, every rounded sum,
        // product and maximum they pass through keeps the order, and the capacity test does not look at the
        // combination.  All rows of a wave's piece share the recomputation choice.  Among the rows that fit,
        // the one with the least traffic therefore has the least cost under every combination and every key
        // -- bit for bit the value a row-by-row minimum gives -- and the loop over the rows only has to keep
        // that least traffic per tiling.  (Rounding may give rows with more traffic the same cost: positions
        // are recovered below by comparing costs, not traffic.)
        auto row_words = [&](const u32x8 off) -> double {
            double w[NSEL];
#pragma unroll
            for (int k = 0; k < NSEL; ++k) w[k] = *reinterpret_cast<const double *>(tab_bytes + off[k]);
            const bool ok = fmax(w[0] + w[2] + w[1], w[3] + w[2] + w[4]) <= cap;     // Eq. (1), (2), (4)
            const double dram_words = w[5] + w[6] + w[7];                            // B*H * Eq. (7)
            return ok ? dram_words : inf;
        };
        // the row side of a candidate's costs, from its traffic: DRAM energy (regrouped: DRAM and buffer
        // energy of the DRAM words) and DRAM time, +inf both when no row fits; the words themselves (0 then)
        struct RowSide { double d, e_part, l_dram; };
        auto row_side = [&](double dram_words) {
            RowSide rs;
            const bool feasible = dram_words < inf;
            rs.d = feasible ? dram_words : 0.0;
            const double over = feasible ? 0.0 : inf;
            rs.e_part = fmax((REGROUP ? mc.e_sum : mc.e_dram) * rs.d, over);
            double l_dram;
            if constexpr (FAST) l_dram = rs.d * mc.dram_k;
            else l_dram = mc.dram_bw > 0.0 ? mc.c_lat * (((rs.d / mc.BH) * mc.word) / mc.dram_bw) : 0.0;
            rs.l_dram = fmax(l_dram, over);
            return rs;
        };
        // ... joined with a combination's constants: energy and latency of the candidate
        auto costs_with = [&](const RowSide &rs, double gb_c, double latc_c, double rf_part, double mac_part, double &en, double &lat) {
            if constexpr (REGROUP) {
                en = rs.e_part + gb_c;
            } else {
                const double gb_words = rs.d + gb_c;
                en = rs.e_part + mc.e_gb * gb_words;
                en = en + rf_part;
                en = en + mac_part;
            }
            lat = fmax(rs.l_dram, latc_c);
        };
        auto costs_of = [&](const RowSide &rs, double gb_c, double latc_c, double &en, double &lat) {
            costs_with(rs, gb_c, latc_c, e_rf_part, e_mac_part, en, lat);
        };
        // key o of a candidate as a (primary, secondary) pair; the secondary is 0 for the scalar keys
        auto key_of = [&](int o, double en, double lat, double &kp, double &ks) {
            kp = o == 0 ? en : (o == 3 ? en * lat : lat);
            ks = o == 2 ? en : 0.0;
        };

        double min_d = inf;
        {
            u32x8 off_next = row_offs[min(row_lo, a.n_rows - 1)];
#pragma unroll 4
            for (uint32_t i = 0; i < n_rows; ++i) {
                const u32x8 off_now = off_next;
                off_next = row_offs[row_lo + min(i + 1, n_rows - 1)];
                min_d = fmin(min_d, row_words(off_now));
            }
        }

        // ---- fold the item into the wave's running best
        if (n_rows) {
            double en9[9], lat9[9];
            const RowSide best_row = row_side(min_d);
#pragma unroll
            for (int c9 = 0; c9 < 9; ++c9) costs_of(best_row, gb[c9], latc[c9], en9[c9], lat9[c9]);
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                // only minima were kept; the position is recovered where it can matter
                double mine_p = inf, mine_s = inf;
#pragma unroll
                for (int c9 = 0; c9 < 9; ++c9) {
                    double kp, ks;
                    key_of(o, en9[c9], lat9[c9], kp, ks);
                    const bool lt = (kp < mine_p) | ((kp == mine_p) & (ks < mine_s));
                    mine_p = lt ? kp : mine_p;
                    mine_s = lt ? ks : mine_s;
                }
                const double wave_p = uniform_f64(wave_min_f64(mine_p));
                // nothing feasible, or this wave already holds a lower value
                if (!(wave_p < inf) || wave_p > run_p[o]) continue;
                const double wave_s = o == 2 ? uniform_f64(wave_min_f64(mine_p == wave_p ? mine_s : inf)) : 0.0;
                if (wave_p == run_p[o] && wave_s > run_s[o]) continue;
                // the lowest combination in which some tiling reaches the minimum
                uint32_t cstar = 9;
#pragma unroll
                for (int c9 = 8; c9 >= 0; --c9) {
                    double kp, ks;
                    key_of(o, en9[c9], lat9[c9], kp, ks);
                    cstar = ((kp == wave_p) & (ks == wave_s)) ? (uint32_t)c9 : cstar;
                }
                const uint32_t c_u = __builtin_amdgcn_readfirstlane(wave_min_u32(cstar));
                const uint32_t combo_rows = 30000u * (c_u % 3) + 90000u * (c_u / 3);
                // Index order is (combination, row, tiling).  An equal value only matters where it can sit at a
                // lower index than the running best: in a lower combination; or in the same one in an earlier
                // row, or in the same row if this chunk comes before the running best's.
                // (A wave's pieces all lie in one group's list, whatever the share: list places compare like indices.)
                uint32_t scan = n_rows;
                if (wave_p == run_p[o] && wave_s == run_s[o]) {
                    if (c_u > run_c[o]) continue;
                    if (c_u == run_c[o]) {
                        const uint32_t upto = t0 < run_t0[o] ? run_i[o] + 1 : run_i[o];    // list places below this one matter
                        scan = upto > row_lo ? min(upto - row_lo, n_rows) : 0u;
                    }
                }
                double gb_u = gb[0], latc_u = latc[0];
#pragma unroll
                for (int c9 = 1; c9 < 9; ++c9) {
                    gb_u = c_u == (uint32_t)c9 ? gb[c9] : gb_u;
                    latc_u = c_u == (uint32_t)c9 ? latc[c9] : latc_u;
                }
                // The first row (index order) in which a tiling reaches it, at its lowest such tiling.  Only a
                // tiling whose least-traffic row reaches the value can hold it at all.
                uint32_t found_i = 0xFFFFFFFFu, found_lane = 0;
                double en_u, lat_u, kp_u, ks_u;
                costs_of(best_row, gb_u, latc_u, en_u, lat_u);
                key_of(o, en_u, lat_u, kp_u, ks_u);
                unsigned long long cands = __ballot((kp_u == wave_p) & (ks_u == wave_s));
                if (n_rows <= 64 && 2u * (uint32_t)__popcll(cands) <= scan) {
                    // Few such tilings: take them one by one with lane = row, all rows of the piece at once.
                    const uint4 *ro = reinterpret_cast<const uint4 *>(a.row_off) + 2 * (row_lo + min(lane, n_rows - 1));
                    const uint4 oa = ro[0], ob = ro[1];
                    const uint32_t off[NSEL] = {oa.x, oa.y, oa.z, oa.w, ob.x, ob.y, ob.z, ob.w};
                    while (cands) {
                        const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)__ffsll((long long)cands) - 1u);
                        cands &= cands - 1;
                        const char *col = reinterpret_cast<const char *>(tab) + l * 8;
                        double w[NSEL];
#pragma unroll
                        for (int k = 0; k < NSEL; ++k) w[k] = *reinterpret_cast<const double *>(col + off[k]);
                        // (a tiling beyond the chunk's end is never among them: plain capacity)
                        const bool ok = fmax(w[0] + w[2] + w[1], w[3] + w[2] + w[4]) <= mc.cap_words;
                        double en, lat, kp, ks;
                        costs_with(row_side(ok ? w[5] + w[6] + w[7] : inf), lane_value_f64(gb_u, l), lane_value_f64(latc_u, l),
                                   lane_value_f64(e_rf_part, l), lane_value_f64(e_mac_part, l), en, lat);
                        key_of(o, en, lat, kp, ks);
                        const unsigned long long hits = __ballot((lane < scan) & (kp == wave_p) & (ks == wave_s));
                        if (!hits) continue;
                        const uint32_t i = (uint32_t)__ffsll((long long)hits) - 1u;
                        if (i < found_i) { found_i = i; found_lane = l; }     // ascending tilings: the lower one stays on equal rows
                        if (found_i == 0) break;
                    }
                } else {
                    u32x8 scan_next = row_offs[row_lo];
                    for (uint32_t i = 0; i < scan; ++i) {
                        double en, lat, kp, ks;
                        const u32x8 scan_now = scan_next;
                        scan_next = row_offs[row_lo + min(i + 1, n_rows - 1)];
                        costs_of(row_side(row_words(scan_now)), gb_u, latc_u, en, lat);
                        key_of(o, en, lat, kp, ks);
                        const unsigned long long hits = __ballot((kp == wave_p) & (ks == wave_s));
                        if (!hits) continue;
                        found_i = i;
                        found_lane = (uint32_t)__ffsll((long long)hits) - 1u;
                        break;
                    }
                }
                if (found_i != 0xFFFFFFFFu) {
                    const uint64_t idx = (uint64_t)t0 + found_lane + (uint64_t)T * (index_row_base(row_df[row_lo + found_i]) + combo_rows);
                    if (wave_p < run_p[o] || wave_s < run_s[o] || idx < run_idx[o]) {
                        run_p[o] = wave_p; run_s[o] = wave_s; run_idx[o] = idx; run_c[o] = c_u; run_i[o] = row_lo + found_i; run_t0[o] = t0;
                    }
                }
            }
        }

        // ---- after the stretch's last item its record leaves the block
        const bool flush = visit + 1 == seg_len;
        if (!flush) {
            __syncthreads();                                 // every wave is done with the staged tables
            continue;
        }
        if (lane == 0) {
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                Key k;
                k.p = run_p[o]; k.s = run_s[o]; k.idx = run_idx[o];
                wave_best[o][wave] = k;
            }
        }
        reset_running();
        __syncthreads();
        if (threadIdx.x == 0) {
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                Key k = wave_best[o][0];
                for (int wv = 1; wv < BATCH_WAVES; ++wv)
                    if (key_less(wave_best[o][wv], k)) k = wave_best[o][wv];
                a.item_keys[(uint64_t)seg_first * N_OBJ + o] = k;       // read by the finish kernel, after this one
            }
        }
        __syncthreads();                                     // wave_best and the staged tables are free again
      }
      seg_first = seg_end;
    }
}


// After the search: one block per problem reduces the problem's records -- one per (block, problem)
// stretch of the search launch, at the problem's first item and at every block boundary inside the
// problem -- and writes the winner's full cost record and mapping.
template <int MASK>
__global__ __launch_bounds__(256) void k_batch_finish(BatchArgs a)
{
    __shared__ Key wave_best[N_OBJ][4];
    __shared__ BatchProblemHead head_s;                      // the problem's description, fetched while the records arrive
    __shared__ DivTable dv_s;
    const double inf = pos_inf();
    const uint32_t p = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const BatchProblem *probs;
    ConstPtr<uint32_t> firsts;
    batch_tables(a, probs, firsts);
    const BatchProblem *pr = probs + p;
    {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&pr->h);
        uint32_t *dst = reinterpret_cast<uint32_t *>(&head_s);
        for (uint32_t k = threadIdx.x; k < sizeof(BatchProblemHead) / 4; k += 256) dst[k] = src[k];
        // the packed lists back into the table form the decoding helpers take
        uint32_t first = 0;
        for (int q = 0; q < 4; ++q) {
            const uint32_t n = pr->h.ndiv[q];
            for (uint32_t k = threadIdx.x; k < n; k += 256) dv_s.div[q][k] = pr->list[first + k];
            first += n;
        }
        if (threadIdx.x < 4) { dv_s.X[threadIdx.x] = pr->h.X[threadIdx.x]; dv_s.ndiv[threadIdx.x] = pr->h.ndiv[threadIdx.x]; }
    }
    const uint32_t item0 = pr->h.first_item, n_work = pr->h.n_work;
    const uint32_t inner0 = item0 / a.per_block + 1;         // first block boundary after the problem's first item
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) {
        if (!((MASK >> o) & 1)) continue;
        Key k; k.p = inf; k.s = 0.0; k.idx = ~0ull;
        for (uint32_t b = threadIdx.x;; b += 256) {
            const uint64_t at = b == 0 ? (uint64_t)item0 : (uint64_t)(inner0 + b - 1) * a.per_block;
            if (at >= (uint64_t)item0 + n_work) break;
            const Key c = a.item_keys[at * N_OBJ + o];
            if (key_less(c, k)) k = c;
        }
        k = wave_min(k);
        if (lane == 0) wave_best[o][wave] = k;
    }
    __syncthreads();
    if (threadIdx.x < N_OBJ && ((MASK >> threadIdx.x) & 1)) {
        const int o = threadIdx.x;
        Key k = wave_best[o][0];
        for (int wv = 1; wv < 4; ++wv)
            if (key_less(wave_best[o][wv], k)) k = wave_best[o][wv];
        FinalRecord *fr = a.final_out + (uint64_t)head_s.slot * N_OBJ + o;
        fr->key = k;
        mmee_cost c;
        mmee_mapping m;
        if (k.p < inf) {
            eval_candidate_direct(a.enc, dv_s, head_s.mc, k.idx, c);
            decode_candidate(dv_s, head_s.mc.T, k.idx, m);
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
