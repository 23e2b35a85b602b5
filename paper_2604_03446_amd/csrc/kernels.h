// HIP kernels of libmmee for gfx950 (wave64).  Included once by mmee.hip.
//
//   k_build_rows     offline:  row id -> selectors (the query-matrix side, Sec. V-E / VI-A)
//   k_prune_rows     offline:  symbolic dominance test inside each group (Sec. VI-B)
//   k_compact_rows   offline:  ballot + prefix compaction of surviving rows
//   k_build_tilings  online:   tiling id -> boundaries -> per-tiling tables (the boundary-matrix side)
//   k_search         online:   contraction, capacity mask, energy/latency, hierarchical argmin (lane = row)
//   k_search_dense   online:   the same for one key over the full row set (lane = tiling)
//   k_front_step     online:   one point of the buffer-size / DRAM-access front
//   k_eval_batch     online:   the same model, one 64-byte record per candidate
//   k_decode         online:   index -> mapping
// (k_search_batch and k_batch_finish, the pruned search over many problems per launch: batch.h)
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <math.h>
#include "../../include/mmee.h"
#include "layout.h"

namespace mmee {

// ---------------------------------------------------------------------------
// small helpers

__device__ __forceinline__ double pos_inf() { return __longlong_as_double(0x7ff0000000000000ll); }

__device__ __forceinline__ bool key_less(const Key &a, const Key &b)
{
    if (a.p != b.p) return a.p < b.p;
    if (a.s != b.s) return a.s < b.s;
    return a.idx < b.idx;
}

// ---- cross-lane moves for the wave-level argmin (DPP inside a row of 16 lanes,
// ds_swizzle across rows of a half wave, ds_bpermute across the halves) --------
template <int STEP>
__device__ __forceinline__ uint32_t lane_exchange(uint32_t v)
{
    if constexpr (STEP == 0) return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    if constexpr (STEP == 1) return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    if constexpr (STEP == 2) return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xF, 0xF, false);  // row_half_mirror
    if constexpr (STEP == 3) return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xF, 0xF, false);  // row_mirror
    if constexpr (STEP == 4) return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);                          // lane ^ 16
    return (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((threadIdx.x & 63) ^ 32) << 2), (int)v);                   // lane ^ 32
}

template <int STEP>
__device__ __forceinline__ Key key_exchange(const Key &k)
{
    Key o;
    unsigned long long p = (unsigned long long)__double_as_longlong(k.p);
    unsigned long long s = (unsigned long long)__double_as_longlong(k.s);
    uint32_t plo = lane_exchange<STEP>((uint32_t)p), phi = lane_exchange<STEP>((uint32_t)(p >> 32));
    uint32_t slo = lane_exchange<STEP>((uint32_t)s), shi = lane_exchange<STEP>((uint32_t)(s >> 32));
    uint32_t ilo = lane_exchange<STEP>((uint32_t)k.idx), ihi = lane_exchange<STEP>((uint32_t)(k.idx >> 32));
    o.p = __longlong_as_double((long long)(((unsigned long long)phi << 32) | plo));
    o.s = __longlong_as_double((long long)(((unsigned long long)shi << 32) | slo));
    o.idx = ((uint64_t)ihi << 32) | ilo;
    return o;
}

// after this every lane of the wave holds the wave's minimum
__device__ __forceinline__ Key wave_min(Key k)
{
    Key o;
    o = key_exchange<0>(k); if (key_less(o, k)) k = o;
    o = key_exchange<1>(k); if (key_less(o, k)) k = o;
    o = key_exchange<2>(k); if (key_less(o, k)) k = o;
    o = key_exchange<3>(k); if (key_less(o, k)) k = o;
    o = key_exchange<4>(k); if (key_less(o, k)) k = o;
    o = key_exchange<5>(k); if (key_less(o, k)) k = o;
    return k;
}

// Read-only tables that the kernel never writes are read through the constant address space, so
// that wave-uniform reads become scalar loads even next to atomics and inline assembly.
template <class T> using ConstPtr = const T __attribute__((address_space(4))) *;
typedef ConstPtr<double> ConstF64;
template <class T> __device__ __forceinline__ ConstPtr<T> as_constant(const T *p) { return (ConstPtr<T>)p; }

// value-only wave reductions and wave-uniform reads (used by the lazy argmin)
__device__ __forceinline__ double wave_min_f64(double x)
{
#define MMEE_STEP_(S)                                                                                   \
    {                                                                                                   \
        unsigned long long b = (unsigned long long)__double_as_longlong(x);                             \
        uint32_t lo = lane_exchange<S>((uint32_t)b), hi = lane_exchange<S>((uint32_t)(b >> 32));        \
        x = fmin(x, __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo)));            \
    }
    MMEE_STEP_(0) MMEE_STEP_(1) MMEE_STEP_(2) MMEE_STEP_(3) MMEE_STEP_(4) MMEE_STEP_(5)
#undef MMEE_STEP_
    return x;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x)
{
    x = min(x, lane_exchange<0>(x)); x = min(x, lane_exchange<1>(x)); x = min(x, lane_exchange<2>(x));
    x = min(x, lane_exchange<3>(x)); x = min(x, lane_exchange<4>(x)); x = min(x, lane_exchange<5>(x));
    return x;
}

// lane l's value of x, l wave-uniform
__device__ __forceinline__ double lane_value_f64(double x, uint32_t l)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), (int)l), hi = __builtin_amdgcn_readlane(__double2hiint(x), (int)l);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double uniform_f64(double x)
{
    unsigned long long b = (unsigned long long)__double_as_longlong(x);
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// ---------------------------------------------------------------------------
// offline stage: the query side

// the 24 inter-tile loop orders, outer -> inner, in lexicographic order over i<k<l<j;
// 2 bits per slot, slot 0 = outermost
__device__ __forceinline__ uint32_t order_of_rank(uint32_t rank)
{
    uint32_t avail = 0xE4;            // nibble list 3,2,1,0 packed 2 bits each: entry e at bits 2e
    uint32_t packed = 0;
    uint32_t f = 6, left = 4;
    for (uint32_t slot = 0; slot < 4; ++slot) {
        uint32_t pick = rank / f;
        rank -= pick * f;
        uint32_t sym = (avail >> (2 * pick)) & 3;
        packed |= sym << (2 * slot);
        // delete entry `pick` from the list
        uint32_t low = avail & ((1u << (2 * pick)) - 1);
        uint32_t high = (avail >> (2 * pick + 2)) << (2 * pick);
        avail = low | high;
        --left;
        if (left) f /= left;
    }
    return packed;
}

// selector of a DRAM term: which of the two loops an operand does not own multiply its
// matrix size.  nest_mask: loops of the operand's operator nest; own0/own1: its own dims;
// n0/n1: the other two dims in table order.
__device__ __forceinline__ uint32_t dram_selector(const int pos[4], uint32_t nest_mask, uint32_t prefix_mask,
                                                  int own0, int own1, int n0, int n1, int level)
{
    // blocker: innermost own loop outside the buffering level (Sec. V-A)
    int bpos = 99, bdim = -1;
    if (pos[own0] >= level) { bpos = pos[own0]; bdim = own0; }
    if (pos[own1] >= level && pos[own1] < bpos) { bpos = pos[own1]; bdim = own1; }
    if (bdim < 0) return 0;                                   // whole matrix resident: fetched once
    uint32_t counted;
    if (level == 0 && ((prefix_mask >> bdim) & 1)) {
        counted = prefix_mask;                                // evicted at every operator switch
    } else {
        counted = 0;                                          // Scenario 1: blocker and all loops above it
        for (int q = 0; q < 4; ++q)
            if (((nest_mask >> q) & 1) && pos[q] >= bpos) counted |= 1u << q;
    }
    return ((counted >> n0) & 1) | (((counted >> n1) & 1) << 1);
}

__global__ void k_build_rows(uint4 *enc, uint32_t *sig)
{
    uint32_t row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= N_DFROWS) return;
    uint32_t x = row;
    int lvl[5];
    lvl[OA] = x % 5; x /= 5;
    lvl[OB] = x % 5; x /= 5;
    lvl[OD] = x % 5; x /= 5;
    lvl[OE] = x % 5; x /= 5;
    lvl[OC] = 0;
    uint32_t rank = x % 24; x /= 24;
    uint32_t r = x & 1, f = x >> 1;

    uint32_t ord = order_of_rank(rank);
    int pos[4];
    for (int slot = 0; slot < 4; ++slot) pos[(ord >> (2 * slot)) & 3] = 3 - slot;

    // loops iterated by both operators lead the nest (Sec. IV-B); the rest splits per operator
    uint32_t shared_mask = (1u << DI) | (1u << DL) | (r ? (1u << DJ) : 0u);
    uint32_t prefix_mask = 0;
    for (int slot = 0; slot < 4; ++slot) {
        uint32_t q = (ord >> (2 * slot)) & 3;
        if (!((shared_mask >> q) & 1)) break;
        prefix_mask |= 1u << q;
    }
    uint32_t nest1 = prefix_mask | (1u << DI) | (1u << DK) | (1u << DL);
    uint32_t nest2 = prefix_mask | (1u << DI) | (1u << DL) | (1u << DJ);

    const int own[5][2] = {{DI, DK}, {DK, DL}, {DI, DL}, {DL, DJ}, {DI, DJ}};
    uint32_t bs_sel[5];
    for (int X = 0; X < 5; ++X) {
        if (X == OC) continue;
        bs_sel[X] = (uint32_t)(pos[own[X][0]] < lvl[X]) | ((uint32_t)(pos[own[X][1]] < lvl[X]) << 1);
    }
    // C holds every tile the producer finishes before the consumer starts (fused), else one tile
    bs_sel[OC] = f ? ((uint32_t)!((prefix_mask >> DI) & 1) | ((uint32_t)!((prefix_mask >> DL) & 1) << 1)) : 0u;
    // retained operands (buffered at an inter-tile loop) also occupy the other operator's buffer
    const int ret[4] = {OA, OB, OD, OE};
    uint32_t tau_bits = 0, ret_sel[4];
    for (int y = 0; y < 4; ++y) {
        bool tau = lvl[ret[y]] >= 1;
        tau_bits |= (uint32_t)tau << y;
        ret_sel[y] = tau ? bs_sel[ret[y]] : 4u;
    }
    uint32_t da_sel[4];
    da_sel[0] = dram_selector(pos, nest1, prefix_mask, DI, DK, DL, DJ, lvl[OA]);
    da_sel[1] = dram_selector(pos, nest1, prefix_mask, DK, DL, DI, DJ, lvl[OB]);
    da_sel[2] = dram_selector(pos, nest2, prefix_mask, DL, DJ, DI, DK, lvl[OD]);
    da_sel[3] = dram_selector(pos, nest2, prefix_mask, DI, DJ, DK, DL, lvl[OE]);
    uint32_t dac_sel = 0, dac_opt = 4;                        // fused: DA_C = 0 (Sec. V-C)
    if (!f) {
        uint32_t out_k = dram_selector(pos, nest1, prefix_mask, DI, DL, DK, DJ, 0) & 1;
        uint32_t in_j = (dram_selector(pos, nest2, prefix_mask, DI, DL, DK, DJ, 0) >> 1) & 1;
        dac_sel = dac_opt = out_k | (in_j << 1);
    }
    // recomputation must revisit C tiles (j outside k) and needs an on-chip C
    bool valid = !(r && (!f || pos[DK] > pos[DJ]));
    uint8_t sel[16];
    sel[0] = (uint8_t)(ENT_BS_AB + bs_sel[OA] + 4 * bs_sel[OB]);
    sel[1] = (uint8_t)(ENT_RET_DE + ret_sel[2] + 5 * ret_sel[3]);
    sel[2] = (uint8_t)(ENT_BS_C + bs_sel[OC]);
    sel[3] = (uint8_t)(ENT_BS_DE + bs_sel[OD] + 4 * bs_sel[OE]);
    sel[4] = (uint8_t)(ENT_RET_AB + ret_sel[0] + 5 * ret_sel[1]);
    sel[5] = (uint8_t)(ENT_DA_AB + da_sel[0] + 4 * da_sel[1]);
    sel[6] = (uint8_t)(ENT_DA_DE + da_sel[2] + 4 * da_sel[3]);
    sel[7] = (uint8_t)(ENT_DA_C + dac_opt);
    sel[ROW_FLAGS] = (uint8_t)((valid ? 1u : 0u) | (r << 1) | (f << 2));
    for (int k = ROW_FLAGS + 1; k < 16; ++k) sel[k] = 0;

    uint4 packed;
    packed.x = sel[0] | (sel[1] << 8) | (sel[2] << 16) | ((uint32_t)sel[3] << 24);
    packed.y = sel[4] | (sel[5] << 8) | (sel[6] << 16) | ((uint32_t)sel[7] << 24);
    packed.z = sel[8] | (sel[9] << 8) | (sel[10] << 16) | ((uint32_t)sel[11] << 24);
    packed.w = sel[12] | (sel[13] << 8) | (sel[14] << 16) | ((uint32_t)sel[15] << 24);
    enc[row] = packed;

    // symbolic signature: one bit per optional factor of every term; a row whose bits are a
    // subset of another's is no larger in any term, for every tiling (all factors are >= 1)
    uint32_t s = 0;
    for (int X = 0; X < 5; ++X) s |= bs_sel[X] << (2 * X);
    s |= tau_bits << 10;
    for (int y = 0; y < 4; ++y) s |= da_sel[y] << (14 + 2 * y);
    s |= dac_sel << 22;
    sig[row] = valid ? s : 0xFFFFFFFFu;
}

// Eq. (12) in a form that also protects index ties: row v goes if some row u of its group with a
// lower row id is term-wise no larger.  flags[v]: bit0 = denotes a dataflow, bit1 = survives.
__global__ void k_prune_rows(const uint32_t *__restrict__ sig, uint8_t *flags)
{
    __shared__ uint32_t s_sig[ROWS_PER_GROUP];
    const uint32_t g = blockIdx.y;
    for (uint32_t a = threadIdx.x; a < ROWS_PER_GROUP; a += blockDim.x) s_sig[a] = sig[g * ROWS_PER_GROUP + a];
    __syncthreads();
    uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= ROWS_PER_GROUP) return;
    uint32_t sv = s_sig[v];
    bool valid = sv != 0xFFFFFFFFu;
    bool dominated = false;
    if (valid) {
        uint32_t nv = ~sv;
        for (uint32_t u = 0; u < v; ++u) {
            if ((s_sig[u] & nv) == 0) { dominated = true; break; }
        }
    }
    flags[g * ROWS_PER_GROUP + v] = (uint8_t)((valid ? 1u : 0u) | ((valid && !dominated) ? 2u : 0u));
}

// Stable compaction of the rows whose flag bit `which` is set: wave ballot for the position
// inside the wave, LDS prefix over the waves of the block.  One block per (list, group).
__global__ void k_compact_rows(const uint8_t *__restrict__ flags, const uint4 *__restrict__ enc, uint32_t *rows_valid,
                               uint32_t *rows_kept, uint4 *enc_valid, uint4 *enc_kept, uint32_t *counts)
{
    __shared__ uint32_t wave_cnt[16];
    __shared__ uint32_t running;
    const uint32_t g = blockIdx.x & 3, which = blockIdx.x >> 2;
    uint32_t *out = (which ? rows_kept : rows_valid) + g * ROWS_PER_GROUP;
    // the encoded rows in list order, row number in the spare word: one load per lane and item
    uint4 *out_enc = (which ? enc_kept : enc_valid) + g * ROWS_PER_GROUP;
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    if (threadIdx.x == 0) running = 0;
    __syncthreads();
    for (uint32_t start = 0; start < ROWS_PER_GROUP; start += blockDim.x) {
        uint32_t row = start + threadIdx.x;
        bool on = row < ROWS_PER_GROUP && ((flags[g * ROWS_PER_GROUP + row] >> which) & 1);
        unsigned long long mask = __ballot(on);
        uint32_t before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        uint32_t base = running;
        for (uint32_t wv = 0; wv < wave; ++wv) base += wave_cnt[wv];
        if (on) {
            const uint32_t dfrow = g * ROWS_PER_GROUP + row;
            uint4 e = enc[dfrow];
            e.w = dfrow;
            out[base + before] = dfrow;
            out_enc[base + before] = e;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t tot = 0;
            for (uint32_t wv = 0; wv < nwaves; ++wv) tot += wave_cnt[wv];
            running += tot;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) counts[blockIdx.x] = running;
}

// ---------------------------------------------------------------------------
// online stage: the boundary side

// tile extents are 32-bit; only the column capacity C*g can exceed 32 bits (then one fold suffices)
__device__ __forceinline__ uint64_t cdiv(uint32_t a, uint64_t b) { return b > a ? 1u : (a - 1u) / (uint32_t)b + 1u; }

// words crossing buffer<->RF and cycles of one tile matmul m x r x n; mode 0 WS, 1 IS, 2 OS
__device__ __forceinline__ void tile_cost(uint32_t m, uint32_t r, uint32_t n, int mode, uint32_t R, uint32_t C,
                                          uint32_t g, uint64_t &words, uint64_t &cycles)
{
    uint32_t rows_dim = mode == 0 ? r : m;                 // spread over PE rows
    uint32_t cols_dim = mode == 1 ? r : n;                 // spread over PE columns
    uint64_t time_dim = mode == 0 ? m : (mode == 1 ? n : r);
    uint64_t row_folds = cdiv(rows_dim, R);
    words = (uint64_t)rows_dim * cols_dim + time_dim * rows_dim * cdiv(cols_dim, (uint64_t)C * g) +
            time_dim * cols_dim * row_folds;
    cycles = row_folds * cdiv(cols_dim, C) * time_dim;
}

// Five threads per tiling (one wave per share of the entries, 64 tilings per block): decode the four
// tiling digits, derive the boundary vector and store the subset products a row may select
// (entry-major, coalesced in the tiling).  The grid covers the padded width mc.tpad.
constexpr int BUILD_PARTS = 5;
__global__ __launch_bounds__(64 * BUILD_PARTS) void k_build_tilings(DivTable dv, ModelConst mc, double *__restrict__ btab,
                                                                    double *__restrict__ ctab_s, uint64_t *__restrict__ ctab_e,
                                                                    DivTable *__restrict__ dv_copy)
{
    const uint32_t t = blockIdx.x * 64 + (threadIdx.x & 63);
    const uint32_t part = threadIdx.x >> 6;
    // leave the divisor lists in device memory for the search's final record (index -> mapping)
    if (dv_copy && blockIdx.x == 0) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&dv);
        uint32_t *dst = reinterpret_cast<uint32_t *>(dv_copy);
        for (uint32_t a = threadIdx.x; a < sizeof(DivTable) / 4; a += blockDim.x) dst[a] = src[a];
    }
    if (t >= mc.tpad) return;
    // the columns between the last tiling and the padded width repeat the last tiling (the search
    // takes tilings in groups)
    const bool padding = t >= mc.T;
    uint64_t G[4], D[4];
    uint32_t x = padding ? mc.T - 1 : t;
    for (int q = 0; q < 4; ++q) {
        uint32_t digit = x % dv.ndiv[q];
        x /= dv.ndiv[q];
        G[q] = dv.div[q][digit];
        D[q] = dv.X[q] / (uint32_t)G[q];
    }
    const uint64_t tp = mc.tpad;
    const uint64_t BH = (uint64_t)mc.BH;
    if (part == 0 || part == 2) {
        const int own[5][2] = {{DI, DK}, {DK, DL}, {DI, DL}, {DL, DJ}, {DI, DJ}};
        uint64_t bs[5][5];                                       // option 4 = absent
        for (int X = 0; X < 5; ++X) {
            uint64_t tile = G[own[X][0]] * G[own[X][1]];
            uint64_t d0 = D[own[X][0]], d1 = D[own[X][1]];
            bs[X][0] = tile; bs[X][1] = tile * d0; bs[X][2] = tile * d1; bs[X][3] = tile * d0 * d1;
            bs[X][4] = 0;
        }
        if (part == 0) {
            for (int b = 0; b < 4; ++b)
                for (int a = 0; a < 4; ++a) {
                    btab[(ENT_BS_AB + a + 4 * b) * tp + t] = (double)(bs[OA][a] + bs[OB][b]);
                    btab[(ENT_BS_DE + a + 4 * b) * tp + t] = (double)(bs[OD][a] + bs[OE][b]);
                }
            for (int c = 0; c < 4; ++c) btab[(ENT_BS_C + c) * tp + t] = (double)bs[OC][c];
            // unfused C: spilled by Op1, fetched by Op2, plus one softmax pass over S and P
            uint64_t whole = (uint64_t)dv.X[DI] * dv.X[DL];
            for (uint32_t c = 0; c < 4; ++c) {
                uint64_t spill = (c & 1) ? D[DK] : 1, fetch = (c & 2) ? D[DJ] : 1;
                btab[(ENT_DA_C + c) * tp + t] = (double)(BH * whole * (spill + fetch + 2));
                btab[(ENT_DA_C + ENT_RAW_DA + c) * tp + t] = (double)(whole * (spill + fetch + 2));
            }
            btab[(ENT_DA_C + 4) * tp + t] = 0.0;
            btab[(ENT_DA_C + ENT_RAW_DA + 4) * tp + t] = 0.0;
        } else {
            for (int b = 0; b < 5; ++b)
                for (int a = 0; a < 5; ++a) {
                    btab[(ENT_RET_DE + a + 5 * b) * tp + t] = (double)(bs[OD][a] + bs[OE][b]);
                    btab[(ENT_RET_AB + a + 5 * b) * tp + t] = (double)(bs[OA][a] + bs[OB][b]);
                }
        }
        return;
    }
    if (part == 1) {
        const int da_own[4][2] = {{DI, DK}, {DK, DL}, {DL, DJ}, {DI, DJ}};
        const int da_other[4][2] = {{DL, DJ}, {DI, DJ}, {DI, DK}, {DK, DL}};
        uint64_t da[4][4];
        for (int y = 0; y < 4; ++y) {
            uint64_t whole = (uint64_t)dv.X[da_own[y][0]] * dv.X[da_own[y][1]];
            uint64_t n0 = D[da_other[y][0]], n1 = D[da_other[y][1]];
            da[y][0] = whole; da[y][1] = whole * n0; da[y][2] = whole * n1; da[y][3] = whole * n0 * n1;
        }
        for (int b = 0; b < 4; ++b)
            for (int a = 0; a < 4; ++a) {
                btab[(ENT_DA_AB + a + 4 * b) * tp + t] = (double)(BH * (da[0][a] + da[1][b]));
                btab[(ENT_DA_DE + a + 4 * b) * tp + t] = (double)(BH * (da[2][a] + da[3][b]));
                btab[(ENT_DA_AB + ENT_RAW_DA + a + 4 * b) * tp + t] = (double)(da[0][a] + da[1][b]);
                btab[(ENT_DA_DE + ENT_RAW_DA + a + 4 * b) * tp + t] = (double)(da[2][a] + da[3][b]);
            }
        return;
    }
    if (padding) return;

    // parts 3 and 4 (r = 0 / 1), stationary-mode dependent: buffer<->RF words and cycles per tile stage
    uint64_t br1[3], cy1[3], br2[3], cy2[3];
    for (int s = 0; s < 3; ++s) {
        tile_cost((uint32_t)G[DI], (uint32_t)G[DK], (uint32_t)G[DL], s, mc.pe_rows, mc.pe_cols, mc.g_words, br1[s], cy1[s]);
        tile_cost((uint32_t)G[DI], (uint32_t)G[DL], (uint32_t)G[DJ], s, mc.pe_rows, mc.pe_cols, mc.g_words, br2[s], cy2[s]);
    }
    const uint64_t I = dv.X[DI], K = dv.X[DK], L = dv.X[DL], J = dv.X[DJ];
    {
        const uint32_t r = part - 3;
        uint64_t rho = r ? D[DJ] : 1;                         // producer repeated per j tile (Sec. V-D)
        uint64_t st1 = rho * D[DI] * D[DK] * D[DL], st2 = D[DI] * D[DL] * D[DJ];
        uint64_t mac = rho * I * K * L + I * L * J;
        uint64_t sm = rho * I * L;
        double *cs = ctab_s + ((uint64_t)t * 2 + r) * NCS;
        const double e_rf_part = mc.e_rf * (double)(BH * 3 * mac);
        const double e_mac_part = mc.e_mac * (double)(BH * (mac + (uint64_t)mc.c_softmax * sm));
        cs[18] = e_rf_part;
        cs[19] = e_mac_part;
        for (uint32_t c9 = 0; c9 < 9; ++c9) {
            uint32_t s1 = c9 % 3, s2 = c9 / 3;
            uint64_t br = st1 * br1[s1] + st2 * br2[s2];
            uint64_t cyc = st1 * cy1[s1] + st2 * cy2[s2];
            double t_gb = mc.gb_bw > 0.0 ? (double)(br * (uint64_t)mc.word) / mc.gb_bw : 0.0;
            const double c_lat_part = mc.c_lat * fmax((double)cyc, t_gb);
            cs[c9] = mc.regroup ? (mc.e_gb * (double)(BH * br) + e_rf_part) + e_mac_part : (double)(BH * br);
            cs[9 + c9] = c_lat_part;
            ctab_e[((uint64_t)r * NCE + c9) * tp + t] = br;
            ctab_e[((uint64_t)r * NCE + 9 + c9) * tp + t] = cyc;
            ctab_e[((uint64_t)r * NCE + 20 + c9) * tp + t] = (uint64_t)__double_as_longlong(c_lat_part);
        }
        ctab_e[((uint64_t)r * NCE + 18) * tp + t] = mac;
        ctab_e[((uint64_t)r * NCE + 19) * tp + t] = sm;
        ctab_e[((uint64_t)r * NCE + 29) * tp + t] = (uint64_t)__double_as_longlong(e_rf_part);
        ctab_e[((uint64_t)r * NCE + 30) * tp + t] = (uint64_t)__double_as_longlong(e_mac_part);
    }
}

// ---------------------------------------------------------------------------
// one candidate, complete (shared by k_eval_batch and by the search's final record)

struct EvalArgs {
    const uint4 *enc;
    const double *btab;
    const uint64_t *ctab_e;
    ModelConst mc;
};

__device__ __forceinline__ uint32_t sel_of(const uint4 &e, int k)
{
    uint32_t w = k < 4 ? e.x : (k < 8 ? e.y : (k < 12 ? e.z : e.w));
    return (w >> (8 * (k & 3))) & 0xFF;
}

// One candidate from the global tables.  The tables are read-only while this runs, so they are
// read through the constant address space: with a wave-uniform row the selectors land in scalar
// registers and each table read is one load at (uniform base + lane's tiling).
__device__ __forceinline__ void eval_candidate(const EvalArgs &a, uint32_t row, uint32_t t, mmee_cost &c)
{
    // row = levels/order (15000) + 15000 r + 30000 s1 + 90000 s2 + 270000 f
    uint32_t lo = row % 15000, hi = row / 15000;
    uint32_t r = hi & 1; hi >>= 1;
    uint32_t s1 = hi % 3; hi /= 3;
    uint32_t s2 = hi % 3; uint32_t f = hi / 3;
    ConstPtr<uint32_t> ew = as_constant(reinterpret_cast<const uint32_t *>(a.enc + lo + ROWS_PER_GROUP * (r + 2 * f)));
    uint4 e;
    e.x = ew[0]; e.y = ew[1]; e.z = ew[2]; e.w = ew[3];
    uint32_t flags = sel_of(e, ROW_FLAGS);
    if (!(flags & 1)) {
        c.bs_words = c.da_words = c.br_words = c.mac_total = c.comp_cycles = 0;
        c.energy_pj = pos_inf(); c.latency_cycles = pos_inf();
        c.valid = 0; c.reason = 1;
        return;
    }
    const uint64_t tp = a.mc.tpad;
    ConstPtr<double> bt = as_constant(a.btab);
    ConstPtr<uint64_t> ce = as_constant(a.ctab_e) + (uint64_t)r * NCE * tp;
    double v[NSEL];
#pragma unroll
    for (int k = 0; k < 5; ++k) v[k] = bt[sel_of(e, k) * tp + t];
#pragma unroll
    for (int k = 5; k < NSEL; ++k) v[k] = bt[(sel_of(e, k) + ENT_RAW_DA) * tp + t];
    uint32_t c9 = s1 + 3 * s2;
    uint64_t br = ce[(uint64_t)c9 * tp + t];
    uint64_t cyc = ce[(uint64_t)(9 + c9) * tp + t];
    uint64_t mac = ce[18ull * tp + t];
    double lat_part = __longlong_as_double((long long)ce[(uint64_t)(20 + c9) * tp + t]);
    double e_rf_part = __longlong_as_double((long long)ce[29ull * tp + t]);
    double e_mac_part = __longlong_as_double((long long)ce[30ull * tp + t]);
    // Eq. (1), (2), (4), (7)
    double bs = fmax(v[0] + v[2] + v[1], v[3] + v[2] + v[4]);
    double da = v[5] + v[6] + v[7];
    c.bs_words = (uint64_t)bs; c.da_words = (uint64_t)da; c.br_words = br;
    c.mac_total = mac; c.comp_cycles = cyc;
    if (bs > a.mc.cap_words) {
        c.energy_pj = pos_inf(); c.latency_cycles = pos_inf();
        c.valid = 0; c.reason = 2;
        return;
    }
    const double BH = a.mc.BH;
    double en = a.mc.e_dram * (BH * da);
    en = en + a.mc.e_gb * (BH * (da + (double)br));
    en = en + e_rf_part;
    en = en + e_mac_part;
    // c * max(max(comp, dram), gb) = max(c * dram, c * max(comp, gb)): scaling by c >= 0 and max commute exactly
    double l_dram;
    if (a.mc.bw_pow2) l_dram = da * a.mc.eval_k;
    else l_dram = (da * a.mc.word) / a.mc.dram_bw;
    c.energy_pj = en;
    c.latency_cycles = fmax(a.mc.c_lat * l_dram, lat_part);
    c.valid = 1; c.reason = 0;
}

__device__ __forceinline__ void decode_candidate(const DivTable &dv, uint32_t T, uint64_t idx, mmee_mapping &m)
{
    uint32_t t = (uint32_t)(idx % T);
    uint32_t row = (uint32_t)(idx / T);
    m.idx = idx;
    for (int q = 0; q < 4; ++q) {
        uint32_t digit = t % dv.ndiv[q];
        t /= dv.ndiv[q];
        m.xG[q] = dv.div[q][digit];
        m.xD[q] = dv.X[q] / m.xG[q];
    }
    for (int y = 0; y < 4; ++y) { m.level[y] = (uint8_t)(row % 5); row /= 5; }
    uint32_t ord = order_of_rank(row % 24); row /= 24;
    for (int slot = 0; slot < 4; ++slot) m.order[slot] = (uint8_t)((ord >> (2 * slot)) & 3);
    m.recompute = (uint8_t)(row & 1); row >>= 1;
    m.stat1 = (uint8_t)(row % 3); row /= 3;
    m.stat2 = (uint8_t)(row % 3); row /= 3;
    m.fused = (uint8_t)row;
}

__global__ void k_decode(DivTable dv, uint32_t T, const uint64_t *__restrict__ idx, uint64_t n, mmee_mapping *out)
{
    uint64_t a = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= n) return;
    mmee_mapping m;
    decode_candidate(dv, T, idx[a], m);
    out[a] = m;
}

// One candidate per thread; records leave through LDS so that every store instruction of a wave
// writes one contiguous kilobyte; the stores are streaming (nothing reads the records back on the
// device).
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// Work unit = one 4 KiB page of the output: 64 consecutive candidates, one wave.  Almost every page
// lies inside one index row (all its candidates share order, levels and options), so the row decode
// is wave-uniform; a page that straddles rows takes them one after the other.
// Pages are dealt so that all pages of a block are congruent to the block number modulo 8: blocks go
// round the eight XCDs, and an XCD that keeps to every eighth page writes at a measurably higher rate
// than one whose pages lie side by side (6.7 against 6.0 TB/s for plain 4 KiB stores).
__global__ __launch_bounds__(256) void k_eval_batch(EvalArgs a, uint32_t row_first, uint32_t t_first, uint32_t n, uint32_t n_pages,
                                                    v4u *__restrict__ out)
{
    // record 0 of this launch is candidate row_first * T + t_first; n < 2^31 records per launch keep
    // every tiling offset below 2^32
    __shared__ v4u stage[4][256];                             // [wave][64 records x 4 pieces]
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform on purpose
    const uint32_t page = 32u * (blockIdx.x / 8u) + 8u * wave + blockIdx.x % 8u;
    if (page >= n_pages) return;
    const uint32_t rec0 = page * 64u;
    const bool on = rec0 + lane < n;
    // the page's first candidate, then each lane's own row and tiling
    const uint32_t T = a.mc.T;
    const uint32_t off0 = t_first + rec0;                     // tilings from the start of row_first
    const uint32_t row0 = row_first + off0 / T, x = off0 % T + lane;
    uint32_t my_row, my_t;
    if (T >= 64u) { const bool next = x >= T; my_row = row0 + next; my_t = next ? x - T : x; }
    else { my_row = row0 + x / T; my_t = x % T; }
    const uint32_t row_last = __builtin_amdgcn_readfirstlane(row0 + (off0 % T + 63u) / T);
    for (uint32_t row = __builtin_amdgcn_readfirstlane(row0); row <= row_last; ++row) {
        if (on && my_row == row) {
            mmee_cost c;
            eval_candidate(a, row, my_t, c);
            const v4u *src = reinterpret_cast<const v4u *>(&c);
#pragma unroll
            for (int k = 0; k < 4; ++k) stage[wave][lane * 4 + k] = src[k];
        }
    }
    // only this wave touches stage[wave]: order its LDS writes before its LDS reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // lane L moves piece (L & 3) of record 16 k + L / 4 on pass k
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t rec = 16 * k + (lane >> 2);
        if (rec0 + rec < n) __builtin_nontemporal_store(stage[wave][rec * 4 + (lane & 3)], &out[(rec0 + rec) * 4 + (lane & 3)]);
    }
}

// ---------------------------------------------------------------------------
// the search kernel

struct SearchArgs {
    const uint4 *enc;            // encoded rows
    const uint32_t *rows;        // compacted row ids, one list per (r, f) group
    const uint4 *row_enc;        // their encoded rows in the same order, row id in .w
    // Rows are handed out per recomputation class r: the lists of (r, f=0) and (r, f=1) follow each
    // other in one slot numbering, so that a row block may hold rows of both.
    uint32_t cls_off[2][2];      // [r][f] start of the group's list inside rows[]
    uint32_t cls_cnt[2][2];      // [r][f] rows in it
    uint32_t rb_split;           // row blocks of class r = 0; the rest belong to r = 1
    // A class of at most 256 rows (the pruned lists) is one row block whose waves share the work
    // differently: wave_split[r] = S > 1 means the rows fill 8 / S waves and each of them comes S
    // times, once per S-th of the item's tilings.  S = 1: one row per thread, all tilings.
    uint32_t wave_split[2];
    uint32_t n_rb;               // row blocks in all
    // Tilings [0, n_cc * TC) are cut into chunks of TC, the rest into n_fc chunks of TC_FINE.  Items
    // [0, n_coarse_items) are the (row block, coarse chunk) pairs, the fine ones follow: the short
    // items are handed out last and even out the moment at which the persistent blocks run dry.
    uint32_t n_cc, n_fc;
    uint32_t n_coarse_items;
    uint32_t n_items;
    // k_search_dense: the (order, r, f) classes that denote dataflows (order + 24 * (r + 2 f)),
    // and the split of its items: chunks [0, d_ncc) are handed out as groups of whole tasks
    // (d_gc groups per chunk), the chunks after them as groups of fifths of tasks (d_gf per chunk)
    const uint32_t *cls;
    uint32_t n_cls;
    uint32_t d_ncc, d_gc, d_gf;
    const double *btab;
    const double *ctab_s;
    ModelConst mc;
    Key *partials;               // [gridDim.x][N_OBJ]
    uint32_t *ticket;
    uint32_t *work_counter;
    FinalRecord *final_out;      // [N_OBJ]
    double e_limit;              // LIMIT kernels only: candidates with energy >= e_limit are left out
    Key *final_key_dev;          // [N_OBJ] the winning keys once more, in device memory, for a pass that follows
    const Key *lat_cap;          // LATCAP kernels only: candidates with a latency above lat_cap->p are left out
    const uint64_t *ctab_e;
    DivTable const *dv;          // device copy, for the final record's mapping
    // k_search_dense, scalar keys: per key the lowest value any wave of the launch has recorded so far, as
    // the bit pattern of the (non-negative) double; +inf between launches.  Null: no sharing between blocks.
    unsigned long long *hints;
};

constexpr unsigned long long INF_BITS = 0x7ff0000000000000ull;

constexpr int BLOCKS_PER_CU = 2;       // what LDS (64 KB per block) lets a CU hold
constexpr int TC = 64;                 // tilings per coarse item
constexpr int TC_FINE = 32;            // tilings per fine item
constexpr int SEARCH_THREADS = 512;


// The staged table keeps the global layout, entry-major: the tilings of an entry are consecutive and
// an entry's line is padded to LDS_ENT values, which spreads the entries over the banks.  One address
// register per selector and the immediate offsets of a paired read then reach the tilings of a whole
// loop turn.  LDS access goes through explicit 32-bit addresses.
constexpr int LDS_ENT = 65;            // TC tilings + 1
constexpr int TURN = 8;                // tilings per loop turn
typedef const double __attribute__((address_space(3))) *LdsF64;
__device__ __forceinline__ uint32_t lds_address(const double *p)
{
    return (uint32_t)(uintptr_t)(LdsF64)p;
}
// tilings tl and tl + 1 (tl a constant after unrolling) of the entry at addr
__device__ __forceinline__ void read_tilings(uint32_t &addr, int tl, double &first, double &second)
{
    asm("" : "+v"(addr));                         // one register, two constant offsets
    LdsF64 p = (LdsF64)(uintptr_t)addr;
    first = p[tl];
    second = p[tl + 1];
}

// What a work item covers: the recomputation class r, the tilings [t0, t0 + nt) and, per thread,
// one dataflow row (live = false for the padding lanes of a class's last row block).
struct ItemView {
    uint32_t r, t0, nt;
    uint32_t tl_lo, tl_hi;       // this wave's share of the tilings [0, nt rounded up to whole turns)
    uint32_t dfrow;
    uint4 e;                     // the row's selectors
    bool live, fine;
};

__device__ __forceinline__ ItemView locate_item(const SearchArgs &a, uint32_t item)
{
    ItemView v;
    uint32_t rb;
    v.fine = item >= a.n_coarse_items;
    // neighbouring items share their tilings: blocks that run side by side read the same table slice
    // and the same per-tiling constants
    if (!v.fine) {
        rb = item % a.n_rb;
        v.t0 = (item / a.n_rb) * TC;
        v.nt = TC;
    } else {
        const uint32_t j = item - a.n_coarse_items;
        rb = j % a.n_rb;
        v.t0 = a.n_cc * TC + (j / a.n_rb) * TC_FINE;
        v.nt = min((uint32_t)TC_FINE, a.mc.T - v.t0);
    }
    v.r = rb >= a.rb_split;
    const uint32_t n0 = a.cls_cnt[v.r][0], n1 = a.cls_cnt[v.r][1];
    const uint32_t turns = (v.nt + TURN - 1) / TURN;
    const uint32_t split = a.wave_split[v.r];
    uint32_t slot;
    if (split > 1) {
        // waves_for_rows waves hold the rows; wave w takes row group w % waves_for_rows and the
        // (w / waves_for_rows)-th share of the turns
        const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        const uint32_t waves_for_rows = (n0 + n1 + 63) / 64;
        const uint32_t share = wave / waves_for_rows;
        slot = share < split ? (wave % waves_for_rows) * 64 + lane : 0xFFFFFFFFu;
        v.tl_lo = min(share, split) * turns / split * TURN;
        v.tl_hi = min(share + 1, split) * turns / split * TURN;
    } else {
        slot = (rb - (v.r ? a.rb_split : 0u)) * SEARCH_THREADS + threadIdx.x;
        v.tl_lo = 0;
        v.tl_hi = turns * TURN;
    }
    v.live = slot < n0 + n1 && v.tl_lo < v.tl_hi;
    const uint32_t where = !v.live ? a.cls_off[v.r][n0 ? 0 : 1]
                                   : (slot < n0 ? a.cls_off[v.r][0] + slot : a.cls_off[v.r][1] + (slot - n0));
    v.e = a.row_enc[where];
    v.dfrow = v.e.w;
    return v;
}

// the index row (Sec. VI-A numbering: levels, order, r, stationary modes, f) of a dataflow row's
// combination 0; dataflow rows are numbered levels/order + 15000 * (r + 2 f)
__device__ __forceinline__ uint32_t index_row_base(uint32_t dfrow)
{
    const uint32_t g = dfrow / ROWS_PER_GROUP;
    return dfrow % ROWS_PER_GROUP + 15000u * (g & 1) + 270000u * (g >> 1);
}

// Stage the tilings [t0, t0 + nt) of the boundary-side tables, entry-major in global memory and in
// LDS, two tilings per thread and turn (one 16-byte load, one paired LDS write).  PAIRS =
// tiling pairs per item.  nt is rounded up to whole loop turns: beyond the last tiling the global
// table repeats it up to its padded width (k_build_tilings), and a repeated tiling changes no minimum.
template <int PAIRS, int THREADS = SEARCH_THREADS>
__device__ __forceinline__ void stage_tables(const SearchArgs &a, double *tab, uint32_t t0, uint32_t nt)
{
    typedef double v2f64 __attribute__((ext_vector_type(2)));
    constexpr int TURNS = (NENT * PAIRS + THREADS - 1) / THREADS;
    const uint32_t rows = (nt + TURN - 1) / TURN * TURN;
    // the addresses are worked out anew for every item: kept across items they would cost registers
    uint32_t tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    // all loads first, then all LDS writes: one memory latency per item, not one per turn
    v2f64 two[TURNS];
#pragma unroll
    for (int k = 0; k < TURNS; ++k) {
        const uint32_t i = tid + k * THREADS;
        const uint32_t ent = i / PAIRS, tl = (i % PAIRS) * 2;
        two[k] = v2f64{0.0, 0.0};
        if (i < NENT * PAIRS && tl < rows)
            two[k] = *reinterpret_cast<const v2f64 *>(a.btab + (uint64_t)ent * a.mc.tpad + t0 + tl);
    }
#pragma unroll
    for (int k = 0; k < TURNS; ++k) {
        const uint32_t i = tid + k * THREADS;
        const uint32_t ent = i / PAIRS, tl = (i % PAIRS) * 2;
        if (i < NENT * PAIRS && tl < rows) {
            tab[ent * LDS_ENT + tl] = two[k].x;
            tab[ent * LDS_ENT + tl + 1] = two[k].y;
        }
    }
}

// s_waitcnt lgkmcnt(0) with the other counters left alone (vmcnt 63, expcnt 7)
__device__ __forceinline__ void wait_lds_and_scalar_loads() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// keeps the optimiser from sinking a select below the operations that consume its result
__device__ __forceinline__ void pin(double &x) { asm("" : "+v"(x)); }

// Block and grid stages of the argmin: the waves' LDS slots -> one record per block -> ticket;
// the last block to arrive reduces all records and writes the winner's cost and mapping.
template <int MASK, int THREADS = SEARCH_THREADS>
__device__ __forceinline__ void finish_grid(const SearchArgs &a, Key (*wave_best)[THREADS / 64],
                                            uint32_t *is_last_flag)
{
    const double inf = pos_inf();
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) {
            if (!((MASK >> o) & 1)) continue;
            Key k = wave_best[o][0];
            for (int wv = 1; wv < THREADS / 64; ++wv)
                if (key_less(wave_best[o][wv], k)) k = wave_best[o][wv];
            Key *dst = a.partials + (uint64_t)blockIdx.x * N_OBJ + o;
            __hip_atomic_store(&dst->idx, k.idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(reinterpret_cast<uint64_t *>(&dst->p), (uint64_t)__double_as_longlong(k.p),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(reinterpret_cast<uint64_t *>(&dst->s), (uint64_t)__double_as_longlong(k.s),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __threadfence();
        uint32_t ticket = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        *is_last_flag = ticket == gridDim.x - 1;
    }
    __syncthreads();
    if (!*is_last_flag) return;

    // the last block to finish reduces every block's record
    __threadfence();
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) {
        if (!((MASK >> o) & 1)) continue;
        Key k; k.p = inf; k.s = 0.0; k.idx = ~0ull;
        for (uint32_t b = threadIdx.x; b < gridDim.x; b += THREADS) {
            Key *src = a.partials + (uint64_t)b * N_OBJ + o;
            Key c;
            c.idx = __hip_atomic_load(&src->idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c.p = __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<uint64_t *>(&src->p),
                                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            c.s = __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<uint64_t *>(&src->s),
                                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if (key_less(c, k)) k = c;
        }
        k = wave_min(k);
        if (lane == 0) wave_best[o][wave] = k;
    }
    __syncthreads();
    if (threadIdx.x < N_OBJ && ((MASK >> threadIdx.x) & 1)) {
        const int o = threadIdx.x;
        Key k = wave_best[o][0];
        for (int wv = 1; wv < THREADS / 64; ++wv)
            if (key_less(wave_best[o][wv], k)) k = wave_best[o][wv];
        FinalRecord *fr = a.final_out + o;
        fr->key = k;
        if (a.final_key_dev) a.final_key_dev[o] = k;
        mmee_cost c;
        mmee_mapping m;
        if (k.p < inf) {
            EvalArgs ea;
            ea.enc = a.enc; ea.btab = a.btab; ea.ctab_e = a.ctab_e; ea.mc = a.mc;
            eval_candidate(ea, (uint32_t)(k.idx / a.mc.T), (uint32_t)(k.idx % a.mc.T), c);
            decode_candidate(*a.dv, a.mc.T, k.idx, m);
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
    if (threadIdx.x == 0) { *a.ticket = 0; *a.work_counter = 0; }   // ready for the next launch on this stream
    if (threadIdx.x < N_OBJ && a.hints) a.hints[threadIdx.x] = INF_BITS;
}

// MASK: bit0 energy, bit1 latency, bit2 latency-then-energy, bit3 energy-delay product (Sec. VII-K).
// FAST: DRAM bandwidth is 0 or a power of two and the array count is a power of two, so the
// DRAM latency term is one exact multiply of the table value; otherwise it is divided out.
//
// LIMIT: only candidates whose energy is below a.e_limit take part (one step of the Pareto walk).
// REGROUP: every term of the energy is an exact integer (ModelConst::regroup), so the sum is taken
// as (row, tiling) part + (tiling, combination) part; the bits are those of the general order.
//
// Persistent blocks (as many as the chip holds) pull work items from a global counter.  One item =
// SEARCH_THREADS rows of one recomputation class (lane = row) x up to TC consecutive tilings (loop).
constexpr int popcount4(int m) { return (m & 1) + ((m >> 1) & 1) + ((m >> 2) & 1) + ((m >> 3) & 1); }

template <int MASK, bool FAST, bool LIMIT = false, bool REGROUP = false>
__global__ __launch_bounds__(SEARCH_THREADS, (popcount4(MASK) >= 3 || (MASK & 4 && MASK != 4)) ? 2 : 4) void k_search(SearchArgs a)
{
    __shared__ double tab[NENT * LDS_ENT];
    __shared__ Key wave_best[N_OBJ][SEARCH_THREADS / 64];
    __shared__ uint32_t is_last;

    // Scalar keys (energy, latency, EDP) use the lazy argmin: the loop only tracks minima, and the
    // position of a minimum is recovered afterwards, for the rare item whose best value reaches the
    // wave's running best.  The lexicographic key and the bounded walk keep positions in the loop.
    constexpr bool LAZY = !(MASK & 4) && !LIMIT;

    const double inf = pos_inf();
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // wave_best[o][w]: best key of wave w over all items so far; only wave w touches its slot
    if (lane < N_OBJ) { wave_best[lane][wave].p = inf; wave_best[lane][wave].s = 0.0; wave_best[lane][wave].idx = ~0ull; }
    // lazy path: the wave's running best per key, wave-uniform
    double run_p[N_OBJ];
    uint64_t run_idx[N_OBJ];
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) { run_p[o] = inf; run_idx[o] = ~0ull; }

    // work items are handed out through a global counter; the first one is the block's own number.
    // Thread 0 asks for the next item while the current one is being processed.
    __shared__ uint32_t s_item;
    uint32_t upcoming = blockIdx.x;
    while (true) {
        if (threadIdx.x == 0) s_item = upcoming;
        __syncthreads();                          // also: the previous item's LDS readers are done
        const uint32_t item = s_item;
        if (item >= a.n_items) break;
        if (threadIdx.x == 0)
            upcoming = gridDim.x + __hip_atomic_fetch_add(a.work_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const ItemView it = locate_item(a, item);
        const bool live = it.live;
        const uint32_t dfrow = it.dfrow;
        const uint4 e = it.e;
        const uint32_t r = it.r, t0 = it.t0, nt = it.nt;
        // this wave's tilings of the chunk (all of them unless the class is a short list)
        const uint32_t tl_lo = __builtin_amdgcn_readfirstlane(it.tl_lo), tl_hi = __builtin_amdgcn_readfirstlane(it.tl_hi);
        if (it.fine) stage_tables<TC_FINE / 2>(a, tab, t0, nt);
        else stage_tables<TC / 2>(a, tab, t0, nt);
        __syncthreads();
        // a wave without a single row (the pruned lists are short) has nothing to cost; it meets the
        // others again at the barrier on top of the loop
        if (!__ballot(live)) continue;

        uint32_t off[NSEL];
#pragma unroll
        for (int k = 0; k < NSEL; ++k) off[k] = sel_of(e, k);

        // a lane without a row never passes the capacity test
        const double cap = live ? a.mc.cap_words : -1.0;
        double bestE[9], bestL[9], bestLE_l[9], bestLE_e[9], bestP[9];
        uint32_t codeE[9], codeL[9], codeLE[9], codeP[9];
#pragma unroll
        for (int c9 = 0; c9 < 9; ++c9) {
            bestE[c9] = bestL[c9] = bestLE_l[c9] = bestLE_e[c9] = bestP[c9] = inf;
            codeE[c9] = codeL[c9] = codeLE[c9] = codeP[c9] = 0;
        }

        // Software pipeline in explicit stages.  LDS reads and scalar loads share one counter and
        // scalar loads return out of order, so every wait drains both: requests are therefore issued
        // right after a wait and met by the next one, most of a tiling's arithmetic later.
        //   A  row part of both tilings of a pair (uses the table values read a pair ago)
        //   B  request the next pair's table values and the second tiling's constants (set Y)
        //   C  nine combinations of the first tiling (set X)          -> wait
        //   D  request the next pair's first tiling's constants (set X)
        //   E  nine combinations of the second tiling (set Y)         -> wait
        // Four pairs per loop turn: a paired LDS read reaches every tiling of the turn from one
        // address per selector through its immediate offsets, and the addresses move once a turn.
        ConstF64 cs_base = as_constant(a.ctab_s + ((uint64_t)t0 * 2 + r) * NCS);
        struct TilingConstants { double gb[9], lat[9], e_rf, e_mac; };
        auto request = [&](TilingConstants &c, uint32_t tl) {
            ConstF64 cs = cs_base + (uint64_t)(min(tl, nt - 1) * (2 * NCS));   // past the end: the last tiling again
#pragma unroll
            for (int q = 0; q < 9; ++q) { c.gb[q] = cs[q]; c.lat[q] = cs[9 + q]; }
            if constexpr (!REGROUP) { c.e_rf = cs[18]; c.e_mac = cs[19]; }
        };
        double v[2][NSEL];
        uint32_t sel_addr[NSEL];
#pragma unroll
        for (int k = 0; k < NSEL; ++k) sel_addr[k] = lds_address(tab + off[k] * LDS_ENT + tl_lo);
#pragma unroll
        for (int k = 0; k < NSEL; ++k) read_tilings(sel_addr[k], 0, v[0][k], v[1][k]);
        TilingConstants X, Y;
        request(X, tl_lo);

        // whole turns: the staged tilings beyond nt repeat the last one
        for (uint32_t tl8 = tl_lo; tl8 < tl_hi; tl8 += TURN) {
#pragma unroll
            for (int q = 0; q < TURN / 2; ++q) {
                const uint32_t tl_pair = tl8 + 2 * q;
                // ---- A
                double dram_words[2], e_dram_part[2], l_dram[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    // Eq. (1), (2), (4) and the capacity mask
                    double bs1 = v[u][0] + v[u][2] + v[u][1];
                    double bs2 = v[u][3] + v[u][2] + v[u][4];
                    bool ok = fmax(bs1, bs2) <= cap;
                    dram_words[u] = v[u][5] + v[u][6] + v[u][7];   // B*H * Eq. (7)
                    // regrouped: all of the energy that depends on the row, (e_dram + e_gb) * B*H * DA
                    e_dram_part[u] = (REGROUP ? a.mc.e_sum : a.mc.e_dram) * dram_words[u];
                    if constexpr (FAST) l_dram[u] = dram_words[u] * a.mc.dram_k;
                    else l_dram[u] = a.mc.dram_bw > 0.0 ? a.mc.c_lat * (((dram_words[u] / a.mc.BH) * a.mc.word) / a.mc.dram_bw) : 0.0;
                    // a candidate over capacity costs +inf: neither term is negative, so the larger
                    // of the term and (0 or +inf) is the term or +inf
                    const double over = __hiloint2double(ok ? 0 : 0x7ff00000, 0);
                    e_dram_part[u] = fmax(e_dram_part[u], over);
                    l_dram[u] = fmax(l_dram[u], over);
                    pin(e_dram_part[u]);
                    pin(l_dram[u]);
                }
                __builtin_amdgcn_sched_barrier(0);
                // ---- B: at the end of a turn the addresses move on, except on the last turn, which
                // reads its last pair again
                if (q < TURN / 2 - 1) {
#pragma unroll
                    for (int k = 0; k < NSEL; ++k) read_tilings(sel_addr[k], 2 * (q + 1), v[0][k], v[1][k]);
                } else {
                    const uint32_t step = tl8 + TURN < tl_hi ? TURN * 8 : (TURN - 2) * 8;
#pragma unroll
                    for (int k = 0; k < NSEL; ++k) sel_addr[k] += step;
#pragma unroll
                    for (int k = 0; k < NSEL; ++k) read_tilings(sel_addr[k], 0, v[0][k], v[1][k]);
                }
                request(Y, tl_pair + 1);
                __builtin_amdgcn_sched_barrier(0);

                auto combinations = [&](const TilingConstants &c, int u) {
                    const uint32_t tl = tl_pair + u;
                    const double dw = dram_words[u], edp_ = e_dram_part[u], ld = l_dram[u];
#pragma unroll
                    for (int c9 = 0; c9 < 9; ++c9) {
                        double en;
                        if constexpr (REGROUP) {
                            en = edp_ + c.gb[c9];                 // row part + tiling part, both exact
                        } else {
                            double gb_words = dw + c.gb[c9];
                            en = edp_ + a.mc.e_gb * gb_words;
                            en = en + c.e_rf;
                            en = en + c.e_mac;
                        }
                        double lat = fmax(ld, c.lat[c9]);
                        if constexpr (LIMIT) {
                            bool out_of_range = !(en < a.e_limit);
                            en = out_of_range ? inf : en;
                            lat = out_of_range ? inf : lat;
                        }
                        if constexpr (LAZY) {
                            if constexpr (MASK & 8) bestP[c9] = fmin(bestP[c9], en * lat);
                            if constexpr (MASK & 1) bestE[c9] = fmin(bestE[c9], en);
                            if constexpr (MASK & 2) bestL[c9] = fmin(bestL[c9], lat);
                            continue;
                        }
                        if constexpr (MASK & 8) {
                            double edp = en * lat;
                            bool lt = edp < bestP[c9];
                            bestP[c9] = fmin(bestP[c9], edp);
                            codeP[c9] = lt ? tl : codeP[c9];
                        }
                        if constexpr (MASK & 1) {
                            bool lt = en < bestE[c9];
                            bestE[c9] = fmin(bestE[c9], en);
                            codeE[c9] = lt ? tl : codeE[c9];
                        }
                        if constexpr (MASK & 2) {
                            bool lt = lat < bestL[c9];
                            bestL[c9] = fmin(bestL[c9], lat);
                            codeL[c9] = lt ? tl : codeL[c9];
                        }
                        if constexpr (MASK & 4) {
                            bool lt = (lat < bestLE_l[c9]) | ((lat == bestLE_l[c9]) & (en < bestLE_e[c9]));
                            bestLE_l[c9] = lt ? lat : bestLE_l[c9];
                            bestLE_e[c9] = lt ? en : bestLE_e[c9];
                            codeLE[c9] = lt ? tl : codeLE[c9];
                        }
                    }
                };
                // ---- C
                combinations(X, 0);
                __builtin_amdgcn_sched_barrier(0);
                wait_lds_and_scalar_loads();
                __builtin_amdgcn_sched_barrier(0);
                // ---- D
                request(X, tl_pair + 2);
                __builtin_amdgcn_sched_barrier(0);
                // ---- E
                combinations(Y, 1);
                __builtin_amdgcn_sched_barrier(0);
                wait_lds_and_scalar_loads();
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        const uint64_t row_base = index_row_base(dfrow);
        if constexpr (LAZY) {
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                const double *best = o == 0 ? bestE : (o == 1 ? bestL : bestP);
                double mine_v = best[0];
#pragma unroll
                for (int c9 = 1; c9 < 9; ++c9) mine_v = fmin(mine_v, best[c9]);
                if (!__ballot(mine_v <= run_p[o])) continue;         // the usual case: no lane reaches the running best
                const double wave_v = uniform_f64(wave_min_f64(mine_v));
                // the lowest combination reaching this lane's minimum (lowest index on ties)
                uint32_t cstar = 8;
#pragma unroll
                for (int c9 = 7; c9 >= 0; --c9) cstar = best[c9] == mine_v ? (uint32_t)c9 : cstar;
                // the index row (levels/order/r/combination/f) with the lowest number among those
                // that reach the wave's minimum: its candidates precede every other row's
                const uint32_t my_row = (uint32_t)row_base + 30000u * (cstar % 3) + 90000u * (cstar / 3);
                const uint32_t first_row = __builtin_amdgcn_readfirstlane(
                    wave_min_u32((mine_v == wave_v && mine_v < inf) ? my_row : 0xFFFFFFFFu));
                if (first_row == 0xFFFFFFFFu) continue;              // nothing feasible in this item
                const uint64_t lowest_possible = (uint64_t)t0 + (uint64_t)a.mc.T * first_row;
                if (!(wave_v < run_p[o] || lowest_possible < run_idx[o])) continue;
                // Recover the tiling: the lane that owns first_row lends its selectors, and every
                // lane re-costs one tiling of the chunk for that row and combination, with the very
                // operations of the loop above.
                const unsigned long long owners = __ballot(my_row == first_row && mine_v == wave_v);
                const uint32_t src = (uint32_t)__ffsll((long long)owners) - 1u;
                const uint32_t c_u = __builtin_amdgcn_readlane(cstar, src);
                const uint32_t tl_mine = min(lane, nt - 1);          // lanes beyond the chunk repeat its last tiling
                double w[NSEL];
#pragma unroll
                for (int k = 0; k < NSEL; ++k) w[k] = tab[__builtin_amdgcn_readlane(off[k], src) * LDS_ENT + tl_mine];
                bool ok2 = fmax(w[0] + w[2] + w[1], w[3] + w[2] + w[4]) <= a.mc.cap_words;
                double dram2 = w[5] + w[6] + w[7];
                double e_dram2 = ok2 ? (REGROUP ? a.mc.e_sum : a.mc.e_dram) * dram2 : inf;
                double l_dram2;
                if constexpr (FAST) l_dram2 = dram2 * a.mc.dram_k;
                else l_dram2 = a.mc.dram_bw > 0.0 ? a.mc.c_lat * (((dram2 / a.mc.BH) * a.mc.word) / a.mc.dram_bw) : 0.0;
                l_dram2 = ok2 ? l_dram2 : inf;
                pin(e_dram2);
                pin(l_dram2);
                ConstF64 cl = cs_base + (uint64_t)tl_mine * 2 * NCS;
                double en2;
                if constexpr (REGROUP) {
                    en2 = e_dram2 + cl[c_u];
                } else {
                    double gb2 = dram2 + cl[c_u];
                    en2 = e_dram2 + a.mc.e_gb * gb2;
                    en2 = en2 + cl[18];
                    en2 = en2 + cl[19];
                }
                double lat2 = fmax(l_dram2, cl[9 + c_u]);
                double val2 = o == 0 ? en2 : (o == 1 ? lat2 : en2 * lat2);
                const unsigned long long hits = __ballot(lane >= tl_lo && lane < min(tl_hi, nt) && val2 == wave_v);
                if (!hits) continue;                                 // cannot happen: the loop found it
                const uint64_t idx = (uint64_t)t0 + ((uint32_t)__ffsll((long long)hits) - 1u) +
                                     (uint64_t)a.mc.T * first_row;
                if (wave_v < run_p[o] || idx < run_idx[o]) { run_p[o] = wave_v; run_idx[o] = idx; }
            }
            continue;
        }
        // fold the nine per-combination minima of this lane (ascending combination = ascending
        // index, so a strict < keeps the lowest index), reduce over the wave, keep the wave's best
        Key mine[N_OBJ];
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) { mine[o].p = inf; mine[o].s = 0.0; mine[o].idx = ~0ull; }
#pragma unroll
        for (int c9 = 0; c9 < 9; ++c9) {
            const uint64_t combo_rows = row_base + 30000ull * (c9 % 3) + 90000ull * (c9 / 3);
            if constexpr (MASK & 1) {
                if (bestE[c9] < mine[0].p) {
                    mine[0].p = bestE[c9];
                    mine[0].idx = (uint64_t)(t0 + codeE[c9]) + (uint64_t)a.mc.T * combo_rows;
                }
            }
            if constexpr (MASK & 2) {
                if (bestL[c9] < mine[1].p) {
                    mine[1].p = bestL[c9];
                    mine[1].idx = (uint64_t)(t0 + codeL[c9]) + (uint64_t)a.mc.T * combo_rows;
                }
            }
            if constexpr (MASK & 4) {
                if (bestLE_l[c9] < mine[2].p || (bestLE_l[c9] == mine[2].p && bestLE_e[c9] < mine[2].s)) {
                    mine[2].p = bestLE_l[c9];
                    mine[2].s = bestLE_e[c9];
                    mine[2].idx = (uint64_t)(t0 + codeLE[c9]) + (uint64_t)a.mc.T * combo_rows;
                }
            }
            if constexpr (MASK & 8) {
                if (bestP[c9] < mine[3].p) {
                    mine[3].p = bestP[c9];
                    mine[3].idx = (uint64_t)(t0 + codeP[c9]) + (uint64_t)a.mc.T * combo_rows;
                }
            }
        }
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) {
            if (!((MASK >> o) & 1)) continue;
            // a lane that found nothing feasible must not win a tie between infinities
            if (!(mine[o].p < inf)) { mine[o].s = 0.0; mine[o].idx = ~0ull; }
            Key k = wave_min(mine[o]);
            if (lane == 0 && key_less(k, wave_best[o][wave])) wave_best[o][wave] = k;
        }
    }

    if constexpr (LAZY) {
        if (lane == 0) {
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                wave_best[o][wave].p = run_p[o]; wave_best[o][wave].s = 0.0; wave_best[o][wave].idx = run_idx[o];
            }
        }
    }
    finish_grid<MASK>(a, wave_best, &is_last);
}

// ---------------------------------------------------------------------------
// Exhaustive search over the full row set.
//
// The rows of one (order, r, f) class are the 5^4 buffering levels, and the selectors split: those of
// A and B (buffer, retained, DRAM) depend on (p_A, p_B) only, those of D and E on (p_D, p_E) only,
// those of C on the class (k_build_rows).  So here a lane is a tiling, a wave takes the 125 rows of a
// (class, p_E) task, all selectors are wave-uniform, and a row's three sums are formed from an
// (A, B) part shared by five rows and a (D, E) part held in registers: 3 + 3/5 LDS reads and
// 10 + 3/5 operations per (row, tiling) before the nine combinations, whose per-tiling constants
// are lane registers for the whole task.  All of these sums are exact integers below 2^53 (the
// host refuses a workload where they are not), so their association is free.
//
// A block stages one chunk of TC tilings (stage_tables_direct below) and its waves take neighbouring tasks.
// Persistent blocks, global work counter and grid finish as in k_search; the last chunks are handed
// out in fifths of tasks (one p_D each) to even out the end.  The host sends single-key passes
// here: the 18 per-tiling constants, the (D, E) parts and one key's nine minima fit 128 registers
// (four waves per SIMD), two keys' minima do not.
constexpr int DENSE_THREADS = 512;           // eight waves, two blocks per CU
constexpr int DENSE_BLOCKS_PER_CU = 2;
constexpr int DENSE_WAVES = DENSE_THREADS / 64;

// k_search_dense keeps its table slice as pairs of entries: the direct global-to-LDS load writes one
// contiguous KiB per wave instruction (lane l's 16 bytes at base + 16 l), i.e. the 64 tilings of two
// entries; 16 bytes of padding per pair spread the pairs over the banks for the reads that go across
// entries.  Entry e of tiling t: tab[dense_at(e) + t].
constexpr int DENSE_PAIRS = (NENT + 1) / 2;
constexpr int DENSE_PAIR_F64 = 2 * TC + 2;
__device__ __forceinline__ uint32_t dense_at(uint32_t e) { return e * (DENSE_PAIR_F64 / 2) - (e & 1u); }

// The chunk's 64 tilings of every entry, straight from the global table into LDS: no registers, no
// LDS write instructions, all of a wave's loads in flight at once.  Columns beyond the last tiling exist
// in the global table (it is padded to whole chunks and repeats its last tiling there); so does the
// entry after the last one of an odd count.
template <int WAVES>
__device__ __forceinline__ void stage_tables_direct(const SearchArgs &a, double *tab, uint32_t t0, uint32_t wave, uint32_t lane)
{
    static_assert(NENT + 1 <= NENT_ALL, "the pair of the last entry reads one entry beyond it");
    for (uint32_t pair = wave; pair < (uint32_t)DENSE_PAIRS; pair += WAVES) {
        const uint32_t e = 2 * pair + (lane >> 5);
        const double *src = a.btab + (uint64_t)e * a.mc.tpad + t0 + 2 * (lane & 31);
        __builtin_amdgcn_global_load_lds(src, tab + pair * DENSE_PAIR_F64, 16, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0);               // the loads count as vector memory operations: all of them have landed
}

template <int MASK, bool FAST, bool LIMIT = false, bool REGROUP = false, bool LATCAP = false>
__global__ __launch_bounds__(DENSE_THREADS, 4) void k_search_dense(SearchArgs a)
{
    static_assert(!LATCAP || (MASK == 1 && !LIMIT), "the latency cap goes with the energy key alone");
    __shared__ double tab[DENSE_PAIRS * DENSE_PAIR_F64];
    __shared__ Key wave_best[N_OBJ][DENSE_WAVES];
    __shared__ uint32_t is_last;
    __shared__ uint32_t s_item;
    // Scalar keys: the lowest value any wave of this block has recorded (bit pattern; the keys are
    // non-negative, so the patterns order like the values), refreshed once per item from the launch-wide
    // one.  A wave whose values all lie strictly above it cannot hold the optimum and recovers no position.
    __shared__ unsigned long long hint_bits[N_OBJ];

    constexpr bool LAZY = !(MASK & 4);             // the energy bound of LIMIT masks values, which the lazy argmin handles too
    const double inf = pos_inf();
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (lane < N_OBJ) { wave_best[lane][wave].p = inf; wave_best[lane][wave].s = 0.0; wave_best[lane][wave].idx = ~0ull; }
    if (threadIdx.x < N_OBJ) hint_bits[threadIdx.x] = INF_BITS;
    unsigned long long hint_seen[N_OBJ];          // thread 0: the launch-wide values as last read
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) hint_seen[o] = INF_BITS;
    double run_p[N_OBJ];
    uint64_t run_idx[N_OBJ];
#pragma unroll
    for (int o = 0; o < N_OBJ; ++o) { run_p[o] = inf; run_idx[o] = ~0ull; }
    // encoded rows through the constant address space: wave-uniform row numbers, scalar loads
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    struct EncTable {
        ConstPtr<u32x4> p;
        __device__ __forceinline__ uint4 operator[](uint32_t row) const
        {
            const u32x4 v = p[row];
            return make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    const EncTable enc = {(ConstPtr<u32x4>)a.enc};
    ConstPtr<uint32_t> cls_list = as_constant(a.cls);
    // LATCAP: the second pass of the (latency, energy) key over the full row set.  The first pass found
    // the lowest latency; a candidate's latency max(l_dram, constant) stays within it exactly when both
    // parts do, so the cap masks rows and combinations separately and the pass costs what an
    // energy-only pass costs.
    const double lat_cap = LATCAP ? uniform_f64(a.lat_cap->p) : inf;

    uint32_t upcoming = blockIdx.x;
    while (true) {
        if (threadIdx.x == 0) {
            s_item = upcoming;
            if constexpr (LAZY) {
                // exchange with the launch-wide values read during the previous item: take what is lower there,
                // hand over what is lower here (no reply awaited)
                if (a.hints) {
#pragma unroll
                    for (int o = 0; o < N_OBJ; ++o) {
                        if (!((MASK >> o) & 1)) continue;
                        const unsigned long long here = hint_bits[o];
                        if (hint_seen[o] < here) atomicMin(&hint_bits[o], hint_seen[o]);
                        else if (here < hint_seen[o])
                            (void)__hip_atomic_fetch_min(a.hints + o, here, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
        __syncthreads();                          // also: the previous item's LDS readers are done
        const uint32_t item = s_item;
        if (item >= a.n_items) break;
        if (threadIdx.x == 0) {
            upcoming = gridDim.x + __hip_atomic_fetch_add(a.work_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if constexpr (LAZY) {
                if (a.hints) {
#pragma unroll
                    for (int o = 0; o < N_OBJ; ++o)
                        if ((MASK >> o) & 1) hint_seen[o] = __hip_atomic_load(a.hints + o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        const bool fine = item >= a.n_coarse_items;
        uint32_t chunk, group;
        if (!fine) { chunk = item / a.d_gc; group = item % a.d_gc; }
        else { const uint32_t j = item - a.n_coarse_items; chunk = a.d_ncc + j / a.d_gf; group = j % a.d_gf; }
        const uint32_t t0 = chunk * TC;
        const uint32_t nt = min((uint32_t)TC, a.mc.T - t0);
        stage_tables_direct<DENSE_WAVES>(a, tab, t0, wave, lane);
        __syncthreads();

        const uint32_t per_class = fine ? 25u : 5u;
        const uint32_t task = group * DENSE_WAVES + wave;
        if (task >= a.n_cls * per_class) continue;            // no barrier below: safe to leave early
        const uint32_t cls = cls_list[task / per_class], part = task % per_class;
        const uint32_t rank = cls % 24, g = cls / 24, r = g & 1;
        const uint32_t pE = fine ? part / 5 : part, pd0 = fine ? part % 5 : 0u, npd = fine ? 1u : 5u;
        const uint32_t row0 = 625u * rank + ROWS_PER_GROUP * g;         // (p_A, p_B, p_D, p_E) = 0
        const uint32_t row_de0 = row0 + 25u * (pd0 + 5u * pE);          // first row of the task

        // this lane's tiling: beyond the chunk, its last tiling once more, masked out by the capacity
        const uint32_t tl = min(lane, nt - 1);
        const double cap = lane < nt ? a.mc.cap_words : -1.0;
        const double *cs = a.ctab_s + ((uint64_t)(t0 + tl) * 2 + r) * NCS;
        double gb[9], latc[9];
#pragma unroll
        for (int c = 0; c < 9; ++c) { gb[c] = cs[c]; latc[c] = cs[9 + c]; }
        const double e_rf_part = REGROUP ? 0.0 : cs[18], e_mac_part = REGROUP ? 0.0 : cs[19];
        double too_slow[9];                                   // 0, or +inf for a combination beyond the cap
#pragma unroll
        for (int c = 0; c < 9; ++c) {
            too_slow[c] = LATCAP && !(latc[c] <= lat_cap && lat_cap < inf) ? inf : 0.0;   // no cap found: nothing qualifies
            if constexpr (LATCAP && REGROUP) gb[c] = fmax(gb[c], too_slow[c]);
        }
        const double *col = tab + tl;                         // entry e of this tiling: col[dense_at(e)]

        // the class row and the task's (D, E) rows: all requested before the first is used
        const uint4 e_c = enc[row0];
        uint4 e_de5[5];
#pragma unroll
        for (int q = 0; q < 5; ++q) e_de5[q] = enc[row_de0 + 25u * min((uint32_t)q, npd - 1)];
        const double c_bs = col[dense_at(sel_of(e_c, 2))], c_da = col[dense_at(sel_of(e_c, 7))];

        double bestE[9], bestL[9], bestLE_l[9], bestLE_e[9], bestP[9];
        uint32_t codeE[9], codeL[9], codeLE[9], codeP[9];
#pragma unroll
        for (int c9 = 0; c9 < 9; ++c9) {
            bestE[c9] = bestL[c9] = bestLE_l[c9] = bestLE_e[c9] = bestP[c9] = inf;
            codeE[c9] = codeL[c9] = codeLE[c9] = codeP[c9] = 0;
        }

        // one row of this lane's tiling: Eq. (1), (2), (4), the capacity mask, B*H * Eq. (7), then
        // the nine combinations.  code = the row's place in the task, in index order.
        auto cost_row = [&](double bs1, double bs2, double dram_words, uint32_t code) {
            bool ok = fmax(bs1, bs2) <= cap;
            double e_part = (REGROUP ? a.mc.e_sum : a.mc.e_dram) * dram_words;
            double l_dram;
            if constexpr (FAST) l_dram = dram_words * a.mc.dram_k;
            else l_dram = a.mc.dram_bw > 0.0 ? a.mc.c_lat * (((dram_words / a.mc.BH) * a.mc.word) / a.mc.dram_bw) : 0.0;
            if constexpr (LATCAP) ok = ok & (l_dram <= lat_cap);
            if constexpr (MASK == 1) {
                e_part = ok ? e_part : inf;             // the energy alone: one select, the DRAM time is not needed
            } else {
                const double over = __hiloint2double(ok ? 0 : 0x7ff00000, 0);
                e_part = fmax(e_part, over);
                l_dram = fmax(l_dram, over);
                pin(l_dram);
            }
            pin(e_part);
#pragma unroll
            for (int c9 = 0; c9 < 9; ++c9) {
                double en;
                if constexpr (REGROUP) {
                    en = e_part + gb[c9];
                } else {
                    double gb_words = dram_words + gb[c9];
                    en = e_part + a.mc.e_gb * gb_words;
                    en = en + e_rf_part;
                    en = en + e_mac_part;
                    if constexpr (LATCAP) en = fmax(en, too_slow[c9]);
                }
                double lat = fmax(l_dram, latc[c9]);
                if constexpr (LIMIT) {
                    bool out_of_range = !(en < a.e_limit);
                    en = out_of_range ? inf : en;
                    lat = out_of_range ? inf : lat;
                }
                if constexpr (LAZY) {
                    if constexpr (MASK & 8) bestP[c9] = fmin(bestP[c9], en * lat);
                    if constexpr (MASK & 1) bestE[c9] = fmin(bestE[c9], en);
                    if constexpr (MASK & 2) bestL[c9] = fmin(bestL[c9], lat);
                } else {
                    if constexpr (MASK & 8) {
                        double edp = en * lat;
                        bool lt = edp < bestP[c9];
                        bestP[c9] = fmin(bestP[c9], edp);
                        codeP[c9] = lt ? code : codeP[c9];
                    }
                    if constexpr (MASK & 1) {
                        bool lt = en < bestE[c9];
                        bestE[c9] = fmin(bestE[c9], en);
                        codeE[c9] = lt ? code : codeE[c9];
                    }
                    if constexpr (MASK & 2) {
                        bool lt = lat < bestL[c9];
                        bestL[c9] = fmin(bestL[c9], lat);
                        codeL[c9] = lt ? code : codeL[c9];
                    }
                    if constexpr (MASK & 4) {
                        bool lt = (lat < bestLE_l[c9]) | ((lat == bestLE_l[c9]) & (en < bestLE_e[c9]));
                        bestLE_l[c9] = lt ? lat : bestLE_l[c9];
                        bestLE_e[c9] = lt ? en : bestLE_e[c9];
                        codeLE[c9] = lt ? code : codeLE[c9];
                    }
                }
            }
        };

        if constexpr (LAZY) {
            // (D, E) parts of the task's p_D values in registers; the (A, B) parts are read one step
            // ahead of their use and their selectors one step ahead of that
            double y_ret[5], y_bs[5], y_da[5];
#pragma unroll
            for (int q = 0; q < 5; ++q) {
                // the class's C terms ride on the (D, E) parts
                y_ret[q] = c_bs + col[dense_at(sel_of(e_de5[q], 1))];
                y_bs[q] = col[dense_at(sel_of(e_de5[q], 3))] + c_bs;
                y_da[q] = c_da + col[dense_at(sel_of(e_de5[q], 6))];
            }
            double x_bs = col[dense_at(sel_of(e_c, 0))], x_ret = col[dense_at(sel_of(e_c, 4))],
                   x_da = col[dense_at(sel_of(e_c, 5))];                  // row0 is (p_A, p_B) = 0
            uint4 e_ab = enc[row0 + 1];
            // the loop over (p_A, p_B), for a task of five p_D values or of one: no branch between the rows
            auto ab_loop = [&](auto five) {
                constexpr int NPD = decltype(five)::value ? 5 : 1;
#pragma unroll 5
                for (uint32_t ab = 0; ab < 25; ++ab) {
                    const double now_bs = x_bs, now_ret = x_ret, now_da = x_da;
                    x_bs = col[dense_at(sel_of(e_ab, 0))];
                    x_ret = col[dense_at(sel_of(e_ab, 4))];
                    x_da = col[dense_at(sel_of(e_ab, 5))];
                    e_ab = enc[row0 + min(ab + 2, 24u)];
#pragma unroll
                    for (int q = 0; q < NPD; ++q) cost_row(now_bs + y_ret[q], y_bs[q] + now_ret, now_da + y_da[q], 0);
                }
            };
            if (npd == 5) ab_loop(std::true_type{});
            else ab_loop(std::false_type{});
        } else {
            // index order (p_D, then (p_A, p_B)): a strict < then keeps the lowest index on ties
            for (uint32_t q = 0; q < npd; ++q) {
                const uint4 e_de = enc[row_de0 + 25u * q];
                const double y_ret = col[dense_at(sel_of(e_de, 1))], y_bs = col[dense_at(sel_of(e_de, 3))],
                             y_da = col[dense_at(sel_of(e_de, 6))];
                for (uint32_t ab = 0; ab < 25; ++ab) {
                    const uint4 e_ab = enc[row0 + ab];
                    const double x_bs = col[dense_at(sel_of(e_ab, 0))], x_ret = col[dense_at(sel_of(e_ab, 4))],
                                 x_da = col[dense_at(sel_of(e_ab, 5))];
                    cost_row((x_bs + c_bs) + y_ret, (y_bs + c_bs) + x_ret, (x_da + y_da) + c_da, q * 25u + ab);
                }
            }
        }

        // index row (Sec. VI-A numbering) of the task's row number `code`, combination 0
        auto index_row_of = [&](uint32_t code) { return index_row_base(row_de0 + 25u * (code / 25u) + code % 25u); };

        if constexpr (LAZY) {
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                const double *best = o == 0 ? bestE : (o == 1 ? bestL : bestP);
                double mine_v = best[0];
#pragma unroll
                for (int c9 = 1; c9 < 9; ++c9) mine_v = fmin(mine_v, best[c9]);
                const double hint = __longlong_as_double((long long)hint_bits[o]);
                if (!__ballot(mine_v <= run_p[o] && mine_v < inf && mine_v <= hint)) continue;   // the usual case: nothing new here
                const double wave_v = uniform_f64(wave_min_f64(mine_v));
                // the lowest combination in which some tiling reaches the minimum: its candidates
                // precede those of every higher combination
                uint32_t cstar = 9;
#pragma unroll
                for (int c9 = 8; c9 >= 0; --c9) cstar = best[c9] == wave_v ? (uint32_t)c9 : cstar;
                const uint32_t c_u = __builtin_amdgcn_readfirstlane(wave_min_u32(cstar));
                const uint32_t combo_rows = 30000u * (c_u % 3) + 90000u * (c_u / 3);
                const uint64_t lowest_possible = (uint64_t)t0 + (uint64_t)a.mc.T * (index_row_of(0) + combo_rows);
                if (!(wave_v < run_p[o] || lowest_possible < run_idx[o])) continue;
                // Make the value known before its position is: of the waves of a block that reach this point
                // together, only those holding the lowest value go on (the holder of the lowest value always
                // passes its own mark, so what the others leave out is recorded by it).
                if (lane == 0) atomicMin(&hint_bits[o], (unsigned long long)__double_as_longlong(wave_v));
                if (wave_v > __longlong_as_double((long long)hint_bits[o])) continue;
                // Recover the row: the first row of the task (index order) in which a tiling reaches the
                // minimum under combination c_u holds the lowest index, at its lowest such tiling.  Rows are
                // costed again with the very operations of the loop above.
                double gb_u = gb[0], latc_u = latc[0], slow_u = too_slow[0], best_u = best[0];
#pragma unroll
                for (int c9 = 1; c9 < 9; ++c9) {
                    gb_u = c_u == (uint32_t)c9 ? gb[c9] : gb_u;
                    latc_u = c_u == (uint32_t)c9 ? latc[c9] : latc_u;
                    slow_u = c_u == (uint32_t)c9 ? too_slow[c9] : slow_u;
                    best_u = c_u == (uint32_t)c9 ? best[c9] : best_u;
                }
                // one row of one tiling: table values x (A, B), y (D, E), the class's C terms, the tiling's constants
                auto recost = [&](double x_bs, double x_ret, double x_da, double y_ret, double y_bs, double y_da, double cbs,
                                  double cda, double cap_t, double gb_t, double latc_t, double slow_t, double rf_t, double mac_t) {
                    const double bs1 = (x_bs + cbs) + y_ret;
                    const double bs2 = y_bs + (cbs + x_ret);
                    const double dram2 = (x_da + cda) + y_da;
                    bool ok2 = fmax(bs1, bs2) <= cap_t;
                    double e2 = (REGROUP ? a.mc.e_sum : a.mc.e_dram) * dram2;
                    double l2;
                    if constexpr (FAST) l2 = dram2 * a.mc.dram_k;
                    else l2 = a.mc.dram_bw > 0.0 ? a.mc.c_lat * (((dram2 / a.mc.BH) * a.mc.word) / a.mc.dram_bw) : 0.0;
                    if constexpr (LATCAP) ok2 = ok2 & (l2 <= lat_cap);
                    const double over2 = __hiloint2double(ok2 ? 0 : 0x7ff00000, 0);
                    e2 = fmax(e2, over2);
                    l2 = fmax(l2, over2);
                    pin(e2);
                    pin(l2);
                    double en2;
                    if constexpr (REGROUP) {
                        en2 = e2 + gb_t;
                    } else {
                        double gb2 = dram2 + gb_t;
                        en2 = e2 + a.mc.e_gb * gb2;
                        en2 = en2 + rf_t;
                        en2 = en2 + mac_t;
                        if constexpr (LATCAP) en2 = fmax(en2, slow_t);
                    }
                    double lat2 = fmax(l2, latc_t);
                    if constexpr (LIMIT) {
                        const bool out_of_range = !(en2 < a.e_limit);
                        en2 = out_of_range ? inf : en2;
                        lat2 = out_of_range ? inf : lat2;
                    }
                    return o == 0 ? en2 : (o == 1 ? lat2 : en2 * lat2);
                };
                const uint32_t n_codes = npd * 25u;
                uint32_t found_code = 0xFFFFFFFFu, found_lane = 0;
                // only a tiling whose own minimum under c_u is the wave's can hold it
                unsigned long long cands = __ballot(best_u == wave_v);
                if (__popcll(cands) <= 4) {
                    // few such tilings: one at a time with lane = row (64 rows of the task per step)
                    while (cands) {
                        const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)__ffsll((long long)cands) - 1u);
                        cands &= cands - 1;
                        const double *col_l = tab + l;                  // l < nt: a lane beyond the chunk holds +inf
                        const double cbs_l = lane_value_f64(c_bs, l), cda_l = lane_value_f64(c_da, l);
                        const double gb_l = lane_value_f64(gb_u, l), latc_l = lane_value_f64(latc_u, l), slow_l = lane_value_f64(slow_u, l);
                        const double rf_l = lane_value_f64(e_rf_part, l), mac_l = lane_value_f64(e_mac_part, l);
                        for (uint32_t code0 = 0; code0 < n_codes && code0 < found_code; code0 += 64) {
                            const uint32_t code = min(code0 + lane, n_codes - 1);
                            const uint4 e_de = a.enc[row_de0 + 25u * (code / 25u)];
                            const uint4 e_ab = a.enc[row0 + code % 25u];
                            const double val2 = recost(col_l[dense_at(sel_of(e_ab, 0))], col_l[dense_at(sel_of(e_ab, 4))],
                                                       col_l[dense_at(sel_of(e_ab, 5))], col_l[dense_at(sel_of(e_de, 1))],
                                                       col_l[dense_at(sel_of(e_de, 3))], col_l[dense_at(sel_of(e_de, 6))], cbs_l, cda_l,
                                                       a.mc.cap_words, gb_l, latc_l, slow_l, rf_l, mac_l);
                            const unsigned long long hits = __ballot(code0 + lane < n_codes && val2 == wave_v);
                            if (!hits) continue;
                            const uint32_t c_hit = code0 + (uint32_t)__ffsll((long long)hits) - 1u;
                            if (c_hit < found_code) { found_code = c_hit; found_lane = l; }   // ascending tilings: the lower one stays
                            break;
                        }
                        if (found_code == 0) break;
                    }
                } else {
                    for (uint32_t code = 0; code < n_codes; ++code) {
                        const uint4 e_de = enc[row_de0 + 25u * (code / 25u)];
                        const uint4 e_ab = enc[row0 + code % 25u];
                        const double val2 = recost(col[dense_at(sel_of(e_ab, 0))], col[dense_at(sel_of(e_ab, 4))],
                                                   col[dense_at(sel_of(e_ab, 5))], col[dense_at(sel_of(e_de, 1))],
                                                   col[dense_at(sel_of(e_de, 3))], col[dense_at(sel_of(e_de, 6))], c_bs, c_da, cap,
                                                   gb_u, latc_u, slow_u, e_rf_part, e_mac_part);
                        const unsigned long long hits = __ballot(val2 == wave_v);
                        if (!hits) continue;
                        found_code = code;
                        found_lane = (uint32_t)__ffsll((long long)hits) - 1u;
                        break;
                    }
                }
                if (found_code != 0xFFFFFFFFu) {
                    const uint64_t idx = (uint64_t)t0 + found_lane + (uint64_t)a.mc.T * (index_row_of(found_code) + combo_rows);
                    if (wave_v < run_p[o] || idx < run_idx[o]) { run_p[o] = wave_v; run_idx[o] = idx; }
                }
            }
            continue;
        }
        // eager keys: fold the nine per-combination minima of this lane (ascending combination =
        // ascending index), reduce over the wave, keep the wave's best
        Key mine[N_OBJ];
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) { mine[o].p = inf; mine[o].s = 0.0; mine[o].idx = ~0ull; }
#pragma unroll
        for (int c9 = 0; c9 < 9; ++c9) {
            const uint32_t combo_rows = 30000u * (c9 % 3) + 90000u * (c9 / 3);
            auto idx_of = [&](uint32_t code) { return (uint64_t)(t0 + tl) + (uint64_t)a.mc.T * (index_row_of(code) + combo_rows); };
            if constexpr (MASK & 1) {
                if (bestE[c9] < mine[0].p) { mine[0].p = bestE[c9]; mine[0].idx = idx_of(codeE[c9]); }
            }
            if constexpr (MASK & 2) {
                if (bestL[c9] < mine[1].p) { mine[1].p = bestL[c9]; mine[1].idx = idx_of(codeL[c9]); }
            }
            if constexpr (MASK & 4) {
                if (bestLE_l[c9] < mine[2].p || (bestLE_l[c9] == mine[2].p && bestLE_e[c9] < mine[2].s)) {
                    mine[2].p = bestLE_l[c9];
                    mine[2].s = bestLE_e[c9];
                    mine[2].idx = idx_of(codeLE[c9]);
                }
            }
            if constexpr (MASK & 8) {
                if (bestP[c9] < mine[3].p) { mine[3].p = bestP[c9]; mine[3].idx = idx_of(codeP[c9]); }
            }
        }
#pragma unroll
        for (int o = 0; o < N_OBJ; ++o) {
            if (!((MASK >> o) & 1)) continue;
            if (!(mine[o].p < inf)) { mine[o].s = 0.0; mine[o].idx = ~0ull; }
            Key k = wave_min(mine[o]);
            if (lane == 0 && key_less(k, wave_best[o][wave])) wave_best[o][wave] = k;
        }
    }

    if constexpr (LAZY) {
        if (lane == 0) {
#pragma unroll
            for (int o = 0; o < N_OBJ; ++o) {
                if (!((MASK >> o) & 1)) continue;
                wave_best[o][wave].p = run_p[o]; wave_best[o][wave].s = 0.0; wave_best[o][wave].idx = run_idx[o];
            }
        }
    }
    finish_grid<MASK, DENSE_THREADS>(a, wave_best, &is_last);
}

// One step of the buffer-size / DRAM-access front (Sec. VII-C): the (buffer size, DRAM access,
// index)-smallest dataflow among those whose DRAM access is below a bound.  Neither metric depends
// on the stationary modes, so a (row, tiling) pair stands for its nine combinations through the
// lowest-index one, and the buffer capacity plays no part.  a.e_limit carries the bound in the
// tables' unit, B*H words.  Same items, staging and finish as k_search; result in slot 0.
__global__ __launch_bounds__(SEARCH_THREADS, 4) void k_front_step(SearchArgs a)
{
    __shared__ double tab[NENT * LDS_ENT];
    __shared__ Key wave_best[N_OBJ][SEARCH_THREADS / 64];
    __shared__ uint32_t is_last;
    __shared__ uint32_t s_item;

    const double inf = pos_inf();
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane < N_OBJ) { wave_best[lane][wave].p = inf; wave_best[lane][wave].s = 0.0; wave_best[lane][wave].idx = ~0ull; }

    uint32_t upcoming = blockIdx.x;
    while (true) {
        if (threadIdx.x == 0) s_item = upcoming;
        __syncthreads();
        const uint32_t item = s_item;
        if (item >= a.n_items) break;
        if (threadIdx.x == 0)
            upcoming = gridDim.x + __hip_atomic_fetch_add(a.work_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const ItemView it = locate_item(a, item);
        const bool live = it.live;
        const uint32_t dfrow = it.dfrow;
        const uint4 e = it.e;
        const uint32_t t0 = it.t0, nt = it.nt;
        if (it.fine) stage_tables<TC_FINE / 2>(a, tab, t0, nt);
        else stage_tables<TC / 2>(a, tab, t0, nt);
        __syncthreads();
        if (!__ballot(live)) continue;                       // a wave without a single row
        uint32_t off[NSEL];
#pragma unroll
        for (int k = 0; k < NSEL; ++k) off[k] = sel_of(e, k);
        const double bound = live ? a.e_limit : -1.0;        // a lane without a row takes no part
        double best_bs = inf, best_da = inf;
        uint32_t code = 0;
        for (uint32_t tl = 0; tl < nt; ++tl) {
            double v[NSEL];
#pragma unroll
            for (int k = 0; k < NSEL; ++k) v[k] = tab[off[k] * LDS_ENT + tl];
            double bs = fmax(v[0] + v[2] + v[1], v[3] + v[2] + v[4]);   // Eq. (1), (2), (4)
            double da = v[5] + v[6] + v[7];                             // B*H * Eq. (7)
            bool lt = da < bound && (bs < best_bs || (bs == best_bs && da < best_da));
            best_bs = lt ? bs : best_bs;
            best_da = lt ? da : best_da;
            code = lt ? tl : code;
        }
        Key mine;
        mine.p = best_bs; mine.s = best_da;
        const uint64_t row_base = index_row_base(dfrow);
        mine.idx = (uint64_t)(t0 + code) + (uint64_t)a.mc.T * row_base;
        if (!(mine.p < inf)) { mine.s = 0.0; mine.idx = ~0ull; }
        Key k = wave_min(mine);
        if (lane == 0 && key_less(k, wave_best[0][wave])) wave_best[0][wave] = k;
    }
    finish_grid<1>(a, wave_best, &is_last);
}

// ---------------------------------------------------------------------------
// helpers of the entry point that allocates nothing

// words[0 .. n) = 0 (a fill kernel rather than a memset node, so that a caller may capture the launch)
__global__ void k_clear_words(uint32_t *words, uint32_t n)
{
    const uint32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a < n) words[a] = 0;
}

// the search's final record -> an mmee_result in the caller's device buffer
__global__ void k_pack_result(const FinalRecord *fr, uint64_t space, uint64_t evaluated, mmee_result *out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    mmee_result r;
    __builtin_memset(&r, 0, sizeof(r));
    __builtin_memcpy(&r.cost, fr->cost, sizeof(mmee_cost));
    __builtin_memcpy(&r.best, fr->map, sizeof(mmee_mapping));
    r.space = space;
    r.evaluated = evaluated;
    r.seconds = 0.0;
    r.kernel_seconds = 0.0;
    if (!(fr->key.p < pos_inf())) r.cost.valid = 0;
    *out = r;
}

}  // namespace mmee
