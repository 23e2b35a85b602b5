/*
 * mmee.h -- C ABI of the MI355X (gfx950) implementation of the hot path of MMEE,
 * "Matrix Multiplication Encoded Enumeration" (Fast Cross-Operator Optimization
 * of Attention Dataflow): exhaustive, pruned evaluation of the paper's analytical
 * buffer/DRAM/energy/latency model (Sec. V) over every fused-attention dataflow
 * (Sec. III-IV: tiling, loop order, buffering levels, recomputation, stationary
 * modes, fused or unfused softmax) and reduction to the optimum (Sec. VI).
 *
 * Conventions
 *  - Two chained matmuls per head (Sec. III-A):  C[i,l] = sum_k A[i,k] B[k,l],
 *    E[i,j] = sum_l C[i,l] D[l,j];  for attention A=Q, B=K^T, D=V, E=O, so the
 *    loop extents are I = L = N and K = J = d.  Dimensions are indexed
 *    i=0, k=1, l=2, j=3 everywhere.  Each extent is split in two levels,
 *    X = x_D * x_G: inter-tile count times intra-tile size (Sec. IV-A).
 *  - A candidate is one index in [0, space).  Mixed-radix digits, least
 *    significant first:
 *        t_i, t_k, t_l, t_j   position of x_G in the ascending divisor list of I,K,L,J
 *        p_A, p_B, p_D, p_E   buffering level 0..4 = number of innermost inter-tile
 *                             loops the operand's buffer spans (0 = one tile; the
 *                             paper's layers L3..L7, Sec. IV-B)
 *        order  0..23         lexicographic rank of the inter-tile loop sequence,
 *                             written outer -> inner over the symbols i<k<l<j
 *        r      0..1          recomputation of C tiles (Sec. III-C)
 *        s1,s2  0..2          stationary mode of Op1 / Op2: 0 weight, 1 input, 2 output (Sec. V-D)
 *        f      0..1          1 = softmax fused (C stays on chip), 0 = C staged through DRAM
 *    so space = (#tilings) * 540000.
 *  - All pointers are HOST pointers unless stated otherwise.  The library keeps
 *    none of them after a call returns.  Device scratch is cached inside the
 *    library and released by mmee_shutdown().
 *  - Every function returns 0 on success or a negative MMEE_E* code; nothing is
 *    thrown across this boundary.  Calls are serialised by an internal lock.
 *  - All the arithmetic runs in HIP kernels on the current HIP device; there is
 *    no CPU fallback: without a usable GPU the calls return MMEE_EDEVICE.
 */
#ifndef MMEE_H
#define MMEE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Attention workload (Sec. II-A): B batches of H heads, sequence length N, head dim d. */
typedef struct mmee_workload {
    uint32_t B, H, N, d;
    uint32_t word_bytes;    /* bytes per element, 2 for fp16                              */
    uint32_t tiling_mode;   /* 0: x_G ranges over power-of-two divisors, 1: all divisors   */
    uint32_t c_softmax;     /* softmax cost per element of C in MAC-energy units (Sec. V-D; the paper uses 10) */
    uint32_t reserved;      /* must be 0                                                   */
} mmee_workload;

/* Two chained matrix multiplications of free shape (Sec. VII-J, Table V: two GEMMs, or a
 * convolution chain turned into GEMMs by im2col): Op1 is I x K x L, Op2 is I x L x J, `batch`
 * independent instances.  An attention workload is the chain I = L = N, K = J = d, batch = B*H;
 * every mmee_* call on a workload is the mmee_chain_* call on that chain. */
typedef struct mmee_chain {
    uint32_t batch;
    uint32_t I, K, L, J;
    uint32_t word_bytes;
    uint32_t tiling_mode;   /* as in mmee_workload                                         */
    uint32_t c_softmax;     /* 0 when nothing sits between the two operators               */
} mmee_chain;

/* Spatial accelerator (Sec. II-B): PE arrays with register files, one global buffer, DRAM. */
typedef struct mmee_hw {
    uint32_t pe_rows, pe_cols;  /* one PE array                                            */
    uint32_t n_arrays;          /* heads are spread over the arrays (Sec. V)               */
    uint32_t rf_bytes;          /* register file per PE; half of it holds stationary data  */
    uint64_t gb_bytes;          /* global buffer capacity: BS * word_bytes <= gb_bytes     */
    double e_dram, e_gb, e_rf, e_mac;   /* pJ per word access at each level, pJ per MAC     */
    double dram_bw, gb_bw;      /* bytes per cycle; 0 drops that stream from the latency   */
} mmee_hw;

/* One decoded candidate (Sec. IV-A: loop boundaries, loop order, buffering levels). */
typedef struct mmee_mapping {
    uint64_t idx;
    uint32_t xG[4], xD[4];      /* i,k,l,j                                                 */
    uint8_t order[4];           /* inter-tile loops, outer -> inner, values 0..3 = i,k,l,j */
    uint8_t level[4];           /* p_A, p_B, p_D, p_E                                      */
    uint8_t recompute, stat1, stat2, fused;
} mmee_mapping;

/* Cost of one candidate.  The integer fields are per head (the model omits the head
 * dimension, Sec. V); energy and latency cover all B*H heads.  64 bytes. */
typedef struct mmee_cost {
    uint64_t bs_words;          /* buffer size requirement, Eq. (4)                        */
    uint64_t da_words;          /* DRAM access, Eq. (7) (+ DA_C when f = 0)                */
    uint64_t br_words;          /* buffer <-> register-file traffic                        */
    uint64_t mac_total;         /* N_op1 + N_op2, or j_D*N_op1 + N_op2 with recomputation  */
    uint64_t comp_cycles;       /* compute cycles on one array                             */
    double energy_pj;           /* +inf when valid == 0                                    */
    double latency_cycles;      /* +inf when valid == 0                                    */
    uint32_t valid;             /* 1 = feasible dataflow                                   */
    uint32_t reason;            /* 0 ok; 1 not a dataflow (r=1 with k outside j, or r=1 with f=0):
                                   all integer fields are 0; 2 exceeds the buffer capacity */
} mmee_cost;

typedef struct mmee_result {
    mmee_mapping best;
    mmee_cost cost;
    uint64_t space;             /* size of the index space                                 */
    uint64_t evaluated;         /* candidates whose cost the search actually formed        */
    double seconds;             /* host wall time of the call (upload, kernels, readback)  */
    double kernel_seconds;      /* device time of the search kernel alone (HIP events)     */
} mmee_result;

/* Counts of the offline stage (Sec. VI-B): loop-order x buffering-level rows per
 * (recompute, fused) group before and after symbolic pruning.  Group g = r + 2 f. */
typedef struct mmee_row_stats {
    uint32_t rows_total[4];     /* 15000 each                                              */
    uint32_t rows_valid[4];     /* rows that denote a dataflow                             */
    uint32_t rows_kept[4];      /* survivors of the dominance test                         */
} mmee_row_stats;

enum {
    MMEE_OBJ_ENERGY = 0,                /* key (energy, idx)            */
    MMEE_OBJ_LATENCY = 1,               /* key (latency, idx)           */
    MMEE_OBJ_LATENCY_THEN_ENERGY = 2,   /* key (latency, energy, idx)   */
    MMEE_OBJ_EDP = 3                    /* key (energy * latency, idx), the energy-delay product (Sec. VII-K) */
};

enum {
    MMEE_SEARCH_PRUNED = 0,             /* offline symbolic pruning on (the paper's method) */
    MMEE_SEARCH_EXHAUSTIVE = 1,         /* cost every candidate that denotes a dataflow     */
    /* When the four energies per access are whole numbers and the largest possible total stays
     * below 2^53, every term of the energy is an exact integer and the search adds a (row, tiling)
     * part and a (tiling, stationary modes) part per candidate; the result has the same bits as
     * the sum taken term by term in the order of Sec. V-D.  When only the size condition fails,
     * the searches for the energy, the latency and the (latency, energy) key still start that way
     * and keep the outcome if the optimal energy found is below 2^52 pJ: every candidate whose total
     * reaches 2^53 computes to more than that in either order, all others are exact, so the optimum
     * and its ties are those of the term-by-term sum; otherwise the search is repeated term by term.
     * This flag (may be or-ed with the others) keeps the term-by-term order in every case. */
    MMEE_SEARCH_ORDERED_SUM = 2
};

enum {
    MMEE_OK = 0,
    MMEE_EINVAL = -1,       /* null pointer, zero dimension, unsupported size, bad enum       */
    MMEE_ERANGE = -2,       /* index range outside [0, space)                                 */
    MMEE_ENOFEASIBLE = -3,  /* every candidate is masked; out->cost.valid = 0                 */
    MMEE_EDEVICE = -4,      /* HIP error or no device                                         */
    MMEE_EOVERFLOW = -5,    /* mmee_pareto: more front points than `capacity`                 */
    MMEE_ETOOBIG = -6       /* mmee_search_noalloc: the problem exceeds its fixed scratch     */
};

/* Number of candidates of (workload, hw): #tilings (integer factorisations, Sec. VI-A)
 * times 540000.  Pure host arithmetic. */
int mmee_space_size(const mmee_workload *w, const mmee_hw *hw, uint64_t *out);

/* *out = 1 when the regrouped energy sum (see MMEE_SEARCH_ORDERED_SUM) is exact for every candidate
 * of (workload, hw) and these flags allow it: whole-number energies per access, total energy of any
 * candidate (Sec. V-D) below 2^53, and a power-of-two DRAM bandwidth and array count; else 0.  Pure
 * host arithmetic. */
int mmee_energy_regrouped(const mmee_workload *w, const mmee_hw *hw, uint32_t flags, int *out);

/* On-device mixed-radix decode of n candidate indices (host arrays in and out): index -> loop
 * boundaries, loop order, buffering levels and options, the components of a pseudo nested loop
 * (Sec. IV-A).  A helper next to the three calls of the problem statement. */
int mmee_decode(const mmee_workload *w, const mmee_hw *hw, const uint64_t *idx, uint64_t n,
                mmee_mapping *out);

/* Cost of the n consecutive candidates first_idx .. first_idx+n-1 (Sec. V, Eq. (1)-(7),
 * energy and latency of Sec. V-D).  out_costs holds n records and may be host memory or
 * device memory of the current device (detected); device results are not copied back. */
int mmee_eval_batch(const mmee_workload *w, const mmee_hw *hw, uint64_t first_idx, uint64_t n,
                    mmee_cost *out_costs);

/* Optimal mapping under one objective; ties go to the lowest index (Sec. VI).
 * mmee_search uses the pruned row set. */
int mmee_search(const mmee_workload *w, const mmee_hw *hw, int objective, mmee_result *out);
int mmee_search_ex(const mmee_workload *w, const mmee_hw *hw, int objective, uint32_t flags,
                   mmee_result *out);

/* One pass over the space that reduces n_obj (1..4, distinct) objectives at once: all
 * metrics of a candidate are formed once and shared (Sec. VII-D).  out holds n_obj results. */
int mmee_search_multi(const mmee_workload *w, const mmee_hw *hw, const int *objectives,
                      uint32_t n_obj, uint32_t flags, mmee_result *out);

/* A helper for sweeps over hardware designs and sequence lengths (Sec. VII-I, Table IV; Sec. VII-H):
 * count independent searches (arrays of count workloads, hws, objectives, results) enqueued
 * back to back on one stream with a single synchronisation at the end.  Neighbouring entries
 * with identical workload and hw share one pass.  Pruned passes for one key, or for energy and
 * latency together, share kernel launches across problems (one per kind of pass present); the
 * other passes run problem by problem.  mmee_result::kernel_seconds of a pass that shared
 * launches is the device time of all the launches it shared.  Returns the first non-zero
 * per-entry code (per-entry codes are stored in rc[i] when rc is not null). */
int mmee_search_many(const mmee_workload *w, const mmee_hw *hw, const int *objectives,
                     uint32_t count, uint32_t flags, mmee_result *out, int *rc);

/* Energy-latency Pareto front (Sec. VI-A, Sec. VII-E): the feasible candidates that no other
 * candidate beats in both metrics; among candidates with identical (energy, latency) the lowest
 * index stands for all.  out receives at most `capacity` points by ascending latency (descending
 * energy), *n_points their number.  Each point costs one pass over the space.  Returns
 * MMEE_EOVERFLOW (with the first `capacity` points stored) when the front is longer. */
int mmee_pareto(const mmee_workload *w, const mmee_hw *hw, uint32_t flags, mmee_result *out,
                uint32_t capacity, uint32_t *n_points);

/* DRAM access versus buffer size requirement (Sec. VII-C): the dataflows that no other dataflow
 * beats in both Eq. (4) and Eq. (7), whatever the buffer capacity of hw (their cost records carry
 * valid = 0, reason = 2 where they exceed it).  Neither metric depends on the stationary modes;
 * the lowest index stands for equal pairs.  Points come by ascending buffer size (descending
 * DRAM access); conventions as for mmee_pareto.  `evaluated` counts (row, tiling) pairs. */
int mmee_front_bs_da(const mmee_workload *w, const mmee_hw *hw, uint32_t flags, mmee_result *out,
                     uint32_t capacity, uint32_t *n_points);

/* The same calls for a free chain shape (Sec. VII-J).  Semantics, layouts and error codes are
 * those of the workload calls above. */
int mmee_chain_space_size(const mmee_chain *c, const mmee_hw *hw, uint64_t *out);
int mmee_chain_energy_regrouped(const mmee_chain *c, const mmee_hw *hw, uint32_t flags, int *out);
int mmee_chain_decode(const mmee_chain *c, const mmee_hw *hw, const uint64_t *idx, uint64_t n,
                      mmee_mapping *out);
int mmee_chain_eval_batch(const mmee_chain *c, const mmee_hw *hw, uint64_t first_idx, uint64_t n,
                          mmee_cost *out_costs);
int mmee_chain_search_multi(const mmee_chain *c, const mmee_hw *hw, const int *objectives,
                            uint32_t n_obj, uint32_t flags, mmee_result *out);
int mmee_chain_search_many(const mmee_chain *c, const mmee_hw *hw, const int *objectives,
                           uint32_t count, uint32_t flags, mmee_result *out, int *rc);
int mmee_chain_pareto(const mmee_chain *c, const mmee_hw *hw, uint32_t flags, mmee_result *out,
                      uint32_t capacity, uint32_t *n_points);
int mmee_chain_front_bs_da(const mmee_chain *c, const mmee_hw *hw, uint32_t flags, mmee_result *out,
                           uint32_t capacity, uint32_t *n_points);

/* mmee_search_ex for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  This call allocates and frees nothing, on the host
 * side of HIP or on the device, and does not synchronise: it enqueues a handful of kernels on the
 * library's stream (mmee_set_stream) and returns.  All its working memory (row encodings, the
 * per-tiling tables, partial records) is one fixed array of at most 40 MiB that every GPU the
 * library is loaded on holds until the process ends; problems with more than 16384 tilings do not
 * fit and return MMEE_ETOOBIG (mmee_strerror says by how much) with nothing enqueued.
 *   out_dev   DEVICE pointer (current device) to one mmee_result, written by the last kernel;
 *             valid once the stream has been synchronised by the caller.  `seconds` and
 *             `kernel_seconds` are 0.  When no candidate is feasible the call still returns
 *             MMEE_OK and the record carries cost.valid = 0 (nothing is read back to tell).
 *   flags     as for mmee_search_ex; the regrouped energy sum is used only where it is exact
 *             beforehand (mmee_energy_regrouped), never on trust.
 * The first call on a device runs the offline stage into the array and reads eight counters back
 * (one synchronisation, still no allocation): make it outside any capture.  All calls on one GPU
 * share that GPU's array, which keeps the last call's contents; what must start at zero is cleared
 * by a kernel at the start of each call.  Calls that overlap on one GPU (different streams, or
 * the same stream replayed while an earlier launch still runs) race; so does this call against
 * any other search in flight on a different stream. */
int mmee_search_noalloc(const mmee_workload *w, const mmee_hw *hw, int objective, uint32_t flags,
                        mmee_result *out_dev);

/* Runs the offline stage if needed (row encoding + symbolic pruning, once per process) and
 * reports its counts. */
int mmee_offline_stats(mmee_row_stats *out);

/* The offline stage's row lists (Sec. VI-A: listed ahead of time; Sec. VI-B): the rows of group
 * g = r + 2 f that denote a dataflow (which = 0) or that survive the symbolic pruning of Eq. (12)
 * (which = 1), ascending, as row numbers inside the group: p_A + 5 p_B + 25 p_D + 125 p_E +
 * 625 * order.  rows_out (host) receives at most `capacity` numbers, *n_rows the length of the
 * list; MMEE_EOVERFLOW when the list is longer than `capacity`. */
int mmee_offline_rows(uint32_t group, uint32_t which, uint32_t *rows_out, uint32_t capacity, uint32_t *n_rows);

/* Environment: MMEE_RESIDENT_BLOCKS=<even number>, read at the first call, lowers the number of
 * persistent blocks the search kernels are launched with (default: two per compute unit).  It
 * changes how the work is split and in which order partial results meet, never a result. */

/* Use this HIP stream (a hipStream_t passed as void*) for all later launches; NULL = default. */
int mmee_set_stream(void *hip_stream);

/* Free all cached device memory.  The library re-initialises itself on the next call. */
void mmee_shutdown(void);

const char *mmee_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MMEE_H */
