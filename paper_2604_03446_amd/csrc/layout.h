// Data layout shared by the kernels and the host side of libmmee.
//
// The paper evaluates all (loop order, buffering level) x tiling pairs as one
// matrix product R = exp(Q ln B) (Sec. VI-A, Eq. (11)): a row of Q is a 0/1
// exponent vector over the boundary vector b = [i_D k_D l_D j_D i_G k_G l_G j_G]
// (Eq. (9), (10)).  Every monomial of the model has a fixed intra-tile part
// (the operand's tile, or the whole matrix for a DRAM term) times a subset of at
// most two inter-tile boundaries.  Here the contraction is therefore carried out
// exactly, in integers held in fp64 (all < 2^53), as
//     R[row, tiling] = Btab[tiling][ sel[row] ]
// where Btab holds, per tiling, the handful of subset products each monomial can
// take, and a Q row shrinks to one small selector per monomial.
#pragma once
#include <stdint.h>

namespace mmee {

enum { DI = 0, DK = 1, DL = 2, DJ = 3 };          // loop dimensions
enum { OA = 0, OB = 1, OC = 2, OD = 3, OE = 4 };  // operands

// ---- entries of the per-tiling table ("B side") ------------------------------
// An operand's buffer size is tile_X * {1, d0, d1, d0*d1} (d0/d1 = inter-tile counts of its two
// own dims, option index = bit0 | bit1 << 1); its DRAM traffic is B*H*|X| * {1, n0, n1, n0*n1}
// (n0/n1 = inter-tile counts of the two dims it does not own).  Option 4 stands for "absent"
// (operand not retained / fused C).  Terms that are only ever added are stored as pair sums so
// that one lookup serves two operands:
constexpr int ENT_BS_AB = 0;      // BS_A[a] + BS_B[b]              index a + 4 b        (Eq. (1))
constexpr int ENT_BS_DE = 16;     // BS_D[a] + BS_E[b]                                   (Eq. (2))
constexpr int ENT_RET_DE = 32;    // tau_D BS_D[a] + tau_E BS_E[b]  index a + 5 b, a,b in 0..4
constexpr int ENT_RET_AB = 57;    // tau_A BS_A[a] + tau_B BS_B[b]
constexpr int ENT_BS_C = 82;      // BS_C[c]
constexpr int ENT_DA_AB = 86;     // B*H*(DA_A[a] + DA_B[b])        index a + 4 b        (Eq. (7))
constexpr int ENT_DA_DE = 102;    // B*H*(DA_D[a] + DA_E[b])
constexpr int ENT_DA_C = 118;     // B*H*DA_C[c], c in 0..4: |C| * ((k_D or 1) + (j_D or 1) + 2), or 0
constexpr int NENT = 123;          // entries the search kernel stages into LDS
// the same DRAM terms without the B*H factor, read by the per-candidate kernel only
constexpr int ENT_RAW_DA = 37;     // raw entry = scaled entry + 37
constexpr int NENT_ALL = 160;

// ---- one encoded row ("Q side"): 8 selectors + flags in 16 bytes ----------------
// sel[0] BS_AB  sel[1] RET_DE  sel[2] BS_C  sel[3] BS_DE  sel[4] RET_AB
// sel[5] DA_AB  sel[6] DA_DE   sel[7] DA_C  (absolute entry numbers)
// sel[8] flags: bit0 row denotes a dataflow, bit1 r, bit2 f
constexpr int NSEL = 8;
constexpr int ROW_FLAGS = 8;

constexpr uint32_t ROWS_PER_GROUP = 15000;   // 5^4 levels * 24 orders
constexpr uint32_t N_GROUPS = 4;             // g = r + 2 f
constexpr uint32_t N_DFROWS = ROWS_PER_GROUP * N_GROUPS;
constexpr uint64_t ROWS_PER_TILING = 540000; // * 9 stationary combinations

// per (tiling, r) constants read by the search kernel: 9 + 9 + 2 doubles
//   [0..8]  BH * BR(combo)                      combo = s1 + 3 s2
//   [9..17] c_lat * max(comp(combo), BR*w/gb_bw)
//   [18]    e_rf * T_rf      [19] e_mac * T_mac
// When the energy is regrouped (ModelConst::regroup) [0..8] hold the whole part of the energy that
// does not depend on the row instead: e_gb * BH * BR(combo) + e_rf * T_rf + e_mac * T_mac.
constexpr int NCS = 20;
// per (r, field, tiling) values read by the per-candidate kernel, 64 bits each:
//   [0..8] BR (u64)   [9..17] cycles (u64)   [18] MAC (u64)   [19] softmax elements (u64)
//   [20..28] c_lat * max(cycles, BR*w/gb_bw) (fp64)   [29] e_rf * T_rf (fp64)   [30] e_mac * T_mac (fp64)
constexpr int NCE = 31;

constexpr int MAXDIV = 240;      // divisors per dimension (720720 has 240)

struct DivTable {                // passed by value as a kernel argument
    uint32_t X[4];
    uint32_t ndiv[4];
    uint32_t div[4][MAXDIV];
};

struct ModelConst {
    double BH;          // B*H
    double c_lat;       // BH / n_arrays
    double cap_words;   // floor(gb_bytes / word_bytes)
    double word;        // word_bytes
    double e_dram, e_gb, e_rf, e_mac;
    double e_sum;       // e_dram + e_gb, the weight of a DRAM word when the energy is regrouped
    double dram_bw, gb_bw;
    double dram_k;      // word / dram_bw / n_arrays when that is exact (powers of two), else unused
    double eval_k;      // word / dram_bw when the bandwidth is a power of two (or 0), else unused
    double gb_k;        // word / gb_bw when the buffer bandwidth is a power of two, else unused
    // 1 / pe_rows, 1 / pe_cols, 1 / (pe_cols * g_words), rounded once: floor((a - 0.5) * 1/b) + 1 is
    // ceil(a / b) for every 1 <= a < 2^32 (a - 0.5 over b stays 0.5 / b away from whole numbers, the two
    // roundings move it by less than that)
    double rcp_rows, rcp_cols, rcp_cols_g;
    uint32_t bw_pow2;   // the DRAM bandwidth is 0 or a power of two
    uint32_t gb_pow2;   // the buffer bandwidth is a power of two
    // The four energies are whole numbers and the largest total energy stays below 2^53: every
    // product and partial sum of the energy is then an exact integer, the order of the additions
    // cannot change a bit of the result, and the search adds one row part and one tiling part.
    uint32_t regroup;
    uint32_t pe_rows, pe_cols, g_words, c_softmax;
    uint32_t T, tpad;
};

constexpr int N_OBJ = 4;         // energy, latency, latency-then-energy, energy-delay product

struct Key {            // lexicographic objective key, lowest index wins ties
    double p, s;
    uint64_t idx;
};

struct FinalRecord {    // what a search leaves on the device for the host to read
    Key key;
    uint64_t cost[8];   // mmee_cost image
    uint64_t map[7];    // mmee_mapping image
};

}  // namespace mmee
