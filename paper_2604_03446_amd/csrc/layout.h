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
// BS_X options: tile_X * {1, d0, d1, d0*d1}, d0/d1 = inter-tile counts of X's two own dims
constexpr int ENT_BS = 0;        // + 4*X + sel, X = A,B,C,D,E
constexpr int ENT_ZERO = 20;     // 0 (operand not retained, or fused C in DRAM terms)
// DA_X options: |X| * {1, n0, n1, n0*n1}, n0/n1 = inter-tile counts of the two dims X does not own
constexpr int ENT_DA = 21;       // + 4*Y + sel, Y = A,B,D,E
// unfused C: |C| * ((k_D or 1) + (j_D or 1) + 2)
constexpr int ENT_DAC = 37;      // + sel
constexpr int NENT = 41;

// ---- one encoded row ("Q side"): 14 selectors + flags, 16 bytes ---------------
// sel[0..4]   BS_A BS_B BS_C BS_D BS_E
// sel[5..8]   tau_X * BS_X for X = A,B,D,E   (ENT_ZERO when the operand is not retained)
// sel[9..12]  DA_A DA_B DA_D DA_E
// sel[13]     DA_C
// sel[14]     flags: bit0 row denotes a dataflow, bit1 r, bit2 f
constexpr int NSEL = 14;
constexpr int ROW_FLAGS = 14;

constexpr uint32_t ROWS_PER_GROUP = 15000;   // 5^4 levels * 24 orders
constexpr uint32_t N_GROUPS = 4;             // g = r + 2 f
constexpr uint32_t N_DFROWS = ROWS_PER_GROUP * N_GROUPS;
constexpr uint64_t ROWS_PER_TILING = 540000; // * 9 stationary combinations

// per (tiling, r) constants read by the search kernel: 9 + 9 + 2 doubles
//   [0..8]  BH * BR(combo)                      combo = s1 + 3 s2
//   [9..17] c_lat * max(comp(combo), BR*w/gb_bw)
//   [18]    e_rf * T_rf      [19] e_mac * T_mac
constexpr int NCS = 20;
// per (r, field, tiling) raw integers read by the eval kernel: br[9], comp[9], mac, softmax elems
constexpr int NCE = 20;

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
    double dram_bw, gb_bw;
    double dram_k;      // word / dram_bw when that is exact (power-of-two bandwidth), else unused
    uint32_t pe_rows, pe_cols, g_words, c_softmax;
    uint32_t T, tpad;
};

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
