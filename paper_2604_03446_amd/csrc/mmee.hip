// libmmee: host side of the C ABI declared in include/mmee.h.
// Argument checking, integer factorisation of the loop extents (the online
// tiling enumeration of Sec. VI-A), launch plumbing and result unpacking.
// Every number the calls return is produced by the kernels in kernels.h.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "kernels.h"
#include "batch.h"

// ---- fixed scratch of the entry point that allocates nothing (mmee_search_noalloc) ------------
// One array per GPU, held from the moment the library is loaded until the process ends.  In host
// code the array's name is only a stand-in: its device address comes from hipGetSymbolAddress,
// once per device, and that pointer is what kernels, fills and copies are given.
namespace mmee {
namespace noalloc {
constexpr size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
constexpr uint32_t MAX_TPAD = 16384;        // tilings a problem may have (rounded up to 64)
constexpr uint32_t MAX_BLOCKS = 1024;       // persistent blocks the partial records have room for
constexpr size_t OFF_ENC = 0;
constexpr size_t OFF_SIG = OFF_ENC + up256(sizeof(uint4) * N_DFROWS);
constexpr size_t OFF_FLAGS = OFF_SIG + up256(sizeof(uint32_t) * N_DFROWS);
constexpr size_t OFF_ROWS0 = OFF_FLAGS + up256(N_DFROWS);
constexpr size_t OFF_ROWS1 = OFF_ROWS0 + up256(sizeof(uint32_t) * N_DFROWS);
constexpr size_t OFF_RENC0 = OFF_ROWS1 + up256(sizeof(uint32_t) * N_DFROWS);
constexpr size_t OFF_RENC1 = OFF_RENC0 + up256(sizeof(uint4) * N_DFROWS);
constexpr size_t OFF_COUNTS = OFF_RENC1 + up256(sizeof(uint4) * N_DFROWS);
constexpr size_t OFF_TICKET = OFF_COUNTS + up256(sizeof(uint32_t) * 8);
constexpr size_t OFF_KEYS = OFF_TICKET + up256(sizeof(uint32_t) * 2);
constexpr size_t OFF_PARTIALS = OFF_KEYS + up256(sizeof(Key) * N_OBJ);
constexpr size_t OFF_FINAL = OFF_PARTIALS + up256(sizeof(Key) * N_OBJ * MAX_BLOCKS);
constexpr size_t OFF_DV = OFF_FINAL + up256(sizeof(FinalRecord) * N_OBJ);
constexpr size_t OFF_BTAB = OFF_DV + up256(sizeof(DivTable));
constexpr size_t OFF_CTAB_S = OFF_BTAB + up256(sizeof(double) * NENT_ALL * MAX_TPAD);
constexpr size_t OFF_CTAB_E = OFF_CTAB_S + up256(sizeof(double) * 2 * NCS * MAX_TPAD);
constexpr size_t BYTES = OFF_CTAB_E + up256(sizeof(uint64_t) * 2 * NCE * MAX_TPAD);
static_assert(BYTES <= (40u << 20), "the fixed scratch is documented as at most 40 MiB");
}  // namespace noalloc
}  // namespace mmee

static __device__ __align__(256) unsigned char scratch[mmee::noalloc::BYTES];

namespace mmee {
namespace {

#define HIP_TRY(expr)                                                                        \
    do {                                                                                     \
        hipError_t err_ = (expr);                                                            \
        if (err_ != hipSuccess) {                                                            \
            std::snprintf(g_last_error, sizeof(g_last_error), "%s: %s (%s:%d)", #expr,       \
                          hipGetErrorString(err_), __FILE__, __LINE__);                      \
            return MMEE_EDEVICE;                                                             \
        }                                                                                    \
    } while (0)

char g_last_error[512] = "";
std::mutex g_lock;

struct State {
    bool ready = false;
    hipStream_t stream = nullptr;
    // offline stage
    uint4 *enc = nullptr;
    uint32_t *sig = nullptr;
    uint8_t *flags = nullptr;
    uint32_t *rows[2] = {nullptr, nullptr};     // [0] every row that denotes a dataflow, [1] survivors
    uint4 *row_enc[2] = {nullptr, nullptr};     // the encoded rows in list order
    uint32_t *counts_dev = nullptr;
    uint32_t counts[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    Key *key_dev = nullptr;                     // [N_OBJ] winning keys of a pass, for the pass that follows it
    uint32_t *cls_dev = nullptr;                // (order, r, f) classes whose rows denote dataflows
    uint32_t n_cls = 0;
    // online scratch, grown on demand
    double *btab = nullptr, *ctab_s = nullptr;
    uint64_t *ctab_e = nullptr;
    size_t tiling_cap = 0;
    Key *partials = nullptr;
    size_t partials_cap = 0;
    uint32_t *ticket = nullptr;
    unsigned long long *hints = nullptr;
    // result records: pinned host memory that the search's last block writes directly
    FinalRecord *final_host = nullptr, *final_map = nullptr;     // host address / device address
    DivTable *dv_dev = nullptr;
    size_t slots = 0;
    std::vector<hipEvent_t> events;
    void *eval_dev = nullptr;
    size_t eval_cap = 0;
    uint32_t resident_blocks = 512;
    // batched search over the pruned rows: problem descriptors (pinned staging + device copy), one record
    // per work item and objective; the split of the row lists over the waves of a block
    unsigned char *batch_host = nullptr, *batch_dev = nullptr;
    size_t batch_blob_cap = 0;
    Key *item_keys = nullptr;
    size_t item_cap = 0;
    uint32_t task_lo[BATCH_WAVES] = {}, task_cnt[BATCH_WAVES] = {}, task_g[BATCH_WAVES] = {};
    uint32_t *batch_row_off = nullptr, *batch_row_df = nullptr, *batch_cmap = nullptr;
    uint32_t batch_rows = 0, batch_n_used = 0;
    bool batch_ok = false;      // the surviving rows fit the batched kernel's fixed LDS layout
} S;

// The device buffers one search pass works in.  The allocating entry points fill this from the
// cached State; the entry point that allocates nothing fills it from the static scratch array.
struct Bufs {
    const uint4 *enc = nullptr;
    const uint32_t *rows[2] = {nullptr, nullptr};
    const uint4 *row_enc[2] = {nullptr, nullptr};
    uint32_t counts[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    const uint32_t *cls_dev = nullptr;          // null: no class list, the dense kernel is not used
    uint32_t n_cls = 0;
    double *btab = nullptr, *ctab_s = nullptr;
    uint64_t *ctab_e = nullptr;
    Key *partials = nullptr;
    size_t partials_cap = 0;                    // blocks the partial records have room for
    uint32_t *ticket = nullptr;                 // [0] finish ticket, [1] work counter
    unsigned long long *hints = nullptr;        // [N_OBJ] launch-wide lowest values of the dense kernel; null: not shared
    Key *key_dev = nullptr;
    FinalRecord *final_dev = nullptr;           // device address of this pass's N_OBJ records
    DivTable *dv_dev = nullptr;                 // this pass's copy of the divisor lists
    hipEvent_t ev_begin = nullptr, ev_end = nullptr;   // null: the pass is not timed
    uint32_t resident_blocks = 512;
};

// ---- argument checking and the per-call plan ---------------------------------

struct Plan {
    DivTable dv;
    ModelConst mc;
    uint64_t T;
    uint64_t space;
    bool exact_k;
    bool can_regroup;   // every term of the energy is an exact integer below 2^53
    bool whole_energies; // the four energies per access are whole numbers (their size aside)
};

bool finite_nonneg(double v) { return std::isfinite(v) && v >= 0.0; }

int list_divisors_uncached(uint32_t X, uint32_t mode, uint32_t *out);

// the last few factorisations are kept: a sweep asks for the same extents over and over
int list_divisors(uint32_t X, uint32_t mode, uint32_t *out)
{
    struct Entry { uint32_t X = 0, mode = 0; int n = 0; std::vector<uint32_t> div; };
    static thread_local Entry cache[8];
    static thread_local unsigned next = 0;
    for (const Entry &e : cache)
        if (e.X == X && e.mode == mode && e.n > 0) {
            std::memcpy(out, e.div.data(), sizeof(uint32_t) * std::min(e.n, (int)MAXDIV));
            return e.n;
        }
    Entry &e = cache[next++ % 8];
    e.div.assign(MAXDIV, 0);
    e.n = list_divisors_uncached(X, mode, e.div.data());
    e.X = X; e.mode = mode;
    std::memcpy(out, e.div.data(), sizeof(uint32_t) * std::min(std::max(e.n, 0), (int)MAXDIV));
    return e.n;
}

int list_divisors_uncached(uint32_t X, uint32_t mode, uint32_t *out)
{
    // trial division up to sqrt(X); ascending order
    std::vector<uint32_t> lo, hi;
    for (uint64_t a = 1; a * a <= X; ++a) {
        if (X % a) continue;
        lo.push_back((uint32_t)a);
        if (a * a != X) hi.push_back((uint32_t)(X / a));
    }
    int n = 0;
    auto keep = [&](uint32_t v) {
        if (mode == 0 && (v & (v - 1))) return;
        if (n < MAXDIV) out[n] = v;
        ++n;
    };
    for (uint32_t v : lo) keep(v);
    for (auto it = hi.rbegin(); it != hi.rend(); ++it) keep(*it);
    return n;
}

// attention as a chain (Sec. III-A): A = Q, B = K^T, D = V, E = O, one instance per head
int chain_of(const mmee_workload *w, mmee_chain &c)
{
    if (!w) return MMEE_EINVAL;
    if (w->reserved || (uint64_t)w->B * w->H > 0xffffffffull) return MMEE_EINVAL;
    c.batch = w->B * w->H;
    c.I = w->N; c.K = w->d; c.L = w->N; c.J = w->d;
    c.word_bytes = w->word_bytes; c.tiling_mode = w->tiling_mode; c.c_softmax = w->c_softmax;
    return MMEE_OK;
}

int make_plan(const mmee_chain *w, const mmee_hw *hw, Plan &p)
{
    if (!w || !hw) return MMEE_EINVAL;
    if (!w->batch || !w->I || !w->K || !w->L || !w->J || !w->word_bytes || w->tiling_mode > 1) return MMEE_EINVAL;
    if (!hw->pe_rows || !hw->pe_cols || !hw->n_arrays) return MMEE_EINVAL;
    if ((uint64_t)hw->rf_bytes < 3ull * w->word_bytes) return MMEE_EINVAL;
    if (!finite_nonneg(hw->e_dram) || !finite_nonneg(hw->e_gb) || !finite_nonneg(hw->e_rf) ||
        !finite_nonneg(hw->e_mac) || !finite_nonneg(hw->dram_bw) || !finite_nonneg(hw->gb_bw))
        return MMEE_EINVAL;
    std::memset(&p, 0, sizeof(p));
    p.dv.X[DI] = w->I; p.dv.X[DK] = w->K; p.dv.X[DL] = w->L; p.dv.X[DJ] = w->J;
    p.T = 1;
    for (int q = 0; q < 4; ++q) {
        int n = list_divisors(p.dv.X[q], w->tiling_mode, p.dv.div[q]);
        if (n <= 0 || n > MAXDIV) return MMEE_EINVAL;
        p.dv.ndiv[q] = (uint32_t)n;
        p.T *= (uint64_t)n;
    }
    if (p.T > (1ull << 22)) return MMEE_EINVAL;
    p.space = p.T * ROWS_PER_TILING;
    // every count of the model must stay an exact integer in fp64
    long double bound = (long double)w->batch * (long double)w->I * w->K * (long double)w->L * w->J *
                        (16.0L + (long double)w->c_softmax) * (long double)w->word_bytes;
    if (bound >= 9007199254740992.0L) return MMEE_EINVAL;
    ModelConst &mc = p.mc;
    mc.BH = (double)w->batch;
    mc.c_lat = mc.BH / (double)hw->n_arrays;
    uint64_t cap = hw->gb_bytes / w->word_bytes;
    mc.cap_words = cap >= (1ull << 53) ? 9007199254740992.0 : (double)cap;
    mc.word = (double)w->word_bytes;
    mc.e_dram = hw->e_dram; mc.e_gb = hw->e_gb; mc.e_rf = hw->e_rf; mc.e_mac = hw->e_mac;
    mc.e_sum = hw->e_dram + hw->e_gb;
    {
        // Per instance, with P = I*K*L*J: DRAM words <= 8 P (four operands at most P each, the
        // unfused intermediate at most I*L*(K+J+2) <= 4 P), buffer<->RF words <= 6 P (three terms
        // per tile matmul, each at most its MAC count; MACs <= 2 P with recomputation), RF accesses
        // 3 * MACs <= 6 P, softmax elements <= P.  The total energy bounds every partial sum.
        auto whole = [](double v) { return v == std::floor(v); };
        const long double P = (long double)w->batch * (long double)w->I * w->K * (long double)w->L * w->J;
        const long double worst = P * (8.0L * hw->e_dram + 14.0L * hw->e_gb + 6.0L * hw->e_rf +
                                       (2.0L + (long double)w->c_softmax) * hw->e_mac);
        p.whole_energies = whole(hw->e_dram) && whole(hw->e_gb) && whole(hw->e_rf) && whole(hw->e_mac);
        p.can_regroup = p.whole_energies && worst < 9007199254740992.0L;
    }
    mc.dram_bw = hw->dram_bw; mc.gb_bw = hw->gb_bw;
    // with a power-of-two bandwidth and array count, (B*H/n) * (words*word/bw) is the B*H-scaled
    // table value times one exactly representable constant
    int ex = 0;
    const bool bw_pow2 = hw->dram_bw == 0.0 || std::frexp(hw->dram_bw, &ex) == 0.5;
    const bool n_pow2 = (hw->n_arrays & (hw->n_arrays - 1)) == 0;
    p.exact_k = bw_pow2 && n_pow2;
    mc.dram_k = hw->dram_bw > 0.0 ? mc.word / hw->dram_bw / (double)hw->n_arrays : 0.0;
    mc.eval_k = hw->dram_bw > 0.0 ? mc.word / hw->dram_bw : 0.0;
    mc.bw_pow2 = bw_pow2 ? 1u : 0u;
    mc.pe_rows = hw->pe_rows; mc.pe_cols = hw->pe_cols;
    mc.g_words = hw->rf_bytes / w->word_bytes / 2;
    mc.gb_pow2 = hw->gb_bw > 0.0 && std::frexp(hw->gb_bw, &ex) == 0.5 ? 1u : 0u;
    mc.gb_k = mc.gb_pow2 ? mc.word / hw->gb_bw : 0.0;
    mc.rcp_rows = 1.0 / (double)mc.pe_rows;
    mc.rcp_cols = 1.0 / (double)mc.pe_cols;
    mc.rcp_cols_g = 1.0 / ((double)mc.pe_cols * (double)mc.g_words);
    mc.c_softmax = w->c_softmax;
    mc.T = (uint32_t)p.T;
    mc.tpad = (uint32_t)((p.T + 63) & ~63ull);
    return MMEE_OK;
}

// ---- device state ------------------------------------------------------------

int ensure_ready()
{
    if (S.ready) return MMEE_OK;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        std::snprintf(g_last_error, sizeof(g_last_error), "no HIP device");
        return MMEE_EDEVICE;
    }
    {
        int dev = 0, cus = 0;
        HIP_TRY(hipGetDevice(&dev));
        HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        S.resident_blocks = (uint32_t)std::max(cus, 1) * BLOCKS_PER_CU;
        // MMEE_RESIDENT_BLOCKS (read once, an even number from 2 up to what the chip holds): fewer persistent
        // blocks, i.e. another split of the work over blocks and another order of the reduction.  Results do
        // not depend on it; it exists so that a test can show that.
        if (const char *env = std::getenv("MMEE_RESIDENT_BLOCKS")) {
            const long v = std::atol(env);
            if (v >= 2 && v % 2 == 0 && (uint64_t)v <= S.resident_blocks) S.resident_blocks = (uint32_t)v;
        }
    }
    HIP_TRY(hipMalloc(&S.enc, sizeof(uint4) * N_DFROWS));
    HIP_TRY(hipMalloc(&S.sig, sizeof(uint32_t) * N_DFROWS));
    HIP_TRY(hipMalloc(&S.flags, N_DFROWS));
    HIP_TRY(hipMalloc(&S.rows[0], sizeof(uint32_t) * N_DFROWS));
    HIP_TRY(hipMalloc(&S.rows[1], sizeof(uint32_t) * N_DFROWS));
    HIP_TRY(hipMalloc(&S.counts_dev, sizeof(uint32_t) * 8));
    HIP_TRY(hipMalloc(&S.key_dev, sizeof(Key) * N_OBJ));
    HIP_TRY(hipMalloc(&S.ticket, 2 * sizeof(uint32_t)));        // [0] finish ticket, [1] work counter
    HIP_TRY(hipMalloc(&S.hints, N_OBJ * sizeof(unsigned long long)));
    {
        // +inf until a launch lowers them; the last block of every launch puts +inf back
        static const unsigned long long inf_bits[N_OBJ] = {INF_BITS, INF_BITS, INF_BITS, INF_BITS};
        HIP_TRY(hipMemcpyAsync(S.hints, inf_bits, sizeof(inf_bits), hipMemcpyHostToDevice, S.stream));
    }
    // on the library's stream, like the kernels that follow: a caller's non-blocking stream is not
    // ordered against the null stream
    HIP_TRY(hipMemsetAsync(S.ticket, 0, 2 * sizeof(uint32_t), S.stream));
    HIP_TRY(hipMemsetAsync(S.rows[0], 0, sizeof(uint32_t) * N_DFROWS, S.stream));
    HIP_TRY(hipMemsetAsync(S.rows[1], 0, sizeof(uint32_t) * N_DFROWS, S.stream));
    for (int w = 0; w < 2; ++w) {
        HIP_TRY(hipMalloc(&S.row_enc[w], sizeof(uint4) * N_DFROWS));
        HIP_TRY(hipMemsetAsync(S.row_enc[w], 0, sizeof(uint4) * N_DFROWS, S.stream));
    }
    // offline stage: encode every (order, levels, r, f) row, prune, compact
    hipLaunchKernelGGL(k_build_rows, dim3((N_DFROWS + 255) / 256), dim3(256), 0, S.stream, S.enc, S.sig);
    hipLaunchKernelGGL(k_prune_rows, dim3((ROWS_PER_GROUP + 255) / 256, N_GROUPS), dim3(256), 0, S.stream, S.sig,
                       S.flags);
    hipLaunchKernelGGL(k_compact_rows, dim3(8), dim3(1024), 0, S.stream, S.flags, S.enc, S.rows[0], S.rows[1],
                       S.row_enc[0], S.row_enc[1],
                       S.counts_dev);
    HIP_TRY(hipGetLastError());
    uint32_t h[8];
    HIP_TRY(hipMemcpyAsync(h, S.counts_dev, sizeof(h), hipMemcpyDeviceToHost, S.stream));
    HIP_TRY(hipStreamSynchronize(S.stream));
    for (int g = 0; g < 4; ++g) { S.counts[0][g] = h[g]; S.counts[1][g] = h[4 + g]; }
    {
        // whether a row denotes a dataflow depends on (order, r, f) only: list those classes
        std::vector<uint8_t> flags(N_DFROWS);
        HIP_TRY(hipMemcpy(flags.data(), S.flags, N_DFROWS, hipMemcpyDeviceToHost));
        std::vector<uint32_t> cls;
        for (uint32_t g = 0; g < N_GROUPS; ++g)
            for (uint32_t rank = 0; rank < 24; ++rank) {
                uint32_t on = 0;
                for (uint32_t q = 0; q < 625; ++q) on += flags[g * ROWS_PER_GROUP + rank * 625 + q] & 1u;
                if (on != 0 && on != 625) {
                    std::snprintf(g_last_error, sizeof(g_last_error), "row validity is not uniform within a class");
                    return MMEE_EDEVICE;
                }
                if (on) cls.push_back(rank + 24 * g);
            }
        uint64_t rows = 0;
        for (int g = 0; g < 4; ++g) rows += S.counts[0][g];
        if (cls.empty() || cls.size() * 625ull != rows) {
            std::snprintf(g_last_error, sizeof(g_last_error), "class list does not match the row list");
            return MMEE_EDEVICE;
        }
        HIP_TRY(hipMalloc(&S.cls_dev, sizeof(uint32_t) * 96));
        HIP_TRY(hipMemcpy(S.cls_dev, cls.data(), sizeof(uint32_t) * cls.size(), hipMemcpyHostToDevice));
        S.n_cls = (uint32_t)cls.size();
    }
    {
        // Batched search over the surviving rows.  The rows refer to a subset of the table entries only:
        // the kernel stages just those, and a row becomes the eight byte offsets of its values in that
        // compact table.  Lists follow each other group by group.
        std::vector<uint4> rows;
        std::vector<uint32_t> group_first(N_GROUPS + 1, 0);
        for (uint32_t g = 0; g < N_GROUPS; ++g) {
            const uint32_t n = S.counts[1][g];
            group_first[g] = (uint32_t)rows.size();
            if (!n) continue;
            rows.resize(rows.size() + n);
            HIP_TRY(hipMemcpy(rows.data() + group_first[g], S.row_enc[1] + (size_t)g * ROWS_PER_GROUP, sizeof(uint4) * n,
                              hipMemcpyDeviceToHost));
        }
        group_first[N_GROUPS] = (uint32_t)rows.size();
        auto sel_at = [](const uint4 &e, int k) { const uint32_t w = k < 4 ? e.x : e.y; return (w >> (8 * (k & 3))) & 0xFFu; };
        std::vector<int> compact(NENT, -1);
        std::vector<uint32_t> used;
        for (const uint4 &e : rows)
            for (int k = 0; k < NSEL; ++k) compact[sel_at(e, k)] = 0;
        for (uint32_t ent = 0; ent < (uint32_t)NENT; ++ent)
            if (compact[ent] == 0) { compact[ent] = (int)used.size(); used.push_back(ent); }
        S.batch_rows = (uint32_t)rows.size();
        S.batch_n_used = (uint32_t)used.size();
        S.batch_ok = !rows.empty() && rows.size() <= BATCH_MAX_ROWS && used.size() <= BATCH_MAX_USED;
        if (S.batch_ok) {
            std::vector<uint32_t> off(rows.size() * 8), df(rows.size());
            for (size_t i = 0; i < rows.size(); ++i) {
                for (int k = 0; k < NSEL; ++k) off[i * 8 + k] = (uint32_t)compact[sel_at(rows[i], k)] * BATCH_TC * 8u;
                df[i] = rows[i].w;
            }
            HIP_TRY(hipMalloc(&S.batch_row_off, sizeof(uint32_t) * off.size()));
            HIP_TRY(hipMalloc(&S.batch_row_df, sizeof(uint32_t) * df.size()));
            std::vector<uint32_t> cmap(NENT);
            for (int ent = 0; ent < NENT; ++ent) cmap[ent] = compact[ent] < 0 ? 0xFFFFu : (uint32_t)compact[ent];
            HIP_TRY(hipMalloc(&S.batch_cmap, sizeof(uint32_t) * NENT));
            HIP_TRY(hipMemcpy(S.batch_row_off, off.data(), sizeof(uint32_t) * off.size(), hipMemcpyHostToDevice));
            HIP_TRY(hipMemcpy(S.batch_row_df, df.data(), sizeof(uint32_t) * df.size(), hipMemcpyHostToDevice));
            HIP_TRY(hipMemcpy(S.batch_cmap, cmap.data(), sizeof(uint32_t) * NENT, hipMemcpyHostToDevice));
        }
        // share the rows of each group out over the waves of a block, every wave a contiguous piece of
        // one group's list (rows of one group share r and f)
        uint32_t waves[N_GROUPS] = {0, 0, 0, 0}, taken = 0;
        for (uint32_t g = 0; g < N_GROUPS; ++g)
            if (S.counts[1][g]) { waves[g] = 1; ++taken; }
        while (taken < BATCH_WAVES) {
            uint32_t worst = N_GROUPS, most = 0;
            for (uint32_t g = 0; g < N_GROUPS; ++g) {
                if (!waves[g]) continue;
                const uint32_t per = (S.counts[1][g] + waves[g] - 1) / waves[g];
                if (per > most) { most = per; worst = g; }
            }
            if (worst == N_GROUPS || most <= 1) break;
            ++waves[worst]; ++taken;
        }
        uint32_t wv = 0;
        for (uint32_t g = 0; g < N_GROUPS; ++g)
            for (uint32_t k = 0; k < waves[g]; ++k, ++wv) {
                const uint32_t n = S.counts[1][g], lo = (uint32_t)((uint64_t)n * k / waves[g]),
                               hi = (uint32_t)((uint64_t)n * (k + 1) / waves[g]);
                S.task_lo[wv] = group_first[g] + lo; S.task_cnt[wv] = hi - lo; S.task_g[wv] = g;
            }
        for (; wv < BATCH_WAVES; ++wv) { S.task_lo[wv] = 0; S.task_cnt[wv] = 0; S.task_g[wv] = 0; }
    }
    S.ready = true;
    return MMEE_OK;
}

int ensure_tilings(uint64_t tpad)
{
    if (tpad <= S.tiling_cap) return MMEE_OK;
    if (S.btab) { HIP_TRY(hipStreamSynchronize(S.stream)); (void)hipFree(S.btab); (void)hipFree(S.ctab_s); (void)hipFree(S.ctab_e); }
    S.btab = nullptr; S.ctab_s = nullptr; S.ctab_e = nullptr; S.tiling_cap = 0;
    HIP_TRY(hipMalloc(&S.btab, sizeof(double) * NENT_ALL * tpad));
    HIP_TRY(hipMalloc(&S.ctab_s, sizeof(double) * 2 * NCS * tpad));
    HIP_TRY(hipMalloc(&S.ctab_e, sizeof(uint64_t) * 2 * NCE * tpad));
    S.tiling_cap = tpad;
    return MMEE_OK;
}

int ensure_partials(size_t nblocks)
{
    if (nblocks <= S.partials_cap) return MMEE_OK;
    if (S.partials) { HIP_TRY(hipStreamSynchronize(S.stream)); (void)hipFree(S.partials); }
    S.partials = nullptr; S.partials_cap = 0;
    HIP_TRY(hipMalloc(&S.partials, sizeof(Key) * N_OBJ * nblocks));
    S.partials_cap = nblocks;
    return MMEE_OK;
}

int ensure_slots(size_t n)
{
    if (n <= S.slots) return MMEE_OK;
    if (S.final_host) {
        HIP_TRY(hipStreamSynchronize(S.stream));
        (void)hipFree(S.dv_dev);
        (void)hipHostFree(S.final_host);
    }
    S.slots = 0; S.final_host = nullptr; S.final_map = nullptr; S.dv_dev = nullptr;
    HIP_TRY(hipMalloc(&S.dv_dev, sizeof(DivTable) * n));
    HIP_TRY(hipHostMalloc(&S.final_host, sizeof(FinalRecord) * N_OBJ * n, hipHostMallocMapped));
    HIP_TRY(hipHostGetDevicePointer(reinterpret_cast<void **>(&S.final_map), S.final_host, 0));
    while (S.events.size() < 2 * n) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        S.events.push_back(e);
    }
    S.slots = n;
    return MMEE_OK;
}

// the model constants of one pass: whether the energy is regrouped is settled here, for the tables
// and for the kernel alike
//
// Beyond the size bound the sum may still be regrouped for the scalar keys other than the
// energy-delay product, subject to a check of the outcome (`*unproven` is set): all terms are
// non-negative whole numbers, so a candidate whose true total is below 2^53 is exact in either
// order, and any other candidate computes to more than 2^52 in either order.  An optimum below
// 2^52 pJ therefore is the optimum of the term-by-term sum too, ties included; otherwise the
// caller repeats the pass with MMEE_SEARCH_ORDERED_SUM.
constexpr double REGROUP_PROOF_LIMIT = 4503599627370496.0;   // 2^52
ModelConst pass_constants(const Plan &p, uint32_t flags, int mask = 8, bool *unproven = nullptr)
{
    ModelConst mc = p.mc;
    const bool allowed = p.exact_k && !(flags & MMEE_SEARCH_ORDERED_SUM);
    const bool on_trust = allowed && !p.can_regroup && p.whole_energies && !(mask & 8) && unproven;
    mc.regroup = ((allowed && p.can_regroup) || on_trust) ? 1u : 0u;
    if (unproven) *unproven = on_trust;
    return mc;
}

// the tables of one problem into b's table buffers (which must hold mc.tpad tilings)
int launch_tilings(const Plan &p, const ModelConst &mc, const Bufs &b, DivTable *dv_copy = nullptr)
{
    hipLaunchKernelGGL(k_build_tilings, dim3(mc.tpad / 64), dim3(64 * BUILD_PARTS), 0, S.stream, p.dv, mc, b.btab,
                       b.ctab_s, b.ctab_e, dv_copy);
    HIP_TRY(hipGetLastError());
    return MMEE_OK;
}

// the cached, growing buffers of the allocating entry points, for the pass in result slot `slot`
int state_bufs(const Plan &p, size_t slot, Bufs &b)
{
    if (slot >= S.slots) return MMEE_EINVAL;
    int rc = ensure_tilings(p.mc.tpad);
    if (rc) return rc;
    // persistent blocks: never more than the chip holds at once
    rc = ensure_partials(S.resident_blocks);
    if (rc) return rc;
    b.enc = S.enc;
    for (int w = 0; w < 2; ++w) {
        b.rows[w] = S.rows[w]; b.row_enc[w] = S.row_enc[w];
        for (int g = 0; g < 4; ++g) b.counts[w][g] = S.counts[w][g];
    }
    b.cls_dev = S.cls_dev; b.n_cls = S.n_cls;
    b.btab = S.btab; b.ctab_s = S.ctab_s; b.ctab_e = S.ctab_e;
    b.partials = S.partials; b.partials_cap = S.partials_cap;
    b.ticket = S.ticket; b.hints = S.hints; b.key_dev = S.key_dev;
    b.final_dev = S.final_map + N_OBJ * slot;
    b.dv_dev = S.dv_dev + slot;
    b.ev_begin = S.events[2 * slot]; b.ev_end = S.events[2 * slot + 1];
    b.resident_blocks = S.resident_blocks;
    return MMEE_OK;
}

template <int MASK>
void launch_search_mask(bool exact_k, dim3 grid, const SearchArgs &a)
{
    if (a.mc.regroup) hipLaunchKernelGGL((k_search<MASK, true, false, true>), grid, dim3(SEARCH_THREADS), 0, S.stream, a);
    else if (exact_k) hipLaunchKernelGGL((k_search<MASK, true>), grid, dim3(SEARCH_THREADS), 0, S.stream, a);
    else hipLaunchKernelGGL((k_search<MASK, false>), grid, dim3(SEARCH_THREADS), 0, S.stream, a);
}

// one step of the Pareto walk: latency-then-energy among candidates with energy below a.e_limit
void launch_search_limited(bool exact_k, dim3 grid, const SearchArgs &a)
{
    if (a.mc.regroup) hipLaunchKernelGGL((k_search<4, true, true, true>), grid, dim3(SEARCH_THREADS), 0, S.stream, a);
    else if (exact_k) hipLaunchKernelGGL((k_search<4, true, true>), grid, dim3(SEARCH_THREADS), 0, S.stream, a);
    else hipLaunchKernelGGL((k_search<4, false, true>), grid, dim3(SEARCH_THREADS), 0, S.stream, a);
}

template <int MASK>
void launch_dense_mask(bool exact_k, dim3 grid, const SearchArgs &a)
{
    if (a.mc.regroup) hipLaunchKernelGGL((k_search_dense<MASK, true, false, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
    else if (exact_k) hipLaunchKernelGGL((k_search_dense<MASK, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
    else hipLaunchKernelGGL((k_search_dense<MASK, false>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
}

// second pass of the (latency, energy) key: lowest energy among the candidates within a.lat_cap
void launch_dense_latcap(bool exact_k, dim3 grid, const SearchArgs &a)
{
    if (a.mc.regroup) hipLaunchKernelGGL((k_search_dense<1, true, false, true, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
    else if (exact_k) hipLaunchKernelGGL((k_search_dense<1, true, false, false, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
    else hipLaunchKernelGGL((k_search_dense<1, false, false, false, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
}

// first pass of one step of the Pareto walk over the full row set: lowest latency among the candidates
// with energy below a.e_limit (the second pass is launch_dense_latcap)
void launch_dense_limited(bool exact_k, dim3 grid, const SearchArgs &a)
{
    if (a.mc.regroup) hipLaunchKernelGGL((k_search_dense<2, true, true, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
    else if (exact_k) hipLaunchKernelGGL((k_search_dense<2, true, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
    else hipLaunchKernelGGL((k_search_dense<2, false, true>), grid, dim3(DENSE_THREADS), 0, S.stream, a);
}

// enqueue one pass (tables + search; the final records land in b.final_dev) in the buffers b
int enqueue_search_in(const Bufs &B, const Plan &p, int mask, uint32_t flags, uint64_t *evaluated,
                      const double *e_limit = nullptr, bool build_tables = true, bool bs_da_step = false,
                      bool *unproven = nullptr)
{
    const ModelConst mc = pass_constants(p, flags, bs_da_step ? 8 : mask, unproven);
    int rc = build_tables ? launch_tilings(p, mc, B, B.dv_dev) : MMEE_OK;
    if (rc) return rc;
    const int which = (flags & MMEE_SEARCH_EXHAUSTIVE) ? 0 : 1;
    SearchArgs a;
    std::memset(&a, 0, sizeof(a));
    a.enc = B.enc; a.rows = B.rows[which]; a.row_enc = B.row_enc[which];
    // rows: one slot numbering per recomputation class r, over the lists of (r, f=0) and (r, f=1)
    uint32_t rb = 0;
    uint64_t nrows = 0;
    for (uint32_t r = 0; r < 2; ++r) {
        uint32_t in_class = 0;
        for (uint32_t f = 0; f < 2; ++f) {
            const uint32_t g = r + 2 * f;
            a.cls_off[r][f] = g * ROWS_PER_GROUP;
            a.cls_cnt[r][f] = B.counts[which][g];
            in_class += B.counts[which][g];
        }
        if (r == 0) a.rb_split = (in_class + SEARCH_THREADS - 1) / SEARCH_THREADS;
        rb += (in_class + SEARCH_THREADS - 1) / SEARCH_THREADS;
        nrows += in_class;
        // a short list fills few waves: let them come several times, each with a share of the tilings
        const uint32_t waves_for_rows = (in_class + 63) / 64;
        a.wave_split[r] = (!bs_da_step && waves_for_rows >= 1 && waves_for_rows <= 4) ? (SEARCH_THREADS / 64) / waves_for_rows : 1u;
    }
    const bool short_lists = a.wave_split[0] > 1 || a.wave_split[1] > 1;
    if (rb == 0) return MMEE_EINVAL;
    a.n_rb = rb;
    // tilings: chunks of TC, then chunks of TC_FINE worth about four fine items per resident block
    // (a coarse item's time), at least the ragged end
    {
        // (short lists split an item's tilings over the waves instead: short chunks only while one
        // round of blocks takes them all)
        const uint64_t all_fine = (p.T + TC_FINE - 1) / TC_FINE;
        const uint64_t fine_chunks_wanted = short_lists ? (rb * all_fine <= B.resident_blocks ? all_fine : 0)
                                                        : (4ull * B.resident_blocks + rb - 1) / rb;
        const uint64_t fine_tilings = std::min<uint64_t>(p.T, fine_chunks_wanted * TC_FINE);
        a.n_cc = (uint32_t)((p.T - fine_tilings) / TC);
        a.n_fc = (uint32_t)((p.T - (uint64_t)a.n_cc * TC + TC_FINE - 1) / TC_FINE);
    }
    a.btab = B.btab; a.ctab_s = B.ctab_s; a.ctab_e = B.ctab_e;
    a.mc = mc;
    // One key over the full row set goes through the dense kernel (lane = tiling, wave = 125 rows of
    // a class).  With several keys its accumulators no longer fit four waves per SIMD, and the
    // row-per-lane kernel is the faster one.
    const bool dense = which == 0 && !bs_da_step && (mask & (mask - 1)) == 0 && B.cls_dev;
    uint64_t n_items;
    if (dense) {
        a.cls = B.cls_dev; a.n_cls = B.n_cls;
        const uint32_t n_chunks = (uint32_t)((p.T + TC - 1) / TC);
        a.d_gc = (B.n_cls * 5 + DENSE_WAVES - 1) / DENSE_WAVES;
        a.d_gf = (B.n_cls * 25 + DENSE_WAVES - 1) / DENSE_WAVES;
        // fifths of tasks for the last chunks: about one whole-task item per resident block
        const uint32_t dense_blocks = B.resident_blocks / BLOCKS_PER_CU * DENSE_BLOCKS_PER_CU;
        const uint32_t fine_chunks = std::min<uint32_t>(n_chunks, (dense_blocks + a.d_gc - 1) / a.d_gc);
        a.d_ncc = n_chunks - fine_chunks;
        a.n_coarse_items = a.d_ncc * a.d_gc;
        n_items = (uint64_t)a.n_coarse_items + (uint64_t)fine_chunks * a.d_gf;
    } else {
        n_items = (uint64_t)rb * ((uint64_t)a.n_cc + a.n_fc);
        a.n_coarse_items = rb * a.n_cc;
    }
    if (n_items == 0 || n_items > 0x7fffffffull) return MMEE_EINVAL;
    a.n_items = (uint32_t)n_items;
    // persistent blocks: as many as the chip holds at once (LDS allows two per CU)
    const uint64_t nblocks = std::min<uint64_t>(
        n_items, dense ? (uint64_t)B.resident_blocks / BLOCKS_PER_CU * DENSE_BLOCKS_PER_CU : (uint64_t)B.resident_blocks);
    if (nblocks > B.partials_cap) return MMEE_EINVAL;
    a.partials = B.partials; a.ticket = B.ticket; a.work_counter = B.ticket + 1; a.hints = B.hints;
    a.final_out = B.final_dev;
    a.dv = B.dv_dev;
    if (B.ev_begin) HIP_TRY(hipEventRecord(B.ev_begin, S.stream));
    dim3 grid((uint32_t)nblocks);
    if (bs_da_step) {
        if (!e_limit) return MMEE_EINVAL;
        a.e_limit = *e_limit;
        hipLaunchKernelGGL(k_front_step, grid, dim3(SEARCH_THREADS), 0, S.stream, a);
    } else if (e_limit) {
        if (mask != 4) return MMEE_EINVAL;
        a.e_limit = *e_limit;
        if (dense) {
            // two scalar passes, as for the unbounded key below; the second needs no energy bound: the
            // lowest energy among the candidates within the latency found is below it
            SearchArgs first = a, second = a;
            first.final_key_dev = B.key_dev;
            launch_dense_limited(p.exact_k, grid, first);
            second.lat_cap = B.key_dev + 1;
            second.final_out = a.final_out + 2;
            launch_dense_latcap(p.exact_k, grid, second);
        } else
            launch_search_limited(p.exact_k, grid, a);
    } else if (dense && mask == 4) {
        // The (latency, energy) key over the full row set, as two passes that each cost what a
        // single scalar key costs: the lowest latency first, then the lowest energy among the
        // candidates that reach it (a candidate's latency is a maximum of a row part and a
        // combination part, so the cap applies to the two separately).  The second pass's energy
        // record lands in the slot of this key.
        SearchArgs first = a, second = a;
        first.final_key_dev = B.key_dev;
        launch_dense_mask<2>(p.exact_k, grid, first);
        second.lat_cap = B.key_dev + 1;
        second.final_out = a.final_out + 2;
        launch_dense_latcap(p.exact_k, grid, second);
    } else if (dense)
    switch (mask) {
    case 1: launch_dense_mask<1>(p.exact_k, grid, a); break;
    case 2: launch_dense_mask<2>(p.exact_k, grid, a); break;
    case 4: launch_dense_mask<4>(p.exact_k, grid, a); break;
    case 8: launch_dense_mask<8>(p.exact_k, grid, a); break;
    default: return MMEE_EINVAL;
    }
    else
    switch (mask) {
    case 1: launch_search_mask<1>(p.exact_k, grid, a); break;
    case 2: launch_search_mask<2>(p.exact_k, grid, a); break;
    case 3: launch_search_mask<3>(p.exact_k, grid, a); break;
    case 4: launch_search_mask<4>(p.exact_k, grid, a); break;
    case 5: launch_search_mask<5>(p.exact_k, grid, a); break;
    case 6: launch_search_mask<6>(p.exact_k, grid, a); break;
    case 7: launch_search_mask<7>(p.exact_k, grid, a); break;
    case 8: launch_search_mask<8>(p.exact_k, grid, a); break;
    case 9: launch_search_mask<9>(p.exact_k, grid, a); break;
    case 10: launch_search_mask<10>(p.exact_k, grid, a); break;
    case 11: launch_search_mask<11>(p.exact_k, grid, a); break;
    case 12: launch_search_mask<12>(p.exact_k, grid, a); break;
    case 13: launch_search_mask<13>(p.exact_k, grid, a); break;
    case 14: launch_search_mask<14>(p.exact_k, grid, a); break;
    case 15: launch_search_mask<15>(p.exact_k, grid, a); break;
    default: return MMEE_EINVAL;
    }
    HIP_TRY(hipGetLastError());
    if (B.ev_end) HIP_TRY(hipEventRecord(B.ev_end, S.stream));
    *evaluated = nrows * p.T * (bs_da_step ? 1ull : 9ull);
    return MMEE_OK;
}

// the same in the cached buffers of the allocating entry points, result slot `slot`
int enqueue_search(const Plan &p, int mask, uint32_t flags, size_t slot, uint64_t *evaluated,
                   const double *e_limit = nullptr, bool build_tables = true, bool bs_da_step = false,
                   bool *unproven = nullptr)
{
    Bufs b;
    int rc = state_bufs(p, slot, b);
    if (rc) return rc;
    return enqueue_search_in(b, p, mask, flags, evaluated, e_limit, build_tables, bs_da_step, unproven);
}

static_assert(sizeof(BatchArgs) <= 4096, "kernel arguments are limited to 4 KiB");

// ---- batched search over the pruned rows -----------------------------------------------------

// masks the batched kernel is built for; other key sets take the per-problem kernels
bool batch_mask(int mask) { return mask == 1 || mask == 2 || mask == 3 || mask == 4 || mask == 8; }

int ensure_batch(size_t blob_bytes, size_t n_items)
{
    if (blob_bytes > S.batch_blob_cap) {
        if (S.batch_host) { HIP_TRY(hipStreamSynchronize(S.stream)); (void)hipHostFree(S.batch_host); (void)hipFree(S.batch_dev); }
        S.batch_host = nullptr; S.batch_dev = nullptr; S.batch_blob_cap = 0;
        const size_t cap = std::max<size_t>(blob_bytes * 2, 1 << 16);
        HIP_TRY(hipHostMalloc(&S.batch_host, cap, hipHostMallocDefault));
        HIP_TRY(hipMalloc(&S.batch_dev, cap));
        S.batch_blob_cap = cap;
    }
    if (n_items > S.item_cap) {
        if (S.item_keys) { HIP_TRY(hipStreamSynchronize(S.stream)); (void)hipFree(S.item_keys); }
        S.item_keys = nullptr; S.item_cap = 0;
        const size_t cap = std::max<size_t>(n_items * 2, 4096);
        HIP_TRY(hipMalloc(&S.item_keys, sizeof(Key) * N_OBJ * cap));
        S.item_cap = cap;
    }
    return MMEE_OK;
}

template <int MASK>
void launch_batch_mask(bool fast, bool regroup, dim3 grid, const BatchArgs &a)
{
    if (regroup) hipLaunchKernelGGL((k_search_batch<MASK, true, true>), grid, dim3(BATCH_THREADS), 0, S.stream, a);
    else if (fast) hipLaunchKernelGGL((k_search_batch<MASK, true, false>), grid, dim3(BATCH_THREADS), 0, S.stream, a);
    else hipLaunchKernelGGL((k_search_batch<MASK, false, false>), grid, dim3(BATCH_THREADS), 0, S.stream, a);
    // the problems' records are complete when the search kernel has ended: one block per problem finishes
    hipLaunchKernelGGL((k_batch_finish<MASK>), dim3(a.n_prob), dim3(256), 0, S.stream, a);
}

// One problem of a batched launch, as the host sees it.
struct BatchEntry {
    const Plan *plan;
    int mask;
    size_t slot;            // result slot: its N_OBJ final records
    ModelConst mc;          // with the regrouping decision taken
    bool unproven;          // regrouped on trust (pass_constants)
    uint64_t evaluated;
};

// Enqueue the entries (all pruned searches) as few launches as their kernel variants allow: one per
// (key set, exact DRAM constant, regrouped) combination present.  Events of slot `ev_slot` bracket it all.
int enqueue_batches(std::vector<BatchEntry> &entries, uint32_t flags, size_t ev_slot)
{
    if (entries.empty()) return MMEE_OK;
    struct Variant { int mask; bool fast, regroup; std::vector<size_t> members; uint64_t items = 0; uint32_t split = 1; };
    std::vector<Variant> variants;
    uint64_t kept_rows = 0;
    for (int g = 0; g < 4; ++g) kept_rows += S.counts[1][g];
    uint64_t total_items = 0;
    for (size_t k = 0; k < entries.size(); ++k) {
        BatchEntry &e = entries[k];
        e.mc = pass_constants(*e.plan, flags, e.mask, &e.unproven);
        e.evaluated = kept_rows * e.plan->T * 9ull;
        const bool fast = e.plan->exact_k, regroup = e.mc.regroup != 0;
        Variant *v = nullptr;
        for (Variant &c : variants)
            if (c.mask == e.mask && c.fast == fast && c.regroup == regroup) v = &c;
        if (!v) { variants.push_back(Variant{e.mask, fast, regroup, {}, 0, 1}); v = &variants.back(); }
        v->members.push_back(k);
        v->items += (e.plan->T + BATCH_TC - 1) / BATCH_TC;
    }
    for (Variant &v : variants) {
        // a launch with few chunks leaves most of the chip idle: let several blocks share a chunk's rows
        while (v.split < BATCH_MAX_SPLIT && v.items * v.split * 2 <= S.resident_blocks) v.split *= 2;
        v.items *= v.split;
        total_items += v.items;
    }
    if (total_items > 0x7fffffffull) return MMEE_EINVAL;
    auto fill_head = [&](BatchProblemHead &h, uint32_t *list, const BatchEntry &e, uint32_t first_item, uint32_t split) {
        h.mc = e.mc;
        h.first_item = first_item;
        h.n_work = (uint32_t)((e.plan->T + BATCH_TC - 1) / BATCH_TC) * split;
        h.slot = (uint32_t)e.slot;
        h.pad_ = 0;
        uint32_t at = 0;
        for (int q = 0; q < 4; ++q) {
            h.X[q] = e.plan->dv.X[q];
            h.ndiv[q] = e.plan->dv.ndiv[q];
            for (uint32_t k = 0; k < h.ndiv[q]; ++k) list[at++] = e.plan->dv.div[q][k];
        }
    };
    auto list_len = [](const Plan &pl) { return pl.dv.ndiv[0] + pl.dv.ndiv[1] + pl.dv.ndiv[2] + pl.dv.ndiv[3]; };
    // A variant with one problem whose divisor lists fit carries it in the kernel arguments; the others'
    // descriptors go through one blob: per variant its problem descriptors, then its first-item table.
    auto rides_in_arguments = [&](const Variant &v) {
        return v.members.size() == 1 && list_len(*entries[v.members[0]].plan) <= (uint32_t)BATCH_INLINE_DIVS;
    };
    size_t blob = 0;
    for (const Variant &v : variants)
        if (!rides_in_arguments(v))
            blob += sizeof(BatchProblem) * v.members.size() + sizeof(uint32_t) * ((v.members.size() + 1 + 3) & ~(size_t)3);
    int rc = ensure_batch(blob, total_items);
    if (rc) return rc;
    size_t off = 0;
    uint64_t item0 = 0;
    struct Launch { size_t desc_off, firsts_off, n_prob; uint64_t item0, n_items; bool in_args; };
    std::vector<Launch> launches;
    for (const Variant &v : variants) {
        Launch L;
        L.desc_off = L.firsts_off = 0;
        L.n_prob = v.members.size(); L.item0 = item0; L.n_items = v.items; L.in_args = rides_in_arguments(v);
        item0 += v.items;
        if (!L.in_args) {
            L.desc_off = off;
            BatchProblem *bp = reinterpret_cast<BatchProblem *>(S.batch_host + off);
            off += sizeof(BatchProblem) * v.members.size();
            L.firsts_off = off;
            uint32_t *firsts = reinterpret_cast<uint32_t *>(S.batch_host + off);
            off += sizeof(uint32_t) * ((v.members.size() + 1 + 3) & ~(size_t)3);
            uint32_t item = 0;
            for (size_t k = 0; k < v.members.size(); ++k) {
                fill_head(bp[k].h, bp[k].list, entries[v.members[k]], item, v.split);
                firsts[k] = item;
                item += bp[k].h.n_work;
            }
            firsts[v.members.size()] = item;
        }
        launches.push_back(L);
    }
    HIP_TRY(hipEventRecord(S.events[2 * ev_slot], S.stream));
    if (off) HIP_TRY(hipMemcpyAsync(S.batch_dev, S.batch_host, off, hipMemcpyHostToDevice, S.stream));
    for (size_t k = 0; k < variants.size(); ++k) {
        const Variant &v = variants[k];
        const Launch &L = launches[k];
        BatchArgs a;
        std::memset(&a, 0, sizeof(a));
        if (L.in_args) {
            fill_head(a.inl.h, a.inl.list, entries[v.members[0]], 0, v.split);
            a.inl.firsts[0] = 0; a.inl.firsts[1] = a.inl.h.n_work;
            a.inl.on = 1;
        } else {
            a.prob = reinterpret_cast<const BatchProblem *>(S.batch_dev + L.desc_off);
            a.first_items = reinterpret_cast<const uint32_t *>(S.batch_dev + L.firsts_off);
        }
        a.n_prob = (uint32_t)L.n_prob; a.n_items = (uint32_t)L.n_items;
        a.enc = S.enc;
        a.row_off = S.batch_row_off; a.row_df = S.batch_row_df; a.cmap = S.batch_cmap;
        a.n_rows = S.batch_rows; a.n_used = S.batch_n_used;
        // every wave's piece of its group's list, cut once more into one sub-piece per row share
        a.split = v.split;
        for (a.split_log2 = 0; (1u << a.split_log2) < v.split; ++a.split_log2) {}
        for (uint32_t sh = 0; sh < v.split; ++sh)
            for (int wv = 0; wv < BATCH_WAVES; ++wv) {
                const uint32_t n = S.task_cnt[wv], lo = n * sh / v.split, hi = n * (sh + 1) / v.split;
                a.task_lo[sh * BATCH_WAVES + wv] = S.task_lo[wv] + lo;
                a.task_cnt[sh * BATCH_WAVES + wv] = hi - lo;
                a.task_g[sh * BATCH_WAVES + wv] = S.task_g[wv];
            }
        a.item_keys = S.item_keys + N_OBJ * L.item0;
        a.final_out = S.final_map;
        // persistent blocks, two per CU, each with a contiguous range of the items
        dim3 grid((uint32_t)std::min<uint64_t>(L.n_items, (uint64_t)S.resident_blocks));
        a.per_block = (uint32_t)((L.n_items + grid.x - 1) / grid.x);
        switch (v.mask) {
        case 1: launch_batch_mask<1>(v.fast, v.regroup, grid, a); break;
        case 2: launch_batch_mask<2>(v.fast, v.regroup, grid, a); break;
        case 3: launch_batch_mask<3>(v.fast, v.regroup, grid, a); break;
        case 4: launch_batch_mask<4>(v.fast, v.regroup, grid, a); break;
        case 8: launch_batch_mask<8>(v.fast, v.regroup, grid, a); break;
        default: return MMEE_EINVAL;
        }
    }
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipEventRecord(S.events[2 * ev_slot + 1], S.stream));
    return MMEE_OK;
}

int unpack_result(const Plan &p, size_t slot, int objective, uint64_t evaluated, double seconds, double ksec,
                  mmee_result *out)
{
    const FinalRecord &fr = S.final_host[N_OBJ * slot + objective];
    std::memset(out, 0, sizeof(*out));
    std::memcpy(&out->cost, fr.cost, sizeof(mmee_cost));
    std::memcpy(&out->best, fr.map, sizeof(mmee_mapping));
    out->space = p.space;
    out->evaluated = evaluated;
    out->seconds = seconds;
    out->kernel_seconds = ksec;
    if (!(fr.key.p < INFINITY)) { out->cost.valid = 0; return MMEE_ENOFEASIBLE; }
    return MMEE_OK;
}

bool same_problem(const mmee_chain &a, const mmee_hw &b, const mmee_chain &c, const mmee_hw &d)
{
    return std::memcmp(&a, &c, sizeof(a)) == 0 && b.pe_rows == d.pe_rows && b.pe_cols == d.pe_cols &&
           b.n_arrays == d.n_arrays && b.rf_bytes == d.rf_bytes && b.gb_bytes == d.gb_bytes &&
           b.e_dram == d.e_dram && b.e_gb == d.e_gb && b.e_rf == d.e_rf && b.e_mac == d.e_mac &&
           b.dram_bw == d.dram_bw && b.gb_bw == d.gb_bw;
}

double now_seconds()
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

// ---- the entry point that allocates nothing: per-device set-up of the fixed scratch -----------

constexpr int NOALLOC_MAX_DEVICES = 64;
struct NoAllocDevice {
    unsigned char *ptr = nullptr;        // this device's copy of `scratch`
    bool built = false;                  // offline stage done in it
    uint32_t counts[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    uint32_t resident_blocks = 0;
} g_noalloc[NOALLOC_MAX_DEVICES];

// First call on a device: the address of that device's array, then the offline stage (row encoding,
// pruning, compaction) into it and its eight counts back to the host.  Nothing is allocated.
int noalloc_setup(int dev, NoAllocDevice *&out)
{
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return MMEE_EINVAL;
    NoAllocDevice &d = g_noalloc[dev];
    out = &d;
    if (d.built) return MMEE_OK;
    if (!d.ptr) {
        unsigned char *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) {
            std::snprintf(g_last_error, sizeof(g_last_error), "hipGetSymbolAddress returned no address for the scratch array");
            return MMEE_EDEVICE;
        }
        d.ptr = ptr;
    }
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    d.resident_blocks = std::min<uint32_t>((uint32_t)std::max(cus, 1) * BLOCKS_PER_CU, noalloc::MAX_BLOCKS);
    unsigned char *q = d.ptr;
    uint4 *enc = reinterpret_cast<uint4 *>(q + noalloc::OFF_ENC);
    uint32_t *sig = reinterpret_cast<uint32_t *>(q + noalloc::OFF_SIG);
    uint8_t *flags = q + noalloc::OFF_FLAGS;
    uint32_t *rows0 = reinterpret_cast<uint32_t *>(q + noalloc::OFF_ROWS0);
    uint32_t *rows1 = reinterpret_cast<uint32_t *>(q + noalloc::OFF_ROWS1);
    uint4 *renc0 = reinterpret_cast<uint4 *>(q + noalloc::OFF_RENC0);
    uint4 *renc1 = reinterpret_cast<uint4 *>(q + noalloc::OFF_RENC1);
    uint32_t *counts = reinterpret_cast<uint32_t *>(q + noalloc::OFF_COUNTS);
    // the row lists must read as zero beyond their ends (lanes without a row read entry 0 of a list)
    const uint32_t list_words = (uint32_t)((noalloc::OFF_COUNTS - noalloc::OFF_ROWS0) / 4);
    hipLaunchKernelGGL(k_clear_words, dim3((list_words + 255) / 256), dim3(256), 0, S.stream, rows0, list_words);
    hipLaunchKernelGGL(k_build_rows, dim3((N_DFROWS + 255) / 256), dim3(256), 0, S.stream, enc, sig);
    hipLaunchKernelGGL(k_prune_rows, dim3((ROWS_PER_GROUP + 255) / 256, N_GROUPS), dim3(256), 0, S.stream, sig, flags);
    hipLaunchKernelGGL(k_compact_rows, dim3(8), dim3(1024), 0, S.stream, flags, enc, rows0, rows1, renc0, renc1, counts);
    HIP_TRY(hipGetLastError());
    uint32_t h[8];
    HIP_TRY(hipMemcpyAsync(h, counts, sizeof(h), hipMemcpyDeviceToHost, S.stream));
    HIP_TRY(hipStreamSynchronize(S.stream));
    for (int g = 0; g < 4; ++g) { d.counts[0][g] = h[g]; d.counts[1][g] = h[4 + g]; }
    d.built = true;
    return MMEE_OK;
}

}  // namespace
}  // namespace mmee

using namespace mmee;

extern "C" {

int mmee_chain_space_size(const mmee_chain *w, const mmee_hw *hw, uint64_t *out)
{
    if (!out) return MMEE_EINVAL;
    Plan p;
    int rc = make_plan(w, hw, p);
    if (rc) return rc;
    *out = p.space;
    return MMEE_OK;
}

int mmee_set_stream(void *hip_stream)
{
    std::lock_guard<std::mutex> guard(g_lock);
    if (S.ready) { HIP_TRY(hipStreamSynchronize(S.stream)); }
    S.stream = (hipStream_t)hip_stream;
    return MMEE_OK;
}

int mmee_offline_stats(mmee_row_stats *out)
{
    if (!out) return MMEE_EINVAL;
    std::lock_guard<std::mutex> guard(g_lock);
    int rc = ensure_ready();
    if (rc) return rc;
    for (int g = 0; g < 4; ++g) {
        out->rows_total[g] = ROWS_PER_GROUP;
        out->rows_valid[g] = S.counts[0][g];
        out->rows_kept[g] = S.counts[1][g];
    }
    return MMEE_OK;
}

int mmee_offline_rows(uint32_t group, uint32_t which, uint32_t *rows_out, uint32_t capacity, uint32_t *n_rows)
{
    if (group >= N_GROUPS || which > 1 || !n_rows || (capacity && !rows_out)) return MMEE_EINVAL;
    std::lock_guard<std::mutex> guard(g_lock);
    int rc = ensure_ready();
    if (rc) return rc;
    const uint32_t n = S.counts[which][group];
    *n_rows = n;
    const uint32_t take = std::min(n, capacity);
    if (take) {
        HIP_TRY(hipMemcpyAsync(rows_out, S.rows[which] + (size_t)group * ROWS_PER_GROUP, sizeof(uint32_t) * take,
                               hipMemcpyDeviceToHost, S.stream));
        HIP_TRY(hipStreamSynchronize(S.stream));
        for (uint32_t a = 0; a < take; ++a) rows_out[a] -= group * ROWS_PER_GROUP;   // number inside the group
    }
    return n > capacity ? MMEE_EOVERFLOW : MMEE_OK;
}

int mmee_chain_decode(const mmee_chain *w, const mmee_hw *hw, const uint64_t *idx, uint64_t n, mmee_mapping *out)
{
    if (n && (!idx || !out)) return MMEE_EINVAL;
    Plan p;
    int rc = make_plan(w, hw, p);
    if (rc) return rc;
    for (uint64_t a = 0; a < n; ++a)
        if (idx[a] >= p.space) return MMEE_ERANGE;
    if (!n) return MMEE_OK;
    std::lock_guard<std::mutex> guard(g_lock);
    rc = ensure_ready();
    if (rc) return rc;
    uint64_t *d_idx = nullptr;
    mmee_mapping *d_out = nullptr;
    HIP_TRY(hipMalloc(&d_idx, sizeof(uint64_t) * n));
    if (hipMalloc(&d_out, sizeof(mmee_mapping) * n) != hipSuccess) { (void)hipFree(d_idx); return MMEE_EDEVICE; }
    hipError_t e = hipMemcpyAsync(d_idx, idx, sizeof(uint64_t) * n, hipMemcpyHostToDevice, S.stream);
    if (e == hipSuccess) {
        hipLaunchKernelGGL(k_decode, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, S.stream, p.dv, p.mc.T, d_idx, n,
                           d_out);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(out, d_out, sizeof(mmee_mapping) * n, hipMemcpyDeviceToHost, S.stream);
    if (e == hipSuccess) e = hipStreamSynchronize(S.stream);
    (void)hipFree(d_idx); (void)hipFree(d_out);
    if (e != hipSuccess) {
        std::snprintf(g_last_error, sizeof(g_last_error), "mmee_decode: %s", hipGetErrorString(e));
        return MMEE_EDEVICE;
    }
    return MMEE_OK;
}

int mmee_chain_eval_batch(const mmee_chain *w, const mmee_hw *hw, uint64_t first_idx, uint64_t n,
                          mmee_cost *out_costs)
{
    Plan p;
    int rc = make_plan(w, hw, p);
    if (rc) return rc;
    if (first_idx > p.space || n > p.space - first_idx) return MMEE_ERANGE;
    if (!n) return MMEE_OK;
    if (!out_costs) return MMEE_EINVAL;
    std::lock_guard<std::mutex> guard(g_lock);
    rc = ensure_ready();
    if (rc) return rc;
    rc = ensure_tilings(p.mc.tpad);
    if (rc) return rc;
    Bufs tables;
    tables.btab = S.btab; tables.ctab_s = S.ctab_s; tables.ctab_e = S.ctab_e;
    rc = launch_tilings(p, p.mc, tables);
    if (rc) return rc;

    hipPointerAttribute_t attr;
    bool on_device = false;
    if (hipPointerGetAttributes(&attr, out_costs) == hipSuccess) on_device = attr.type == hipMemoryTypeDevice;
    else (void)hipGetLastError();

    EvalArgs ea;
    ea.enc = S.enc; ea.btab = S.btab; ea.ctab_e = S.ctab_e; ea.mc = p.mc;
    // records per launch: 1 GiB of staging for host output, one launch (grid limit) for device output;
    // whole 4 KiB pages of 64 records each
    const uint64_t CHUNK = on_device ? (1ull << 30) : (1ull << 24);
    if (!on_device) {
        size_t need = (size_t)std::min<uint64_t>(n, CHUNK) * sizeof(mmee_cost);
        if (need > S.eval_cap) {
            if (S.eval_dev) { HIP_TRY(hipStreamSynchronize(S.stream)); (void)hipFree(S.eval_dev); }
            S.eval_dev = nullptr; S.eval_cap = 0;
            HIP_TRY(hipMalloc(&S.eval_dev, need));
            S.eval_cap = need;
        }
    }
    for (uint64_t done = 0; done < n; done += CHUNK) {
        const uint64_t cnt = std::min<uint64_t>(CHUNK, n - done);
        const uint64_t n_pages = (cnt + 63) / 64;
        // blocks come in groups of eight that share 32 neighbouring pages
        const uint64_t nblocks = (n_pages + 31) / 32 * 8;
        if (nblocks > 0x7fffffffull) return MMEE_EINVAL;
        v4u *dst = on_device ? reinterpret_cast<v4u *>(out_costs + done) : reinterpret_cast<v4u *>(S.eval_dev);
        const uint64_t first = first_idx + done;
        hipLaunchKernelGGL(k_eval_batch, dim3((uint32_t)nblocks), dim3(256), 0, S.stream, ea, (uint32_t)(first / p.T),
                           (uint32_t)(first % p.T), (uint32_t)cnt, (uint32_t)n_pages, dst);
        HIP_TRY(hipGetLastError());
        if (!on_device) {
            HIP_TRY(hipMemcpyAsync(out_costs + done, S.eval_dev, cnt * sizeof(mmee_cost), hipMemcpyDeviceToHost,
                                   S.stream));
            HIP_TRY(hipStreamSynchronize(S.stream));
        }
    }
    HIP_TRY(hipStreamSynchronize(S.stream));
    return MMEE_OK;
}

int mmee_chain_search_many(const mmee_chain *w, const mmee_hw *hw, const int *objectives, uint32_t count,
                           uint32_t flags, mmee_result *out, int *rc_out)
{
    if (!count) return MMEE_OK;
    if (!w || !hw || !objectives || !out) return MMEE_EINVAL;
    if (flags & ~(uint32_t)(MMEE_SEARCH_EXHAUSTIVE | MMEE_SEARCH_ORDERED_SUM)) return MMEE_EINVAL;
    std::lock_guard<std::mutex> guard(g_lock);
    const double t_start = now_seconds();
    int rc = ensure_ready();
    if (rc) return rc;

    // group neighbouring entries that describe the same problem into one pass
    struct Pass {
        uint32_t first, n; int mask; Plan plan; int rc; uint64_t evaluated; bool unproven;
        bool batched = false; size_t ev_slot = 0;
    };
    std::vector<Pass> passes;
    std::vector<int> codes(count, MMEE_OK);
    for (uint32_t a = 0; a < count;) {
        Pass ps;
        ps.first = a; ps.n = 0; ps.mask = 0; ps.evaluated = 0; ps.unproven = false;
        ps.rc = make_plan(w + a, hw + a, ps.plan);
        uint32_t b = a;
        while (b < count && same_problem(w[a], hw[a], w[b], hw[b])) {
            int o = objectives[b];
            if (o < 0 || o >= N_OBJ) codes[b] = MMEE_EINVAL;     // this entry only; its neighbours still run
            else if (ps.mask & (1 << o)) break;      // same objective twice: start a new pass
            else ps.mask |= 1 << o;
            ++b; ++ps.n;
        }
        if (ps.n == 0) { ps.n = 1; b = a + 1; }
        if (ps.mask == 0 && !ps.rc) ps.rc = MMEE_EINVAL;         // no valid objective in the group
        passes.push_back(ps);
        a = b;
    }
    rc = ensure_slots(passes.size());
    if (rc) return rc;
    // Pruned searches whose key set the batched kernel is built for share launches; everything else
    // (the full row set, other key sets) goes problem by problem.  `round_flags` adds
    // MMEE_SEARCH_ORDERED_SUM on the second round, which repeats what the first could not prove.
    auto run_round = [&](uint32_t round_flags, bool only_unproven) -> int {
        std::vector<BatchEntry> batch;
        std::vector<size_t> batch_pass;
        for (size_t s = 0; s < passes.size(); ++s) {
            Pass &ps = passes[s];
            if (ps.rc != MMEE_OK || (only_unproven && !ps.unproven)) continue;
            ps.batched = S.batch_ok && !(round_flags & MMEE_SEARCH_EXHAUSTIVE) && batch_mask(ps.mask);
            if (ps.batched) {
                BatchEntry e;
                e.plan = &ps.plan; e.mask = ps.mask; e.slot = s; e.unproven = false; e.evaluated = 0;
                batch.push_back(e);
                batch_pass.push_back(s);
            } else {
                bool unproven = false;
                ps.rc = enqueue_search(ps.plan, ps.mask, round_flags, s, &ps.evaluated, nullptr, true, false,
                                       only_unproven ? nullptr : &unproven);
                ps.unproven = unproven;
            }
        }
        if (!batch.empty()) {
            int brc = enqueue_batches(batch, round_flags, batch_pass[0]);
            for (size_t k = 0; k < batch.size(); ++k) {
                Pass &ps = passes[batch_pass[k]];
                ps.rc = brc;
                ps.evaluated = batch[k].evaluated;
                ps.unproven = !only_unproven && batch[k].unproven;
                ps.ev_slot = batch_pass[0];
            }
        }
        HIP_TRY(hipStreamSynchronize(S.stream));
        return MMEE_OK;
    };
    rc = run_round(flags, false);
    if (rc) return rc;
    // a regrouped sum taken on trust (pass_constants) stands only if the energies found prove it
    {
        bool again = false;
        for (size_t s = 0; s < passes.size(); ++s) {
            Pass &ps = passes[s];
            if (ps.rc != MMEE_OK || !ps.unproven) continue;
            bool proven = true;
            for (int o : {MMEE_OBJ_ENERGY, MMEE_OBJ_LATENCY_THEN_ENERGY}) {
                if (!(ps.mask & (1 << o))) continue;
                const FinalRecord &fr = S.final_host[N_OBJ * s + o];
                double energy;
                std::memcpy(&energy, &fr.cost[5], sizeof(double));          // mmee_cost::energy_pj
                if (fr.key.p < INFINITY && !(energy < REGROUP_PROOF_LIMIT)) proven = false;
            }
            ps.unproven = !proven;
            again = again || !proven;
        }
        if (again) {
            rc = run_round(flags | MMEE_SEARCH_ORDERED_SUM, true);
            if (rc) return rc;
        }
    }
    const double seconds = now_seconds() - t_start;
    int first_bad = MMEE_OK;
    for (size_t s = 0; s < passes.size(); ++s) {
        Pass &ps = passes[s];
        float ms = 0.f;
        // a batched pass reports the device time of the launches it shared
        const size_t ev = ps.batched ? ps.ev_slot : s;
        if (ps.rc == MMEE_OK) (void)hipEventElapsedTime(&ms, S.events[2 * ev], S.events[2 * ev + 1]);
        for (uint32_t a = ps.first; a < ps.first + ps.n; ++a) {
            int code = codes[a] ? codes[a] : ps.rc;
            if (code == MMEE_OK)
                code = unpack_result(ps.plan, s, objectives[a], ps.evaluated, seconds, ms * 1e-3, out + a);
            else
                std::memset(out + a, 0, sizeof(mmee_result));
            if (rc_out) rc_out[a] = code;
            if (code && !first_bad) first_bad = code;
        }
    }
    return first_bad;
}

int mmee_chain_search_multi(const mmee_chain *w, const mmee_hw *hw, const int *objectives, uint32_t n_obj,
                            uint32_t flags, mmee_result *out)
{
    if (!w || !hw || !objectives || !out || n_obj < 1 || n_obj > N_OBJ) return MMEE_EINVAL;
    int seen = 0;
    for (uint32_t a = 0; a < n_obj; ++a) {
        if (objectives[a] < 0 || objectives[a] >= N_OBJ || (seen & (1 << objectives[a]))) return MMEE_EINVAL;
        seen |= 1 << objectives[a];
    }
    mmee_chain ws[N_OBJ] = {*w, *w, *w, *w};
    mmee_hw hs[N_OBJ] = {*hw, *hw, *hw, *hw};
    return mmee_chain_search_many(ws, hs, objectives, n_obj, flags, out, nullptr);
}

// Walk along a front.  Energy-latency (Sec. VII-E): by ascending latency, each step the
// latency-then-energy optimum among the candidates whose energy is strictly below the previous
// point's.  Buffer size / DRAM access (Sec. VII-C): by ascending buffer size, each step the
// (size, traffic)-smallest dataflow whose traffic is strictly below the previous point's.
static int walk_front(const mmee_chain *w, const mmee_hw *hw, bool bs_da, uint32_t flags, mmee_result *out,
               uint32_t capacity, uint32_t *n_points)
{
    if (!w || !hw || !out || !n_points || !capacity) return MMEE_EINVAL;
    if (flags & ~(uint32_t)(MMEE_SEARCH_EXHAUSTIVE | MMEE_SEARCH_ORDERED_SUM)) return MMEE_EINVAL;
    *n_points = 0;
    Plan p;
    int rc = make_plan(w, hw, p);
    if (rc) return rc;
    std::lock_guard<std::mutex> guard(g_lock);
    const double t_start = now_seconds();
    rc = ensure_ready();
    if (rc) return rc;
    rc = ensure_slots(1);
    if (rc) return rc;
    double limit = INFINITY, ksec = 0.0;
    uint64_t evaluated = 0;
    for (uint32_t k = 0;; ++k) {
        uint64_t ev = 0;
        bool unproven = false;
        rc = enqueue_search(p, bs_da ? 1 : 4, flags, 0, &ev, &limit, k == 0, bs_da, &unproven);
        if (rc) return rc;
        HIP_TRY(hipStreamSynchronize(S.stream));
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, S.events[0], S.events[1]);
        ksec += ms * 1e-3;
        evaluated += ev;
        mmee_result r;
        rc = unpack_result(p, 0, bs_da ? 0 : MMEE_OBJ_LATENCY_THEN_ENERGY, 0, 0.0, 0.0, &r);
        if (rc == MMEE_ENOFEASIBLE) break;          // nothing below the bound is left: the front is complete
        if (unproven && !(r.cost.energy_pj < REGROUP_PROOF_LIMIT)) {
            // the regrouped sum was taken on trust and this point does not prove it (energies fall
            // along the front, so only its first point can): start again, term by term
            flags |= MMEE_SEARCH_ORDERED_SUM;
            limit = INFINITY;
            *n_points = 0;
            k = (uint32_t)-1;
            continue;
        }
        if (k == capacity) return MMEE_EOVERFLOW;   // out holds the first `capacity` points
        out[k] = r;
        *n_points = k + 1;
        limit = bs_da ? p.mc.BH * (double)r.cost.da_words : r.cost.energy_pj;
    }
    const double seconds = now_seconds() - t_start;
    for (uint32_t k = 0; k < *n_points; ++k) {
        out[k].evaluated = evaluated; out[k].seconds = seconds; out[k].kernel_seconds = ksec;
    }
    return *n_points ? MMEE_OK : MMEE_ENOFEASIBLE;
}

int mmee_chain_pareto(const mmee_chain *w, const mmee_hw *hw, uint32_t flags, mmee_result *out, uint32_t capacity,
                      uint32_t *n_points)
{
    return walk_front(w, hw, false, flags, out, capacity, n_points);
}

int mmee_chain_front_bs_da(const mmee_chain *w, const mmee_hw *hw, uint32_t flags, mmee_result *out,
                           uint32_t capacity, uint32_t *n_points)
{
    return walk_front(w, hw, true, flags, out, capacity, n_points);
}

// ---- attention workloads: the chain I = L = N, K = J = d, batch = B*H --------------------------

int mmee_pareto(const mmee_workload *w, const mmee_hw *hw, uint32_t flags, mmee_result *out, uint32_t capacity,
                uint32_t *n_points)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_pareto(&c, hw, flags, out, capacity, n_points);
}

int mmee_front_bs_da(const mmee_workload *w, const mmee_hw *hw, uint32_t flags, mmee_result *out,
                     uint32_t capacity, uint32_t *n_points)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_front_bs_da(&c, hw, flags, out, capacity, n_points);
}

int mmee_chain_energy_regrouped(const mmee_chain *w, const mmee_hw *hw, uint32_t flags, int *out)
{
    if (!out || (flags & ~(uint32_t)(MMEE_SEARCH_EXHAUSTIVE | MMEE_SEARCH_ORDERED_SUM))) return MMEE_EINVAL;
    Plan p;
    int rc = make_plan(w, hw, p);
    if (rc) return rc;
    *out = (int)pass_constants(p, flags).regroup;
    return MMEE_OK;
}

int mmee_energy_regrouped(const mmee_workload *w, const mmee_hw *hw, uint32_t flags, int *out)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_energy_regrouped(&c, hw, flags, out);
}

int mmee_space_size(const mmee_workload *w, const mmee_hw *hw, uint64_t *out)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_space_size(&c, hw, out);
}

int mmee_decode(const mmee_workload *w, const mmee_hw *hw, const uint64_t *idx, uint64_t n, mmee_mapping *out)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_decode(&c, hw, idx, n, out);
}

int mmee_eval_batch(const mmee_workload *w, const mmee_hw *hw, uint64_t first_idx, uint64_t n, mmee_cost *out_costs)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_eval_batch(&c, hw, first_idx, n, out_costs);
}

int mmee_search_many(const mmee_workload *w, const mmee_hw *hw, const int *objectives, uint32_t count,
                     uint32_t flags, mmee_result *out, int *rc_out)
{
    if (!count) return MMEE_OK;
    if (!w || !hw || !objectives || !out) return MMEE_EINVAL;
    std::vector<mmee_chain> chains(count);
    for (uint32_t a = 0; a < count; ++a) {
        // a malformed workload becomes a malformed chain and is reported per entry
        if (chain_of(w + a, chains[a])) std::memset(&chains[a], 0, sizeof(mmee_chain));
    }
    return mmee_chain_search_many(chains.data(), hw, objectives, count, flags, out, rc_out);
}

int mmee_search_multi(const mmee_workload *w, const mmee_hw *hw, const int *objectives, uint32_t n_obj,
                      uint32_t flags, mmee_result *out)
{
    mmee_chain c;
    int rc = chain_of(w, c);
    return rc ? rc : mmee_chain_search_multi(&c, hw, objectives, n_obj, flags, out);
}

int mmee_search_ex(const mmee_workload *w, const mmee_hw *hw, int objective, uint32_t flags, mmee_result *out)
{
    return mmee_search_multi(w, hw, &objective, 1, flags, out);
}

int mmee_search(const mmee_workload *w, const mmee_hw *hw, int objective, mmee_result *out)
{
    return mmee_search_ex(w, hw, objective, MMEE_SEARCH_PRUNED, out);
}

int mmee_search_noalloc(const mmee_workload *w, const mmee_hw *hw, int objective, uint32_t flags,
                        mmee_result *out_dev)
{
    if (!out_dev || objective < 0 || objective >= N_OBJ) return MMEE_EINVAL;
    if (flags & ~(uint32_t)(MMEE_SEARCH_EXHAUSTIVE | MMEE_SEARCH_ORDERED_SUM)) return MMEE_EINVAL;
    mmee_chain c;
    int rc = chain_of(w, c);
    if (rc) return rc;
    Plan p;
    rc = make_plan(&c, hw, p);
    if (rc) return rc;
    if (p.mc.tpad > noalloc::MAX_TPAD) {
        std::snprintf(g_last_error, sizeof(g_last_error),
                      "mmee_search_noalloc: %llu tilings, the fixed scratch holds %u; use mmee_search_ex",
                      (unsigned long long)p.T, noalloc::MAX_TPAD);
        return MMEE_ETOOBIG;
    }
    std::lock_guard<std::mutex> guard(g_lock);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        std::snprintf(g_last_error, sizeof(g_last_error), "no HIP device");
        return MMEE_EDEVICE;
    }
    NoAllocDevice *d = nullptr;
    rc = noalloc_setup(dev, d);
    if (rc) return rc;
    unsigned char *q = d->ptr;
    Bufs b;
    b.enc = reinterpret_cast<const uint4 *>(q + noalloc::OFF_ENC);
    b.rows[0] = reinterpret_cast<const uint32_t *>(q + noalloc::OFF_ROWS0);
    b.rows[1] = reinterpret_cast<const uint32_t *>(q + noalloc::OFF_ROWS1);
    b.row_enc[0] = reinterpret_cast<const uint4 *>(q + noalloc::OFF_RENC0);
    b.row_enc[1] = reinterpret_cast<const uint4 *>(q + noalloc::OFF_RENC1);
    for (int k = 0; k < 2; ++k)
        for (int g = 0; g < 4; ++g) b.counts[k][g] = d->counts[k][g];
    b.cls_dev = nullptr;                       // row-per-lane kernel for every key
    b.btab = reinterpret_cast<double *>(q + noalloc::OFF_BTAB);
    b.ctab_s = reinterpret_cast<double *>(q + noalloc::OFF_CTAB_S);
    b.ctab_e = reinterpret_cast<uint64_t *>(q + noalloc::OFF_CTAB_E);
    b.partials = reinterpret_cast<Key *>(q + noalloc::OFF_PARTIALS);
    b.partials_cap = noalloc::MAX_BLOCKS;
    b.ticket = reinterpret_cast<uint32_t *>(q + noalloc::OFF_TICKET);
    b.key_dev = reinterpret_cast<Key *>(q + noalloc::OFF_KEYS);
    b.final_dev = reinterpret_cast<FinalRecord *>(q + noalloc::OFF_FINAL);
    b.dv_dev = reinterpret_cast<DivTable *>(q + noalloc::OFF_DV);
    b.resident_blocks = d->resident_blocks;
    // the finish ticket and the work counter must start at zero whatever the last call left
    hipLaunchKernelGGL(k_clear_words, dim3(1), dim3(64), 0, S.stream, b.ticket, 2u);
    uint64_t evaluated = 0;
    // the regrouped energy sum only where it is provably exact: nothing is read back to check it
    rc = enqueue_search_in(b, p, 1 << objective, flags, &evaluated);
    if (rc) return rc;
    hipLaunchKernelGGL(k_pack_result, dim3(1), dim3(64), 0, S.stream, b.final_dev + objective, p.space, evaluated,
                       out_dev);
    HIP_TRY(hipGetLastError());
    return MMEE_OK;
}

void mmee_shutdown(void)
{
    std::lock_guard<std::mutex> guard(g_lock);
    if (S.ready || S.btab || S.partials) (void)hipStreamSynchronize(S.stream);
    (void)hipFree(S.enc); (void)hipFree(S.sig); (void)hipFree(S.flags); (void)hipFree(S.cls_dev); (void)hipFree(S.key_dev);
    (void)hipFree(S.rows[0]); (void)hipFree(S.rows[1]); (void)hipFree(S.counts_dev);
    (void)hipFree(S.row_enc[0]); (void)hipFree(S.row_enc[1]);
    (void)hipFree(S.btab); (void)hipFree(S.ctab_s); (void)hipFree(S.ctab_e);
    (void)hipFree(S.partials); (void)hipFree(S.ticket); (void)hipFree(S.hints);
    (void)hipFree(S.dv_dev); (void)hipFree(S.eval_dev);
    if (S.final_host) (void)hipHostFree(S.final_host);
    if (S.batch_host) (void)hipHostFree(S.batch_host);
    (void)hipFree(S.batch_dev); (void)hipFree(S.item_keys);
    (void)hipFree(S.batch_row_off); (void)hipFree(S.batch_row_df); (void)hipFree(S.batch_cmap);
    for (hipEvent_t e : S.events) (void)hipEventDestroy(e);
    hipStream_t keep = S.stream;
    S = State();
    S.stream = keep;
}

const char *mmee_strerror(int code)
{
    switch (code) {
    case MMEE_OK: return "ok";
    case MMEE_EINVAL: return "invalid argument";
    case MMEE_ERANGE: return "candidate index out of range";
    case MMEE_ENOFEASIBLE: return "no feasible candidate";
    case MMEE_EDEVICE: return g_last_error[0] ? g_last_error : "HIP device error";
    case MMEE_EOVERFLOW: return "the Pareto front has more points than the caller made room for";
    case MMEE_ETOOBIG: return g_last_error[0] ? g_last_error : "the problem exceeds the fixed scratch of mmee_search_noalloc";
    default: return "unknown error";
    }
}

}  // extern "C"
