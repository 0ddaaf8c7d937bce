// Internal definitions shared by the HIP translation units of libmlmc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mlmc.h"

namespace mlmc {

constexpr int LMAX = MLMC_MAX_LEVELS;   // drawable levels 1..L
constexpr int TMAX = LMAX + 1;          // rank thresholds t = 0..L (one per ladder entry)
constexpr int SMAX = TMAX;              // distinct boundary buckets per row
constexpr int NB1 = 16384;              // first-digit buckets: 8 exponent bits + 6 mantissa bits of the key
constexpr int B1_SHIFT = 17;            // key >> 17 = first digit
constexpr int GMAX = 320;               // (exponent, band) sum groups per row: <= 255 + TMAX
constexpr int PMAX = 2 * TMAX;          // boundary-bucket pieces per row
constexpr int TILE = MLMC_TILE;
constexpr int ACC_SLOTS = 2048;         // LDS u64 accumulators of the band-sum pass
constexpr int MAX_PLANES = 25;          // 1 sign + at most 24 field planes

constexpr uint16_t CODE_IGNORE = 0x7FFF;
constexpr uint16_t CODE_CAND = 0x8000;

constexpr int THR_NONE = -1;      // k_t == 0: nothing is within the top k_t
constexpr int THR_ALL = -2;       // k_t >= d: everything is
constexpr int THR_INACTIVE = -3;  // not needed by this call

struct Piece {          // exact sum of squared significands of one part of a boundary bucket
    int32_t band_plus1; // 0 = unused
    int32_t exp;        // max(exponent field, 1)
    uint64_t lo, hi;    // value = hi * 2^32 + lo, in units of 2^(2 (exp - 150))
};

struct RowInfo {  // per row, rewritten by every call
    uint32_t thr_tau[TMAX];   // key at rank k_t - 1
    uint32_t thr_q[TMAX];     // how many entries equal to thr_tau are within the top k_t
    int32_t thr_slot[TMAX];   // boundary-bucket slot, or THR_*
    uint32_t thr_resid[TMAX]; // rank of the threshold inside its bucket (1-based)
    int32_t n_slots, n_groups, rep_shift, level;
    float weight;
    uint32_t draw_x;
    uint32_t slot_bucket[SMAX], slot_off[SMAX], slot_cnt[SMAX];
    uint16_t g_exp[GMAX], g_band[GMAX];
};

struct RowAcc {  // per row, zeroed at the start of every call
    uint32_t slot_fill[SMAX];
    uint32_t rowmax_key;
    uint64_t gsum[GMAX][2];
    Piece pieces[PMAX];
};

struct TopkArgs {
    const void* g;
    int64_t ld, d;
    int32_t M, L;
    int64_t k[TMAX];
    int32_t all_thresholds;  // 1: every ladder threshold + band sums (adaptive); 0: thresholds 0, l-1, l only
    int32_t chunk;           // elements per workgroup chunk (multiple of TILE)
    int64_t ntiles;
    uint32_t* hist1;         // [M][NB1]
    uint16_t* table;         // [M][NB1]
    RowInfo* rinfo;          // [M]
    RowAcc* racc;            // [M]
    uint32_t* cand;          // [M][d]
    unsigned long long* desc; // [M][units_per_row][4] look-back descriptors of the compaction (zeroed per call)
    uint32_t* ticket;        // [1] work counter of the compaction (zeroed per call)
    int64_t units_per_row;   // compaction units (cwaves * 1024 elements) per row
    int32_t cwaves;          // waves per compaction workgroup
    uint32_t* tile_off;      // [M][ntiles + 1]
    double* norms;           // [M][L]
    double* norms_user;      // optional copy
    int32_t* dev_status;
    // level draw (Alg. 2 / Alg. 3 "Sample l"): mode 0 p_fixed, 1 dev p, 2 dev norms, 3 norms computed by this call
    int32_t draw_mode;
    double p_fixed[LMAX];
    const double* p_dev;     // [M][L]
    uint64_t seed, step;
    // outputs of the compaction
    int32_t* level;
    int64_t* row_off;
    uint32_t* idx;
    float* val;
    int64_t capacity;
};

struct DrawArgs {
    int32_t M, L, mode;      // mode 0: p_fixed; 1: dev p; 2: dev norms
    double p_fixed[LMAX];
    const double* p_dev;     // [M][L]
    int64_t k[TMAX];         // Top-k: ladder; bits: unused
    int32_t is_topk;
    uint64_t seed, step;
    RowInfo* rinfo;
    int32_t* level;
    int64_t* row_off;
    int64_t capacity;
    int32_t* dev_status;
};

struct BitsArgs {
    const void* g;
    int64_t ld, d;
    int32_t M, L;
    int32_t F[TMAX];
    double p_fixed[LMAX];
    int32_t nplanes;         // planes per row in the message buffer
    int64_t nwords;          // ceil(d / 64)
    int32_t chunk;
    RowInfo* rinfo;
    RowAcc* racc;
    int32_t* level;
    int32_t* scale_exp;
    uint64_t* planes;
    int32_t* dev_status;
};

// ---- optional per-kernel timing with HIP events (host side, see mlmc_profile_* in mlmc.h) ----------
enum KernelId {
    K_ZERO = 0, K_HIST1, K_SCAN1, K_PASS2, K_FINISH, K_NORMS, K_DRAW, K_COMPACT,
    K_BITS_MAX, K_BITS_EXTRACT, K_AGG_BITS, K_TILEOFF, K_AGG_SPARSE, K_NUM
};
extern bool g_prof_on;
void prof_begin(int id, hipStream_t st);
void prof_end(int id, hipStream_t st);

// Launch statement wrapper: optional event pair around it, then the launch error check.
#define MLMC_LAUNCH(id, st, ...)                                \
    do {                                                        \
        if (::mlmc::g_prof_on) ::mlmc::prof_begin(id, st);      \
        __VA_ARGS__;                                            \
        if (::mlmc::g_prof_on) ::mlmc::prof_end(id, st);        \
        if (hipGetLastError() != hipSuccess) return MLMC_EHIP;  \
    } while (0)

}  // namespace mlmc

struct mlmc_plan_s {
    int kind, M, dtype, L;
    int64_t d;
    int64_t ladder[mlmc::TMAX];
    double p[mlmc::LMAX];
    bool adaptive;
    int64_t ntiles;
    int nplanes;
    int chunk;
    int chunks_per_row;
    // workspace byte offsets
    size_t off_racc, off_hist1, zero_bytes;  // [0, zero_bytes) is cleared per call
    size_t off_desc, off_ticket;
    int64_t units_per_row;
    int cwaves;
    size_t off_rinfo, off_table, off_tileoff, off_norms, off_cand;
    size_t ws_bytes;
};
