// Internal definitions shared by the HIP translation units of libmlmc (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mlmc.h"

namespace mlmc {

constexpr int LMAX = MLMC_MAX_LEVELS;   // drawable levels 1..L
constexpr int TMAX = LMAX + 1;          // rank thresholds t = 0..L (one per ladder entry)
constexpr int ZMAX = TMAX;              // zones (key ranges that may hold a threshold) per row
constexpr int RMAX = ZMAX + 1;          // regions per row: region i lies above zone i, region n_zones below the last zone
constexpr int NB1 = 16384;              // first-digit buckets: 8 exponent bits + 6 mantissa bits of the key
constexpr int B1_SHIFT = 17;            // key >> 17 = first digit
constexpr int GMAX = 292;               // sum groups per row: id = (255 - exponent) + region index <= 255 + ZMAX
constexpr int REP = 32;                 // lane-replicated LDS accumulators: slot = id * REP + (lane & 31)
constexpr int PMAX = 192;               // exact partial sums ("pieces") that the zones of one row contribute
constexpr int PIECE_CLASSES = 96;       // (parts of a zone) x (exponents of a zone) handled by one finish workgroup
constexpr int TILE = MLMC_TILE;
constexpr int MAX_PLANES = 25;          // fixed-point messages: 1 sign + at most 24 field planes
constexpr int MAX_FPLANES = 32;         // also the bound on the code planes of a Round-to-Nearest message
constexpr int RTN_LMAX = MLMC_MAX_RTN_LEVELS;         // floating-point messages: 1 sign + 8 exponent + at most 23 mantissa planes
constexpr int CHUNK_MAX = 1 << 18;      // elements per workgroup chunk of the streaming kernels
constexpr int CHUNKS_MAX = 8192;        // chunks per row
constexpr int FH_BINS = 2048;           // bins of the zone-relative key histogram of the finish kernels
constexpr int COLLECT_CAP = 2048;       // candidates of the thresholds' bins that are ranked in LDS
// The zone passes: FIN_WGS workgroups per row take (zone, slice) items in turn, a zone's candidate list being cut into up
// to FIN_SLICES slices of at least FIN_SLICE candidates.  These are the figures for 16 rows or more (512 workgroups in
// all); with fewer rows there are more workgroups per row, up to FIN_WGS_MAX, and as many more, smaller slices.
constexpr int FIN_SLICES = 16;
constexpr int FIN_SLICE = 32768;
constexpr int FIN_WGS = 32;
constexpr int FIN_WGS_MAX = 128;
// Slot of a part of a zone in the per-chunk table of zone entries: the part inside the top k_t but outside the
// top k of the zone's previous threshold has slot t; the part below every threshold of zone z has slot TMAX + z.
constexpr int ZPMAX = 2 * TMAX;

// Class table code of a first-digit bucket, laid out so that the selection read forms its LDS addresses with
// one or two instructions: bits 0..5 the tag an element is staged under (zone, or TAG_MEMBER); bits 6..12 the
// counter (region 0..63, or 64 + zone), i.e. already multiplied by the 64 bytes of a counter's replicas;
// bit 13 "stage this element" (zone candidate, or member of a band the message is expected to hold);
// bits 23..31 the sum group (after >> 16: multiplied by the 128 bytes of a group's replicas).  Zone buckets
// carry the group G_DUMMY, so the selection read needs no branch around its accumulators.
constexpr uint32_t CODE_STAGE = 0x2000;
constexpr uint32_t TAG_MEMBER = 63;
__host__ __device__ constexpr uint32_t class_code(uint32_t group, uint32_t counter, uint32_t tag, bool stage) {
    return (group << 23) | (counter << 6) | tag | (stage ? CODE_STAGE : 0u);
}
constexpr int G_DUMMY = GMAX - 1;
constexpr int REP_SUM = 16;             // replicas of the 64-bit group sum accumulators: slot = id * 16 + (lane & 15)
constexpr int REP_CNT = 16;             // replicas of the 32-bit region / zone counters
constexpr int CSUB_MAX = 4;             // count chunks per chunk of the selection read

constexpr int THR_NONE = -1;      // k_t == 0: nothing is within the top k_t
constexpr int THR_ALL = -2;       // k_t >= d: everything is
constexpr int THR_INACTIVE = -3;  // not needed by this call

constexpr uint32_t JX_ALL = 0x80000000u;  // every entry equal to the threshold key is inside (indices are < 2^31)

struct Piece {          // exact sum of squared significands of one part of a zone
    int32_t band_plus1; // 0 = unused
    int32_t exp;        // max(exponent field, 1)
    uint64_t lo, hi;    // value = hi * 2^32 + lo, in units of 2^(2 (exp - 150))
};

// What the kernels that write a row's message need, gathered once per row by k_msgplan.
struct MsgPlan {
    int64_t rowstart, rownnz;   // position of the row's message in idx / val, its length k_0 + k_l - k_{l-1}
    uint32_t tau[3], jx[3];     // thresholds 0, l-1, l
    float weight;
    int32_t level;
};

// Per row, rewritten by every call.  Membership of entry (key, j) in the top k_t of its row:
//     key > thr_tau[t]  ||  (key == thr_tau[t] && j < thr_jx[t])
struct RowInfo {
    uint32_t thr_tau[TMAX];   // key at rank k_t - 1
    uint32_t thr_jx[TMAX];    // entries equal to thr_tau with index below thr_jx are within the top k_t
    int32_t thr_zone[TMAX];   // zone that holds the threshold, or THR_*
    int32_t n_zones, level, respec, exact;
    int32_t spec_level;       // level whose band the selection read staged for the message (0: none)
    int32_t spec_ok;          // 1: the drawn level is spec_level, the message is assembled from the staged lists
    MsgPlan msg;
    float weight;
    uint32_t draw_x;
    uint32_t zone_top[ZMAX], zone_bot[ZMAX];   // first-digit buckets of the zone, top >= bot, both inclusive
    uint32_t zone_off[ZMAX], zone_cap[ZMAX];   // its candidate list inside the row's candidate buffer
    int32_t zone_t0[ZMAX], zone_t1[ZMAX];      // thresholds t0..t1 (those that are active) lie in the zone
    int32_t region_label[RMAX];                // band of every element of the region (label L + 1: in no band)
    uint16_t g_exp[GMAX], g_band[GMAX];        // sum group -> max(exponent, 1), band (0xFFFF unused)
};

struct RowAcc {  // per row, zeroed at the start of every call (and again before a row is redone exactly)
    uint32_t zone_fill[ZMAX];
    uint32_t zone_colcnt[ZMAX];   // finish kernels: candidates of the thresholds' bins gathered (or moved to the overflow list) so far
    uint32_t region_cnt[RMAX];
    uint32_t n_pieces;
    uint32_t rowmax_key;
    uint32_t smpmax_key;          // bit-wise path: largest key of the sampled blocks (the scale is predicted from it)
    uint32_t pad_;
    uint64_t gsum[GMAX][2];
    Piece pieces[PMAX];
};
constexpr int SMAX_PARTS_MAX = 1024;   // bit-wise path: per-workgroup maxima of a row, kept in the words of gsum (unused there)
static_assert(sizeof(uint64_t) * GMAX * 2 >= sizeof(uint32_t) * SMAX_PARTS_MAX, "the per-workgroup maxima fit in gsum");

struct TopkArgs {
    const void* g;
    int64_t ld, d;
    int32_t M, L;
    int32_t dtype;           // MLMC_F32 / MLMC_BF16 (the kernels that stream rows are compiled per type; this is for the few loads elsewhere)
    int64_t k[TMAX];
    int32_t all_thresholds;  // 1: every ladder threshold + band sums (adaptive); 0: thresholds 0, l-1, l only
    int32_t chunk;           // elements per workgroup chunk (multiple of TILE, <= CHUNK_MAX)
    int32_t chunks_per_row;
    int32_t cchunk;          // elements per count chunk: chunk / csub (multiple of TILE); message offsets are kept per count chunk
    int32_t csub;            // count chunks per chunk (1 or 4)
    int32_t cchunks_per_row;
    int32_t sample_shift;    // the first histogram reads one 1024-element block out of 2^sample_shift
    int32_t staging;         // 1: the selection read stages the members of the (predicted) drawn band
    int32_t fin_wgs, fin_slice, fin_slices;   // zone passes: workgroups per row, least candidates per slice, most slices per zone
    int64_t ntiles;
    uint32_t* hist;          // [M][NB1] histogram of the sampled blocks
    uint32_t* hist2;         // [M][NB1] full histogram of the rows that are redone exactly
    uint32_t* table;         // [M][NB1]
    uint8_t* table8;         // [M][NB1] the class table in one byte per bucket: counter | stage << 7
    RowInfo* rinfo;          // [M]
    RowAcc* racc;            // [M]
    uint2* cand;             // [M][d] candidate lists of the zones: {fp32 bit pattern, index}
    uint2* cand2;            // [M][d] overflow lists: candidates of threshold bins too full to rank in LDS
    uint2* cand_priv;        // [M][chunks_per_row][16 waves][chunk / 8] staged {bits, offset in chunk << 6 | tag} as the waves met them
    uint32_t* priv_cnt;      // [M][chunks_per_row][16] entries of every wave's private list
    uint32_t* chunk_base;    // [M][cchunks_per_row + 1] message entries of the row before every count chunk
    int32_t* row_order;      // [M] rows by descending message length: the order in which the message kernels take them
    uint32_t* chunk_cnt;     // [M][RMAX][cchunks_per_row] elements of every region per count chunk
    uint32_t* chunk_zcnt;    // [M][ZPMAX][cchunks_per_row] candidates of every part of every zone per count chunk (zeroed per call)
    uint32_t* zhist;         // [M][ZMAX][FH_BINS] zone-relative key histograms (zeroed per call)
    unsigned long long* zpacc; // [M][ZMAX][PIECE_CLASSES][2] sums of squared significands per (part, exponent) (zeroed per call)
    unsigned long long* zcol;  // [M][ZMAX][COLLECT_CAP] candidates of the thresholds' bins
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

struct BitsArgs {
    const void* g;
    int64_t ld, d;
    int32_t M, L;
    int32_t F[TMAX];
    double p_fixed[LMAX];
    int32_t flt;             // 1: floating-point ladder (App. B): F are mantissa digits, no scale
    int32_t vmx;             // 1: fixed-point ladder of |g| / max|g| (the scale field carries the bits of max|g|)
    int32_t rtn;             // 1: Round-to-Nearest ladder: F are bit widths, the scale field is [M][2]: bits of c, bits of the coefficient
    int32_t adaptive;        // RTN: 1 = probabilities from the row's residual norms (Lemma 3.4)
    int32_t smax_parts;      // > 0: k_bits_smax left the maxima of its workgroups (this many per row) in the row's gsum words instead of
                             // one atomic maximum in smpmax_key, which would have to be cleared by a launch before it
    unsigned long long* rtn_sums;   // RTN: [M][L][2] sums of squared residual integers, low and high 32-bit halves (zeroed per call)
    double* norms;           // RTN: [M][L]
    double* norms_user;      // RTN: optional copy
    int32_t nplanes;         // planes per row in the message buffer
    int64_t nwords;          // ceil(d / 64)
    int32_t chunk;
    int32_t sample_shift;    // the row maximum is first taken from one 1024-element block out of 2^sample_shift
    uint64_t seed, step;
    RowInfo* rinfo;
    RowAcc* racc;
    int32_t* level;
    int32_t* scale_exp;
    uint64_t* planes;
    int32_t* dev_status;
};

// s-segmented Top-k (uniform ladder k_l = min(s l, d), thousands of levels)
constexpr int SLMAX = MLMC_MAX_SLEVELS;
struct SRow {           // per row: the drawn segment
    int32_t level;
    float weight;
    int64_t lo, count;  // its positions in the sorted row: [lo, lo + count)
};
struct StopkArgs {
    const void* g;
    int64_t ld, d;
    int32_t M, L;
    int64_t s;
    int32_t nblk;            // sort blocks per row
    int64_t ntiles, bm_words;
    uint2* pa;               // [M][d] {inverted key, index} pairs, ping
    uint2* pb;               // pong
    uint32_t* counts;        // [M][256][nblk] digit counts / offsets of a sort pass
    uint32_t* bin_total;     // [M][256] elements of every digit bin
    uint32_t* bitmap;        // [M][bm_words] entries of the drawn segment
    uint32_t* tile_cnt;      // [M][ntiles] entries of the drawn segment per tile of 4096 indices (right behind the bitmaps: cleared with them)
    size_t clear_bytes;      // bitmaps + tile counts, a multiple of 16
    uint32_t* tile_off;      // [M][ntiles + 1]
    double* norms;           // [M][L]
    double* norms_user;
    SRow* srow;              // [M]
    int32_t* level;
    int64_t* row_off;
    uint32_t* idx;
    float* val;
    int64_t capacity;
    int32_t* dev_status;
    uint64_t seed, step;
};

// ---- optional per-kernel timing with HIP events (host side, see mlmc_profile_* in mlmc.h) ----------
enum KernelId {
    K_ZERO = 0, K_HIST, K_SCAN, K_MAIN, K_FHIST, K_FINISH, K_FINISH1, K_REDO, K_NORMS, K_DRAW, K_MSGPLAN, K_FILTER, K_WRITE,
    K_BITS_MAX, K_BITS_EXTRACT, K_BITS_REDO, K_AGG_BITS, K_TILEOFF, K_AGG_SPARSE, K_MSGBITS, K_RTN_NORMS, K_RTN_DRAW,
    K_RS_HIST, K_RS_SCAN, K_RS_SCATTER, K_SB_NORMS, K_SB_DRAW, K_SB_MARK, K_SB_OFFSETS, K_SB_WRITE, K_NUM
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
    int cchunk, csub, cchunks_per_row;
    int sample_shift;
    int staging;
    // workspace byte offsets
    size_t off_racc, off_hist, off_hist2, off_chunk_zcnt, off_zhist, off_zpacc, zero_bytes;  // [0, zero_bytes) is cleared per call
    size_t off_rinfo, off_table, off_chunk_cnt, off_zcol, off_tileoff, off_norms, off_cand, off_cand2, off_cand_priv, off_priv_cnt, off_chunk_base, off_row_order, off_table8;
    size_t ws_bytes;
    // s-segmented Top-k plans
    int64_t s;
    int nblk;
    int64_t bm_words;
    size_t off_pa, off_pb, off_counts, off_bitmap, off_tilecnt, off_clear_end, off_srow, off_bintot;
    size_t off_rtn_sums;   // Round-to-Nearest plans
    // Side stream of the message step (MLMC_TOPK): the second read of the rows whose band was not staged runs beside the
    // assembly of the other rows' messages from the staged lists.  Created at the first call that uses it, on the device
    // current then; default priority.  Host objects only; destroyed with the plan.
    mutable hipStream_t side_stream;
    mutable hipEvent_t side_fork, side_join;
    mutable int side_device;      // device the three objects belong to
    mutable int side_state;       // 0: not created yet, 1: ready, -1: could not be created (the step then runs on one stream)
    int side_enable;              // mlmc_plan_set_overlap
};
