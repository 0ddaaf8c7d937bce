// C ABI of libmlmc: plan construction / validation on the host and the entry points that enqueue the
// kernels (see include/mlmc.h for the contract of every call).
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "mlmc_internal.h"

namespace mlmc {
mlmc_status topk_zero(const mlmc_plan_t* pl, void* ws, int32_t* dev_status, hipStream_t st);
mlmc_status topk_select(const mlmc_plan_t* pl, const TopkArgs& a, bool sums, bool vec, hipStream_t st);
mlmc_status topk_compact(const mlmc_plan_t* pl, const TopkArgs& a, bool vec, hipStream_t st);
mlmc_status bits_compress(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, hipStream_t st);
mlmc_status rtn_compress(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, bool message, hipStream_t st);
mlmc_status agg_bits(const mlmc_plan_t* pl, const BitsArgs& b, const int32_t* level, const int32_t* scale_exp,
                     const uint64_t* planes, float alpha, float* out, float eta, float* x, hipStream_t st);
mlmc_status agg_sparse(const mlmc_plan_t* pl, const int64_t* row_off, const uint32_t* idx, const float* val, int64_t capacity,
                       const uint32_t* tile_off, uint32_t* tile_off_ws, float alpha, float* out, float eta, float* x,
                       hipStream_t st);
mlmc_status message_bits(const mlmc_plan_t* pl, const int32_t* level, unsigned long long* bits, hipStream_t st);
mlmc_status stopk_run(const mlmc_plan_t* pl, const StopkArgs& a, bool message, hipStream_t st);

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- static device scratch for mlmc_compress_bits_static --------------------------------------------
// Every GPU that loads the library holds its own copy of this array until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the device address is looked up once per device and
// kept; kernels, like those of mlmc_compress_bits, take the address as an argument.
static __device__ __align__(256) unsigned char scratch[MLMC_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

static mlmc_status static_scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return MLMC_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MLMC_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MLMC_OK;
}

// ---- per-kernel HIP-event timing (off by default; not thread safe) ---------------------------------
bool g_prof_on = false;
static const char* const k_names[K_NUM] = {
    "k_zero", "k_hist", "k_scan", "k_main", "k_fhist", "k_finish", "k_finish_rank", "redo_pass", "k_norms", "k_bits_prep", "k_msgplan", "k_filter", "k_write",
    "k_bits_smax", "k_bits_extract", "k_bits_redo", "k_agg_bits", "k_tileoff", "k_agg_sparse", "k_message_bits", "k_rtn_norms", "k_rtn_draw",
    "k_rs_hist", "k_rs_scan", "k_rs_scatter", "k_sb_norms", "k_sb_draw", "k_sb_mark", "k_sb_offsets", "k_sb_write"};
struct ProfPair { int id; hipEvent_t e0, e1; };
static std::vector<ProfPair> g_pending;
static std::vector<ProfPair> g_free;
static bool g_open = false;   // the last entry of g_pending still waits for its end event
static double g_total_ms[K_NUM];
static int64_t g_launches[K_NUM];

static void prof_drain() {
    for (ProfPair& p : g_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(p.e1) == hipSuccess && hipEventElapsedTime(&ms, p.e0, p.e1) == hipSuccess) {
            g_total_ms[p.id] += ms;
            g_launches[p.id] += 1;
        }
        g_free.push_back(p);
    }
    g_pending.clear();
}

void prof_begin(int id, hipStream_t st) {
    if (g_pending.size() >= 8192) prof_drain();
    ProfPair p;
    g_open = false;
    if (!g_free.empty()) {
        p = g_free.back();
        g_free.pop_back();
    } else {
        if (hipEventCreate(&p.e0) != hipSuccess) return;
        if (hipEventCreate(&p.e1) != hipSuccess) { (void)hipEventDestroy(p.e0); return; }
    }
    p.id = id;
    (void)hipEventRecord(p.e0, st);
    g_pending.push_back(p);
    g_open = true;
}

// Closes the pair that the matching prof_begin opened; when that call could not create its events there is no
// open pair and nothing is recorded (an older pair of the same kernel is never touched).
void prof_end(int id, hipStream_t st) {
    if (!g_open || g_pending.empty() || g_pending.back().id != id) return;
    (void)hipEventRecord(g_pending.back().e1, st);
    g_open = false;
}

// rows can be read with aligned 16-byte (fp32) / 8-byte (bf16) loads
static bool vec_ok(const mlmc_plan_t* pl, const void* g, int64_t ld) {
    if (pl->dtype == MLMC_F32) return ((uintptr_t)g % 16 == 0) && (ld % 4 == 0);
    return ((uintptr_t)g % 8 == 0) && (ld % 4 == 0);
}

static void fill_topk_args(const mlmc_plan_t* pl, TopkArgs& a, const void* g, int64_t ld, void* ws, int32_t* dev_status) {
    std::memset(&a, 0, sizeof(a));
    char* w = (char*)ws;
    a.g = g;
    a.ld = ld;
    a.d = pl->d;
    a.M = pl->M;
    a.L = pl->L;
    a.dtype = pl->dtype;
    for (int t = 0; t <= pl->L; ++t) a.k[t] = pl->ladder[t];
    a.chunk = pl->chunk;
    a.chunks_per_row = pl->chunks_per_row;
    a.cchunk = pl->cchunk;
    a.csub = pl->csub;
    a.cchunks_per_row = pl->cchunks_per_row;
    a.sample_shift = pl->sample_shift;
    a.staging = pl->staging;
    {
        int fx = FIN_WGS;
        if (pl->M < 16) fx = 512 / pl->M < FIN_WGS_MAX ? 512 / pl->M : FIN_WGS_MAX;   // about 512 workgroups in all
        fx = fx / FIN_WGS * FIN_WGS;                                                 // a multiple of FIN_WGS (32, 64, 96, 128)
        a.fin_wgs = fx;
        a.fin_slice = FIN_SLICE * FIN_WGS / fx;
        a.fin_slices = FIN_SLICES * fx / FIN_WGS;
    }
    a.ntiles = pl->ntiles;
    a.racc = (RowAcc*)(w + pl->off_racc);
    a.hist = (uint32_t*)(w + pl->off_hist);
    a.hist2 = (uint32_t*)(w + pl->off_hist2);
    a.rinfo = (RowInfo*)(w + pl->off_rinfo);
    a.table = (uint32_t*)(w + pl->off_table);
    a.table8 = (uint8_t*)(w + pl->off_table8);
    a.chunk_cnt = (uint32_t*)(w + pl->off_chunk_cnt);
    a.chunk_zcnt = (uint32_t*)(w + pl->off_chunk_zcnt);
    a.zhist = (uint32_t*)(w + pl->off_zhist);
    a.zpacc = (unsigned long long*)(w + pl->off_zpacc);
    a.zcol = (unsigned long long*)(w + pl->off_zcol);
    a.tile_off = (uint32_t*)(w + pl->off_tileoff);
    a.norms = (double*)(w + pl->off_norms);
    a.cand = (uint2*)(w + pl->off_cand);
    a.cand2 = (uint2*)(w + pl->off_cand2);
    a.cand_priv = (uint2*)(w + pl->off_cand_priv);
    a.priv_cnt = (uint32_t*)(w + pl->off_priv_cnt);
    a.chunk_base = (uint32_t*)(w + pl->off_chunk_base);
    a.row_order = (int32_t*)(w + pl->off_row_order);
    a.dev_status = dev_status;
}

static void fill_bits_args(const mlmc_plan_t* pl, BitsArgs& b, const void* g, int64_t ld, void* ws, int32_t* dev_status) {
    std::memset(&b, 0, sizeof(b));
    char* w = (char*)ws;
    b.g = g;
    b.ld = ld;
    b.d = pl->d;
    b.M = pl->M;
    b.L = pl->L;
    for (int t = 0; t <= pl->L; ++t) b.F[t] = (int32_t)pl->ladder[t];
    for (int l = 0; l < pl->L; ++l) b.p_fixed[l] = pl->p[l];
    b.flt = pl->kind == MLMC_FBITS ? 1 : 0;
    b.vmx = pl->kind == MLMC_VBITS ? 1 : 0;
    b.rtn = pl->kind == MLMC_RTN ? 1 : 0;
    b.adaptive = pl->adaptive ? 1 : 0;
    if (pl->kind == MLMC_RTN && ws) {
        b.rtn_sums = (unsigned long long*)(w + pl->off_rtn_sums);
        b.norms = (double*)(w + pl->off_norms);
    }
    b.nplanes = pl->nplanes;
    b.nwords = (pl->d + 63) / 64;
    b.chunk = pl->chunk;
    b.sample_shift = pl->sample_shift;
    b.rinfo = ws ? (RowInfo*)(w + pl->off_rinfo) : nullptr;
    b.racc = ws ? (RowAcc*)(w + pl->off_racc) : nullptr;
    b.dev_status = dev_status;
}
}  // namespace mlmc

using namespace mlmc;

extern "C" {

const char* mlmc_status_string(int status) {
    switch (status) {
        case MLMC_OK: return "MLMC_OK";
        case MLMC_EINVAL: return "MLMC_EINVAL: invalid argument";
        case MLMC_ENOMEM: return "MLMC_ENOMEM: host allocation failed";
        case MLMC_EHIP: return "MLMC_EHIP: HIP launch failed";
        case MLMC_ELIMIT: return "MLMC_ELIMIT: the plan needs more scratch than the static array holds";
        default: return "unknown mlmc status";
    }
}

void mlmc_profile_enable(int on) {
    if (!on) prof_drain();
    g_prof_on = on != 0;
}

void mlmc_profile_reset(void) {
    prof_drain();
    for (int i = 0; i < K_NUM; ++i) { g_total_ms[i] = 0.0; g_launches[i] = 0; }
}

int mlmc_profile_num_kernels(void) { return K_NUM; }

const char* mlmc_profile_kernel_name(int id) { return id >= 0 && id < K_NUM ? k_names[id] : ""; }

mlmc_status mlmc_profile_get(int id, double* total_ms, int64_t* launches) {
    if (id < 0 || id >= K_NUM || !total_ms || !launches) return MLMC_EINVAL;
    prof_drain();
    *total_ms = g_total_ms[id];
    *launches = g_launches[id];
    return MLMC_OK;
}

mlmc_status mlmc_geometric_p(int L, double* p) {
    if (L < 1 || L > 1000 || !p) return MLMC_EINVAL;
    const double norm = 1.0 - std::ldexp(1.0, -L);
    for (int l = 1; l <= L; ++l) p[l - 1] = std::ldexp(1.0, -l) / norm;
    return MLMC_OK;
}

// s-segmented Top-k (Sec. 2.2, Sec. 3.2): uniform ladder k_l = min(s l, d), L = ceil(d / s) levels, adaptive p only.
static mlmc_status plan_stopk(mlmc_plan_t** plan, int M, int64_t d, int in_dtype, int L, int64_t s, const double* p_fixed,
                              size_t* workspace_bytes, int64_t* sparse_capacity_worst) {
    if (in_dtype != MLMC_F32 && in_dtype != MLMC_BF16) return MLMC_EINVAL;
    if (M < 1 || M > MLMC_MAX_WORKERS || d < 1 || d >= ((int64_t)1 << 31) || s < 1 || p_fixed) return MLMC_EINVAL;
    const int64_t Lw = (d + s - 1) / s;
    if (Lw > MLMC_MAX_SLEVELS || (int64_t)L != Lw) return MLMC_EINVAL;
    mlmc_plan_t* pl = new (std::nothrow) mlmc_plan_t;
    if (!pl) return MLMC_ENOMEM;
    std::memset(pl, 0, sizeof(*pl));
    pl->kind = MLMC_STOPK;
    pl->M = M;
    pl->dtype = in_dtype;
    pl->L = L;
    pl->d = d;
    pl->s = s;
    pl->adaptive = true;
    pl->ntiles = (d + TILE - 1) / TILE;
    pl->nblk = (int)((d + 4096 - 1) / 4096);   // sort blocks: RS_TILE elements
    pl->bm_words = ((d + 31) / 32 + 3) / 4 * 4;   // whole 16-byte groups per row
    size_t off = 0;
    pl->off_bitmap = off;
    off = align_up(off + sizeof(uint32_t) * (size_t)pl->bm_words * M + 16, 256);
    pl->off_tilecnt = off;
    off = align_up(off + sizeof(uint32_t) * (size_t)pl->ntiles * M, 256);
    pl->off_clear_end = off;
    pl->off_srow = off;
    off = align_up(off + sizeof(SRow) * (size_t)M, 256);
    pl->off_counts = off;
    off = align_up(off + sizeof(uint32_t) * 256 * (size_t)pl->nblk * M, 256);
    pl->off_bintot = off;
    off = align_up(off + sizeof(uint32_t) * 256 * (size_t)M, 256);
    pl->off_tileoff = off;
    off = align_up(off + sizeof(uint32_t) * (size_t)(pl->ntiles + 1) * M, 256);
    pl->off_norms = off;
    off = align_up(off + sizeof(double) * (size_t)L * M, 256);
    pl->off_pa = off;
    off = align_up(off + sizeof(uint2) * (size_t)d * M, 256);
    pl->off_pb = off;
    off = align_up(off + sizeof(uint2) * (size_t)d * M, 256);
    pl->ws_bytes = off;
    if (workspace_bytes) *workspace_bytes = off;
    if (sparse_capacity_worst) *sparse_capacity_worst = (int64_t)M * (s < d ? s : d);
    *plan = pl;
    return MLMC_OK;
}

static void fill_stopk_args(const mlmc_plan_t* pl, StopkArgs& a, const void* g, int64_t ld, void* ws, int32_t* dev_status) {
    std::memset(&a, 0, sizeof(a));
    char* w = (char*)ws;
    a.g = g;
    a.ld = ld;
    a.d = pl->d;
    a.M = pl->M;
    a.L = pl->L;
    a.s = pl->s;
    a.nblk = pl->nblk;
    a.ntiles = pl->ntiles;
    a.bm_words = pl->bm_words;
    a.pa = (uint2*)(w + pl->off_pa);
    a.pb = (uint2*)(w + pl->off_pb);
    a.counts = (uint32_t*)(w + pl->off_counts);
    a.bin_total = (uint32_t*)(w + pl->off_bintot);
    a.bitmap = (uint32_t*)(w + pl->off_bitmap);
    a.tile_cnt = (uint32_t*)(w + pl->off_tilecnt);
    a.clear_bytes = pl->off_clear_end - pl->off_bitmap;
    a.tile_off = (uint32_t*)(w + pl->off_tileoff);
    a.norms = (double*)(w + pl->off_norms);
    a.srow = (SRow*)(w + pl->off_srow);
    a.dev_status = dev_status;
}

mlmc_status mlmc_plan(mlmc_plan_t** plan, int kind, int M, int64_t d, int in_dtype, int L, const int64_t* ladder,
                      const double* p_fixed, size_t* workspace_bytes, int64_t* sparse_capacity_worst) {
    if (plan) *plan = nullptr;
    if (!plan || !ladder) return MLMC_EINVAL;
    if (kind == MLMC_STOPK) return plan_stopk(plan, M, d, in_dtype, L, ladder[0], p_fixed, workspace_bytes, sparse_capacity_worst);
    if (kind != MLMC_TOPK && kind != MLMC_BITS && kind != MLMC_FBITS && kind != MLMC_VBITS && kind != MLMC_RTN) return MLMC_EINVAL;
    if (in_dtype != MLMC_F32 && in_dtype != MLMC_BF16) return MLMC_EINVAL;
    if (M < 1 || M > MLMC_MAX_WORKERS || d < 1 || d >= ((int64_t)1 << 31) || L < 1 || L > MLMC_MAX_LEVELS) return MLMC_EINVAL;
    if (ladder[0] < 0) return MLMC_EINVAL;
    for (int t = 0; t < L; ++t)
        if (ladder[t] >= ladder[t + 1]) return MLMC_EINVAL;
    if (kind == MLMC_TOPK && ladder[L] > d) return MLMC_EINVAL;
    if ((kind == MLMC_BITS || kind == MLMC_VBITS) && ladder[L] > 24) return MLMC_EINVAL;
    if (kind == MLMC_FBITS && ladder[L] > 23) return MLMC_EINVAL;
    if (kind == MLMC_RTN && (ladder[L] > 16 || L > MLMC_MAX_RTN_LEVELS)) return MLMC_EINVAL;
    if (kind != MLMC_TOPK && kind != MLMC_RTN && !p_fixed) return MLMC_EINVAL;  // Lemma 3.4 probabilities: rank bands and the Round-to-Nearest ladder
    if (p_fixed) {
        double s = 0.0;
        for (int l = 0; l < L; ++l) {
            if (!(p_fixed[l] > 0.0) || !(p_fixed[l] <= 1.0)) return MLMC_EINVAL;
            s += p_fixed[l];
        }
        if (std::fabs(s - 1.0) > 1e-9) return MLMC_EINVAL;
    }
    mlmc_plan_t* pl = new (std::nothrow) mlmc_plan_t;
    if (!pl) return MLMC_ENOMEM;
    std::memset(pl, 0, sizeof(*pl));
    pl->kind = kind;
    pl->M = M;
    pl->dtype = in_dtype;
    pl->L = L;
    pl->d = d;
    for (int t = 0; t <= L; ++t) pl->ladder[t] = ladder[t];
    pl->adaptive = p_fixed == nullptr;
    if (p_fixed)
        for (int l = 0; l < L; ++l) pl->p[l] = p_fixed[l];
    pl->ntiles = (d + TILE - 1) / TILE;
    pl->nplanes = 0;
    if (kind != MLMC_TOPK) {
        int maxw = 0;
        for (int l = 1; l <= L; ++l) {
            int w = (int)(ladder[l] - ladder[l - 1]);
            if (w > maxw) maxw = w;
        }
        pl->nplanes = (kind == MLMC_FBITS ? 9 : 1) + (int)ladder[0] + maxw;
        if (kind == MLMC_RTN) {   // the codes of the base, the previous and the drawn level
            int most = 0;
            for (int l = 1; l <= L; ++l) {
                const int n = (int)ladder[0] + (l > 1 ? (int)ladder[l - 1] : 0) + (int)ladder[l];
                if (n > most) most = n;
            }
            if (most > MAX_FPLANES) { delete pl; return MLMC_EINVAL; }
            pl->nplanes = most;
        }
    }
    // chunking of the streaming kernels: about 2048 workgroups over all rows, but chunks of at least some 96 K
    // elements (a workgroup of the selection read loads a 64 KB table first), whole tiles, at most 2^18 elements
    // per workgroup (the LDS accumulators and the packed candidate offsets rely on that bound)
    int64_t target_per_row = 2048 / M > 0 ? 2048 / M : 1;
    int64_t by_size = (d + 98303) / 98304;
    if (by_size < 4) by_size = 4;   // a short row still spreads over a few CUs
    if (target_per_row > by_size) target_per_row = by_size;
    int64_t chunk = (d + target_per_row - 1) / target_per_row;
    chunk = (chunk + 4 * TILE - 1) / (4 * TILE) * (4 * TILE);
    if (chunk < 4 * TILE) chunk = 4 * TILE;
    if (chunk > CHUNK_MAX) chunk = CHUNK_MAX;
    // A workgroup of the selection read holds a whole CU, so its M * chunks workgroups run in rounds of one per
    // CU: among the chunk sizes within a quarter of the one above, take the one whose last round is the fullest
    // (rounds x chunk = the elements a CU streams through).
    {
        constexpr int64_t NUM_CUS = 256;   // MI355X
        int64_t best = chunk, best_cost = -1;
        for (int64_t c = chunk - chunk / 4; c <= chunk + chunk / 4; c += 4 * TILE) {
            const int64_t cc = (c + 4 * TILE - 1) / (4 * TILE) * (4 * TILE);
            if (cc < 4 * TILE || cc > CHUNK_MAX) continue;
            const int64_t n = (d + cc - 1) / cc;
            if (n > CHUNKS_MAX / CSUB_MAX) continue;
            const int64_t rounds = ((int64_t)M * n + NUM_CUS - 1) / NUM_CUS;
            const int64_t cost = rounds * (cc + 16384);   // + a workgroup's fixed part (table load, flush), in elements
            if (best_cost < 0 || cost < best_cost || (cost == best_cost && cc == chunk)) { best = cc; best_cost = cost; }
        }
        chunk = best;
    }
    pl->chunk = (int)chunk;
    pl->chunks_per_row = (int)((d + chunk - 1) / chunk);   // <= 2^31 / 2^18 = CHUNKS_MAX
    // message offsets are kept per count chunk, a quarter of a chunk (unless that would be too many per row):
    // the second read of a row, when one is needed, then has four times as many workgroups
    pl->csub = (pl->chunks_per_row * CSUB_MAX <= CHUNKS_MAX && chunk >= 16 * TILE) ? CSUB_MAX : 1;
    pl->cchunk = (int)(chunk / pl->csub);
    pl->cchunks_per_row = (int)((d + pl->cchunk - 1) / pl->cchunk);
    // rows long enough that a second full read matters get their thresholds from a sampled histogram
    pl->sample_shift = d >= ((int64_t)1 << 23) ? 4 : d >= ((int64_t)1 << 21) ? 2 : 0;
    if (kind == MLMC_VBITS || kind == MLMC_RTN) pl->sample_shift = 0;   // the largest entry itself is needed, not its binade
    pl->staging = 1;
    // The fork and the join cost some twenty microseconds of stream operations, paid in every call, while the second read
    // has work in a call only when some row's band was not staged: worth it for many long rows (measured: -11 us per call
    // at 16 rows of 2.6e7 elements, +5 us at 4 rows of 1.2e8).
    pl->side_enable = M >= 8 && (int64_t)M * d >= ((int64_t)1 << 28) ? 1 : 0;

    size_t off = 0;
    pl->off_racc = off;
    off = align_up(off + sizeof(RowAcc) * (size_t)M, 256);
    if (kind == MLMC_TOPK) {
        pl->off_hist = off;
        off = align_up(off + sizeof(uint32_t) * NB1 * (size_t)M, 256);
        pl->off_hist2 = off;
        off = align_up(off + sizeof(uint32_t) * NB1 * (size_t)M, 256);
        pl->off_chunk_zcnt = off;
        off = align_up(off + sizeof(uint32_t) * ZPMAX * (size_t)pl->cchunks_per_row * M, 256);
        pl->off_zhist = off;
        off = align_up(off + sizeof(uint32_t) * FH_BINS * ZMAX * (size_t)M, 256);
        pl->off_zpacc = off;
        off = align_up(off + sizeof(unsigned long long) * 2 * PIECE_CLASSES * ZMAX * (size_t)M, 256);
    }
    pl->zero_bytes = off;
    pl->off_rinfo = off;
    off = align_up(off + sizeof(RowInfo) * (size_t)M, 256);
    if (kind == MLMC_RTN) {
        pl->off_rtn_sums = off;
        off = align_up(off + sizeof(unsigned long long) * 2 * (size_t)L * M, 256);
        pl->off_norms = off;
        off = align_up(off + sizeof(double) * (size_t)L * M, 256);
    }
    if (kind == MLMC_TOPK) {
        pl->off_table = off;
        off = align_up(off + sizeof(uint32_t) * NB1 * (size_t)M, 256);
        pl->off_chunk_cnt = off;
        off = align_up(off + sizeof(uint32_t) * RMAX * (size_t)pl->cchunks_per_row * M, 256);
        pl->off_zcol = off;
        off = align_up(off + sizeof(unsigned long long) * COLLECT_CAP * ZMAX * (size_t)M, 256);
        pl->off_tileoff = off;
        off = align_up(off + sizeof(uint32_t) * (size_t)(pl->ntiles + 1) * M, 256);
        pl->off_norms = off;
        off = align_up(off + sizeof(double) * (size_t)L * M, 256);
        pl->off_cand = off;
        off = align_up(off + sizeof(uint2) * (size_t)d * M, 256);
        pl->off_cand2 = off;
        off = align_up(off + sizeof(uint2) * (size_t)d * M, 256);
        pl->off_cand_priv = off;
        off = align_up(off + sizeof(uint2) * 2 * (size_t)pl->chunk * pl->chunks_per_row * M, 256);   // room for twice a wave's even share
        pl->off_priv_cnt = off;
        off = align_up(off + sizeof(uint32_t) * 16 * (size_t)pl->chunks_per_row * M, 256);
        pl->off_chunk_base = off;
        off = align_up(off + sizeof(uint32_t) * (size_t)(pl->cchunks_per_row + 1) * M, 256);
        pl->off_row_order = off;
        off = align_up(off + sizeof(int32_t) * (size_t)M, 256);
        pl->off_table8 = off;
        off = align_up(off + (size_t)NB1 * M, 256);
    }
    pl->ws_bytes = off;
    if (workspace_bytes) *workspace_bytes = off;
    if (sparse_capacity_worst) {
        int64_t cap = 0;
        if (kind == MLMC_TOPK) {
            int64_t widest = 0;
            for (int l = 1; l <= L; ++l)
                if (ladder[l] - ladder[l - 1] > widest) widest = ladder[l] - ladder[l - 1];
            cap = (int64_t)M * (ladder[0] + widest);
        }
        *sparse_capacity_worst = cap;
    }
    *plan = pl;
    return MLMC_OK;
}

void mlmc_plan_destroy(mlmc_plan_t* plan) {
    if (!plan) return;
    // the side stream of the message step: its work was joined to the caller's stream, nothing is pending on it alone
    if (plan->side_stream) { (void)hipStreamSynchronize(plan->side_stream); (void)hipStreamDestroy(plan->side_stream); }
    if (plan->side_fork) (void)hipEventDestroy(plan->side_fork);
    if (plan->side_join) (void)hipEventDestroy(plan->side_join);
    delete plan;
}

mlmc_status mlmc_plan_set_overlap(mlmc_plan_t* plan, int enable) {
    if (!plan || plan->kind != MLMC_TOPK) return MLMC_EINVAL;
    plan->side_enable = enable ? 1 : 0;
    return MLMC_OK;
}

mlmc_status mlmc_plan_set_sampling(mlmc_plan_t* plan, int shift) {
    if (!plan || shift < 0 || shift > 12 || plan->kind == MLMC_VBITS || plan->kind == MLMC_RTN) return MLMC_EINVAL;
    plan->sample_shift = shift;
    return MLMC_OK;
}

mlmc_status mlmc_plan_set_staging(mlmc_plan_t* plan, int enable) {
    if (!plan || plan->kind != MLMC_TOPK) return MLMC_EINVAL;
    plan->staging = enable ? 1 : 0;
    return MLMC_OK;
}

int64_t mlmc_plan_num_tiles(const mlmc_plan_t* plan) { return plan ? plan->ntiles : 0; }
int64_t mlmc_plan_chunk(const mlmc_plan_t* plan) { return plan && plan->kind == MLMC_TOPK ? plan->chunk : 0; }
int mlmc_plan_num_planes(const mlmc_plan_t* plan) { return plan ? plan->nplanes : 0; }

mlmc_status mlmc_level_norms(const mlmc_plan_t* plan, const void* g, int64_t ld, double* norms, int32_t* dev_status,
                             void* ws, void* hip_stream) {
    if (!plan || (plan->kind != MLMC_TOPK && plan->kind != MLMC_STOPK && plan->kind != MLMC_RTN) || !g || !norms || !dev_status || !ws || ld < plan->d) return MLMC_EINVAL;
    if ((uintptr_t)ws % 256) return MLMC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (plan->kind == MLMC_RTN) {
        BitsArgs b;
        fill_bits_args(plan, b, g, ld, ws, dev_status);
        b.norms_user = norms;
        return rtn_compress(plan, b, vec_ok(plan, g, ld), false, st);
    }
    if (plan->kind == MLMC_STOPK) {
        StopkArgs sa;
        fill_stopk_args(plan, sa, g, ld, ws, dev_status);
        sa.norms_user = norms;
        return stopk_run(plan, sa, false, st);
    }
    TopkArgs a;
    fill_topk_args(plan, a, g, ld, ws, dev_status);
    a.all_thresholds = 1;
    a.draw_mode = -1;  // norms only, no draw
    a.norms_user = norms;
    mlmc_status rc = topk_zero(plan, ws, dev_status, st);
    if (rc != MLMC_OK) return rc;
    return topk_select(plan, a, true, vec_ok(plan, g, ld), st);
}

mlmc_status mlmc_compress_topk(const mlmc_plan_t* plan, const void* g, int64_t ld, const double* p, int p_is_norms,
                               uint64_t seed, uint64_t step, int32_t* level, int64_t* row_off, uint32_t* idx, float* val,
                               int64_t capacity, uint32_t* tile_off, double* norms_out, int32_t* dev_status, void* ws,
                               void* hip_stream) {
    if (!plan || (plan->kind != MLMC_TOPK && plan->kind != MLMC_STOPK) || !g || !level || !row_off || !idx || !val || !dev_status || !ws) return MLMC_EINVAL;
    if (ld < plan->d || capacity < 0 || (uintptr_t)ws % 256) return MLMC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (plan->kind == MLMC_STOPK) {
        if (p || p_is_norms) return MLMC_EINVAL;   // Lemma 3.4 probabilities from the row itself, nothing else
        StopkArgs sa;
        fill_stopk_args(plan, sa, g, ld, ws, dev_status);
        sa.level = level;
        sa.row_off = row_off;
        sa.idx = idx;
        sa.val = val;
        sa.capacity = capacity;
        if (tile_off) sa.tile_off = tile_off;
        sa.norms_user = norms_out;
        sa.seed = seed;
        sa.step = step;
        return stopk_run(plan, sa, true, st);
    }
    const bool vec = vec_ok(plan, g, ld);
    const bool internal_norms = plan->adaptive && p == nullptr;
    TopkArgs a;
    fill_topk_args(plan, a, g, ld, ws, dev_status);
    a.level = level;
    a.row_off = row_off;
    a.idx = idx;
    a.val = val;
    a.capacity = capacity;
    if (tile_off) a.tile_off = tile_off;
    a.norms_user = internal_norms ? norms_out : nullptr;
    a.all_thresholds = internal_norms ? 1 : 0;

    a.seed = seed;
    a.step = step;
    if (p) {
        a.draw_mode = p_is_norms ? 2 : 1;
        a.p_dev = p;
    } else if (!plan->adaptive) {
        a.draw_mode = 0;
        for (int l = 0; l < plan->L; ++l) a.p_fixed[l] = plan->p[l];
    } else {
        a.draw_mode = 3;
    }
    mlmc_status rc = topk_zero(plan, ws, dev_status, st);
    if (rc != MLMC_OK) return rc;
    // draw_mode < 3: the level is drawn before the data is touched (inside the threshold scan), so only
    // three thresholds are resolved; draw_mode 3: all thresholds and band sums first, then the draw
    rc = topk_select(plan, a, internal_norms, vec, st);
    if (rc != MLMC_OK) return rc;
    return topk_compact(plan, a, vec, st);
}

mlmc_status mlmc_compress_bits(const mlmc_plan_t* plan, const void* g, int64_t ld, uint64_t seed, uint64_t step,
                               int32_t* level, int32_t* scale_exp, uint64_t* planes, int32_t* dev_status, void* ws,
                               void* hip_stream) {
    if (!plan || (plan->kind != MLMC_BITS && plan->kind != MLMC_FBITS && plan->kind != MLMC_VBITS) || !g || !level || !planes || !dev_status || !ws) return MLMC_EINVAL;
    if (plan->kind != MLMC_FBITS && !scale_exp) return MLMC_EINVAL;
    if (ld < plan->d || (uintptr_t)ws % 256) return MLMC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    BitsArgs b;
    fill_bits_args(plan, b, g, ld, ws, dev_status);
    b.level = level;
    b.scale_exp = scale_exp;
    b.planes = planes;
    b.seed = seed;
    b.step = step;
    return bits_compress(plan, b, vec_ok(plan, g, ld), st);
}

mlmc_status mlmc_compress_rtn(const mlmc_plan_t* plan, const void* g, int64_t ld, uint64_t seed, uint64_t step, int32_t* level,
                              int32_t* scale, uint64_t* planes, double* norms_out, int32_t* dev_status, void* ws, void* hip_stream) {
    if (!plan || plan->kind != MLMC_RTN || !g || !level || !scale || !planes || !dev_status || !ws) return MLMC_EINVAL;
    if (ld < plan->d || (uintptr_t)ws % 256) return MLMC_EINVAL;
    BitsArgs b;
    fill_bits_args(plan, b, g, ld, ws, dev_status);
    b.level = level;
    b.scale_exp = scale;
    b.planes = planes;
    b.norms_user = norms_out;
    b.seed = seed;
    b.step = step;
    return rtn_compress(plan, b, vec_ok(plan, g, ld), true, (hipStream_t)hip_stream);
}

mlmc_status mlmc_compress_bits_static(const mlmc_plan_t* plan, const void* g, int64_t ld, uint64_t seed, uint64_t step,
                                      int32_t* level, int32_t* scale_exp, uint64_t* planes, int32_t* dev_status,
                                      void* hip_stream) {
    if (!plan || (plan->kind != MLMC_BITS && plan->kind != MLMC_FBITS && plan->kind != MLMC_VBITS)) return MLMC_EINVAL;
    if (plan->ws_bytes > (size_t)MLMC_STATIC_SCRATCH_BYTES) return MLMC_ELIMIT;   // before any HIP call
    void* ws = nullptr;
    const mlmc_status rc = static_scratch_of_current_device(&ws);
    if (rc != MLMC_OK) return rc;
    // same kernels as mlmc_compress_bits; the part of the scratch that must start at zero is cleared by the first of them
    return mlmc_compress_bits(plan, g, ld, seed, step, level, scale_exp, planes, dev_status, ws, hip_stream);
}

static mlmc_status aggregate_impl(const mlmc_plan_t* plan, const int32_t* level, const int64_t* row_off, const uint32_t* idx,
                                  const float* val, int64_t capacity, const uint32_t* tile_off, const int32_t* scale_exp,
                                  const uint64_t* planes, float alpha, float* out, float eta, float* x, void* ws, void* hip_stream) {
    if (!plan || (!out && !x)) return MLMC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (plan->kind == MLMC_TOPK || plan->kind == MLMC_STOPK) {
        if (!row_off || !idx || !val || capacity < 0 || scale_exp || planes) return MLMC_EINVAL;
        if (!tile_off && (!ws || (uintptr_t)ws % 256)) return MLMC_EINVAL;
        uint32_t* tws = ws ? (uint32_t*)((char*)ws + plan->off_tileoff) : nullptr;
        return agg_sparse(plan, row_off, idx, val, capacity, tile_off, tws, alpha, out, eta, x, st);
    }
    if (!level || !planes || row_off || idx || val || tile_off) return MLMC_EINVAL;
    if (plan->kind != MLMC_FBITS && !scale_exp) return MLMC_EINVAL;
    BitsArgs b;
    fill_bits_args(plan, b, nullptr, plan->d, nullptr, nullptr);
    return agg_bits(plan, b, level, scale_exp, planes, alpha, out, eta, x, st);
}

mlmc_status mlmc_aggregate(const mlmc_plan_t* plan, const int32_t* level, const int64_t* row_off, const uint32_t* idx,
                           const float* val, int64_t capacity, const uint32_t* tile_off, const int32_t* scale_exp, const uint64_t* planes,
                           float alpha, float* out, void* ws, void* hip_stream) {
    if (!out) return MLMC_EINVAL;
    return aggregate_impl(plan, level, row_off, idx, val, capacity, tile_off, scale_exp, planes, alpha, out, 0.0f, nullptr, ws,
                          hip_stream);
}

mlmc_status mlmc_aggregate_update(const mlmc_plan_t* plan, const int32_t* level, const int64_t* row_off, const uint32_t* idx,
                                  const float* val, int64_t capacity, const uint32_t* tile_off, const int32_t* scale_exp,
                                  const uint64_t* planes, float alpha, float eta, float* x, float* out, void* ws,
                                  void* hip_stream) {
    if (!x || x == out) return MLMC_EINVAL;
    return aggregate_impl(plan, level, row_off, idx, val, capacity, tile_off, scale_exp, planes, alpha, out, eta, x, ws, hip_stream);
}

mlmc_status mlmc_message_bits(const mlmc_plan_t* plan, const int32_t* level, uint64_t* bits, void* hip_stream) {
    if (!plan || !level || !bits) return MLMC_EINVAL;
    return message_bits(plan, level, (unsigned long long*)bits, (hipStream_t)hip_stream);
}

}  // extern "C"
