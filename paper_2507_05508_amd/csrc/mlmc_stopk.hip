// s-segmented Top-k MLMC on gfx950 (Sec. 2.2 "s-Top-k", Sec. 3.2, Lemma 3.4, App. D): the ladder k_l = min(s l, d),
// l = 0..L = ceil(d / s), g^0 = 0, adaptive level probabilities over all L bands.  The residual of level l is the
// l-th segment of the row sorted by magnitude, so the whole row is sorted once:
//
//   k_rs_hist / k_rs_scan / k_rs_scatter   stable least-significant-digit radix sort of {inverted |g| key, index} pairs,
//                 8 bits per pass (4 passes for fp32, 2 for bf16 inputs whose keys have 16 significant bits); the
//                 first pass reads the gradients themselves.  Stable + initial index order = ties by lower index.
//   k_sb_norms    Delta_l for every band: exact integer sum of the squares of a segment (640-bit accumulate in LDS),
//                 rounded once to fp64, sqrt (Lemma 3.4, App. D)
//   k_sb_draw     p_l = Delta_l / sum Delta in level order, integer inverse CDF of the Philox word, weight (Alg. 3)
//   k_sb_mark / k_sb_offsets / k_sb_write   the drawn segment as an index-ordered message: its entries are marked in
//                 a bitmap over the row, tiles are counted and scanned, entries written in index order with their
//                 fp32 weight applied (Eq. (6))
#include "mlmc_device.h"

namespace mlmc {

constexpr int RS_TILE = 4096;     // elements of one sort block
constexpr int RS_THREADS = 256;   // four waves; wave w owns a quarter of the block, in order
constexpr int RS_PER_WAVE = RS_TILE / (RS_THREADS / 64);
constexpr int RS_GROUPS = RS_PER_WAVE / 64;   // 64-element groups of a wave

__device__ __forceinline__ uint32_t inv_key(uint32_t bits) { return 0x7FFFFFFFu - key_of_bits(bits); }   // ascending = magnitude descending

// One element of a sort pass.  FIRST: the pairs are formed from the gradients (index = position).
template <int DT, bool FIRST>
__device__ __forceinline__ uint2 rs_load(const StopkArgs& a, const RowLoader<DT, false>& ld, const uint2* src, int row, int64_t i) {
    if (FIRST) return make_uint2(inv_key(ld.load1(i)), (uint32_t)i);
    return src[(size_t)row * a.d + i];
}

// Digit counts of every block: counts[row][bin][blk].
template <int DT, bool FIRST>
__global__ __launch_bounds__(RS_THREADS) void k_rs_hist(StopkArgs a, const uint2* src, int shift) {
    __shared__ uint32_t s_h[256];
    const int row = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    s_h[tid] = 0;
    __syncthreads();
    RowLoader<DT, false> ld(a.g, a.ld, a.d, row);
    const int64_t i0 = (int64_t)blk * RS_TILE;
    const int64_t i1 = i0 + RS_TILE < a.d ? i0 + RS_TILE : a.d;
    bool nonfinite = false;
    // the block's loads issued sixteen at a time per thread (a loop of single loads waits for each in turn)
    batched_loop<RS_TILE / RS_THREADS, RS_THREADS>(0u, (uint32_t)(i1 - i0), (uint32_t)tid,
        [&](uint32_t i) { return rs_load<DT, FIRST>(a, ld, src, row, i0 + i).x; },
        [&](uint32_t, uint32_t key) {
            atomicAdd(&s_h[(key >> shift) & 255u], 1u);
            if (FIRST) nonfinite |= key <= 0x7FFFFFFFu - 0x7F800000u;   // Inf / NaN keys (ordered by their bit pattern)
        });
    if (FIRST && __ballot(nonfinite) && lane_id() == 0) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
    __syncthreads();
    a.counts[((size_t)row * 256 + tid) * a.nblk + blk] = s_h[tid];
}

// Exclusive prefix of counts[row][bin][.] over the blocks, one workgroup per (bin, row), and the bin's total; the
// scatter adds the totals of the lower bins.
__global__ __launch_bounds__(1024) void k_rs_scan(StopkArgs a) {
    __shared__ uint32_t s_scan[1024 / 64 + 1];
    const int bin = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
    uint32_t* c = a.counts + ((size_t)row * 256 + bin) * a.nblk;
    uint32_t carry = 0;
    for (int j0 = 0; j0 < a.nblk; j0 += 1024) {
        const int j = j0 + tid;
        const uint32_t v = j < a.nblk ? c[j] : 0u;
        uint32_t total;
        const uint32_t ex = block_excl_scan<1024>(v, s_scan, total);
        if (j < a.nblk) c[j] = carry + ex;
        carry += total;
    }
    if (tid == 0) a.bin_total[row * 256 + bin] = carry;
}

// Stable scatter of one pass.  Order is kept at every step: a wave walks its elements in order, lanes of a group
// rank themselves among the lanes with the same digit below them, waves and blocks start where the prefixes say.
// The block's pairs are first put in digit order in LDS, then written out: pairs of one digit go to consecutive
// addresses, so the writes come in runs instead of single 8-byte stores.
template <int DT, bool FIRST>
__global__ __launch_bounds__(RS_THREADS) void k_rs_scatter(StopkArgs a, const uint2* src, uint2* dst, int shift) {
    __shared__ uint32_t s_hist[RS_THREADS / 64][256];   // per wave and digit: the count, then (in place) the slot in the block's digit-ordered staging area
    uint32_t (*s_base)[256] = s_hist;
    __shared__ uint32_t s_gstart[256];                  // global position of the block's first pair of a digit minus its slot
    __shared__ uint32_t s_scan[RS_THREADS / 64 + 1];
    __shared__ uint2 s_stage[RS_TILE];
    const int row = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < (RS_THREADS / 64) * 256; i += RS_THREADS) (&s_hist[0][0])[i] = 0;
    __syncthreads();
    RowLoader<DT, false> ld(a.g, a.ld, a.d, row);
    const int64_t b0 = (int64_t)blk * RS_TILE;
    const int64_t w0 = b0 + (int64_t)wave * RS_PER_WAVE;
    uint2 e[RS_GROUPS];
    if (b0 + RS_TILE <= a.d) {   // a whole block (uniform): no bounds check between the loads, they are issued together
#pragma unroll
        for (int q = 0; q < RS_GROUPS; ++q) e[q] = rs_load<DT, FIRST>(a, ld, src, row, w0 + q * 64 + lane);
    } else {
#pragma unroll
        for (int q = 0; q < RS_GROUPS; ++q) {
            const int64_t i = w0 + q * 64 + lane;
            e[q] = i < a.d ? rs_load<DT, FIRST>(a, ld, src, row, i) : make_uint2(0u, 0u);
        }
    }
#pragma unroll
    for (int q = 0; q < RS_GROUPS; ++q)
        if (w0 + q * 64 + lane < a.d) atomicAdd(&s_hist[wave][(e[q].x >> shift) & 255u], 1u);
    __syncthreads();
    {
        // digit `tid`: its pairs of this block start at (lower bins of the row) + (earlier blocks of the bin) in the
        // output, and at (lower digits of this block) in the staging area
        uint32_t row_total, blk_total, mine = 0;
#pragma unroll
        for (int w = 0; w < RS_THREADS / 64; ++w) mine += s_hist[w][tid];
        const uint32_t lower = block_excl_scan<RS_THREADS>(a.bin_total[row * 256 + tid], s_scan, row_total);
        if (tid == 0 && (int64_t)row_total != a.d) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        const uint32_t slot0 = block_excl_scan<RS_THREADS>(mine, s_scan, blk_total);
        s_gstart[tid] = lower + a.counts[((size_t)row * 256 + tid) * a.nblk + blk] - slot0;
        uint32_t run = slot0;
#pragma unroll
        for (int w = 0; w < RS_THREADS / 64; ++w) {
            const uint32_t c = s_hist[w][tid];
            s_base[w][tid] = run;
            run += c;
        }
    }
    __syncthreads();
    const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int q = 0; q < RS_GROUPS; ++q) {
        const bool valid = w0 + q * 64 + lane < a.d;
        const uint32_t digit = (e[q].x >> shift) & 255u;
        uint64_t peers = __ballot(valid);   // lanes with this lane's digit
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t m = __ballot(valid && ((digit >> b) & 1u));
            peers &= ((digit >> b) & 1u) ? m : ~m;
        }
        const uint32_t rank = (uint32_t)__popcll(peers & below);
        const uint32_t base = s_base[wave][digit];
        wave_lds_sync();   // every lane has read its base before a leader moves it on
        if (valid && rank == 0) s_base[wave][digit] = base + (uint32_t)__popcll(peers);
        wave_lds_sync();
        if (valid) s_stage[base + rank] = e[q];
    }
    __syncthreads();
    uint2* out = dst + (size_t)row * a.d;
    const int nvalid = (int)(a.d - b0 < RS_TILE ? a.d - b0 : RS_TILE);
    for (int i = tid; i < nvalid; i += RS_THREADS) {
        const uint2 p = s_stage[i];
        out[s_gstart[(p.x >> shift) & 255u] + (uint32_t)i] = p;
    }
}

// Delta_l of every band of every row from the sorted pairs: a wave takes bands in turn.  The squares of a segment are
// added exactly: sig^2 * 2^(2 (E' - 1)) in units of 2^-298, split into 32-bit words that go to 64-bit counters of their
// word positions (LDS atomics, any order), one carry pass, one rounding to fp64, sqrt.
constexpr int SN_WAVES = 4;
__global__ __launch_bounds__(SN_WAVES * 64) void k_sb_norms(StopkArgs a, const uint2* sorted) {
    __shared__ unsigned long long s_wide[SN_WAVES][20];
    __shared__ uint32_t s_big[SN_WAVES][20];
    const int row = blockIdx.y;
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint2* sp = sorted + (size_t)row * a.d;
    for (int64_t band = (int64_t)blockIdx.x * SN_WAVES + wave; band < a.L; band += (int64_t)gridDim.x * SN_WAVES) {
        if (lane < 20) s_wide[wave][lane] = 0ull;
        wave_lds_sync();
        const int64_t lo = band * a.s, hi = lo + a.s < a.d ? lo + a.s : a.d;
        // A lane meets its keys in descending order, so their exponents come in runs: the squares of a run are summed in
        // registers (low and high halves apart, no overflow for any segment length) and reach LDS once per run.
        auto flush = [&](uint32_t E, uint64_t slo, uint64_t shi) {
            const int shift = 2 * ((int)(E ? E : 1u) - 1);
            auto add = [&](uint64_t v, int sh) {
                if (!v) return;
                const int wi = sh >> 5, bs = sh & 31;
                const uint32_t p0 = (uint32_t)(v << bs);
                const uint32_t p1 = (uint32_t)(bs ? v >> (32 - bs) : v >> 32);
                const uint32_t p2 = bs ? (uint32_t)(v >> (64 - bs)) : 0u;
                if (p0 && wi < 20) atomicAdd(&s_wide[wave][wi], (unsigned long long)p0);
                if (p1 && wi + 1 < 20) atomicAdd(&s_wide[wave][wi + 1], (unsigned long long)p1);
                if (p2 && wi + 2 < 20) atomicAdd(&s_wide[wave][wi + 2], (unsigned long long)p2);
            };
            add(slo, shift);
            add(shi, shift + 32);
        };
        uint32_t curE = 0xFFFFFFFFu;
        uint64_t slo = 0, shi = 0;
        // eight loads of a lane in flight (past the segment's end: its last entry, ignored), consumed in order
        for (int64_t i = lo + lane; i < hi; i += 64 * 8) {
            uint32_t kx[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t j = i + 64 * u;
                kx[u] = sp[j < hi ? j : hi - 1].x;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (i + 64 * u < hi) {
                    const uint32_t key = 0x7FFFFFFFu - kx[u];
                    const uint32_t E = key >> 23;
                    if (E != curE) {
                        if (curE != 0xFFFFFFFFu) flush(curE, slo, shi);
                        curE = E;
                        slo = 0;
                        shi = 0;
                    }
                    const uint64_t sq = sig_square(key);
                    slo += sq & 0xFFFFFFFFull;
                    shi += sq >> 32;
                }
            }
        }
        if (curE != 0xFFFFFFFFu) flush(curE, slo, shi);
        wave_lds_sync();
        if (lane == 0) {
            unsigned long long carry = 0;
            for (int i = 0; i < 20; ++i) {
                const unsigned long long t = s_wide[wave][i] + carry;
                s_big[wave][i] = (uint32_t)t;
                carry = t >> 32;
            }
            BigAcc acc;
            acc.w = s_big[wave];
            const double nrm = __dsqrt_rn(acc.to_double());
            a.norms[(size_t)row * a.L + band] = nrm;
            if (a.norms_user) a.norms_user[(size_t)row * a.L + band] = nrm;
        }
        wave_lds_sync();
    }
}

// Level draw of every row (Alg. 3): p_l = Delta_l / (Delta_1 + ... + Delta_L).  The sum and the running CDF are taken in
// level order by one thread (the order fixes the roundings) - but only the additions: the quotients before them and the
// integer thresholds and comparisons after them are independent per level and spread over the workgroup.  The norms
// pass through LDS in chunks.
constexpr int SD_CHUNK = 8192;
__global__ __launch_bounds__(1024) void k_sb_draw(StopkArgs a) {
    __shared__ double s_n[SD_CHUNK];     // norms, then probabilities, of the chunk
    __shared__ double s_cdf[SD_CHUNK];   // running sums of the probabilities up to every level of the chunk
    __shared__ double s_tot;
    __shared__ int32_t s_found;          // lowest level met so far whose threshold lies above the drawn word
    const int row = blockIdx.x, tid = threadIdx.x;
    const double* nr = a.norms + (size_t)row * a.L;
    const int L = a.L;
    double tot = 0.0;
    for (int c0 = 0; c0 < L; c0 += SD_CHUNK) {
        const int n = L - c0 < SD_CHUNK ? L - c0 : SD_CHUNK;
        __syncthreads();
        for (int i = tid; i < n; i += 1024) s_n[i] = nr[c0 + i];
        __syncthreads();
        if (tid == 0) for (int i = 0; i < n; ++i) tot = __dadd_rn(tot, s_n[i]);
    }
    if (tid == 0) { s_tot = tot; s_found = 0x7FFFFFFF; }
    __syncthreads();
    tot = s_tot;
    const uint32_t x = philox_word0(a.seed, a.step, (uint32_t)row);
    const double uni = __ddiv_rn(1.0, (double)L);
    double c = 0.0, pl = 0.0;
    int level = L;
    for (int c0 = 0; c0 < L; c0 += SD_CHUNK) {
        const int n = L - c0 < SD_CHUNK ? L - c0 : SD_CHUNK;
        __syncthreads();
        for (int i = tid; i < n; i += 1024) s_n[i] = tot == 0.0 ? uni : __ddiv_rn(nr[c0 + i], tot);
        __syncthreads();
        if (tid == 0) {
            for (int i = 0; i < n; ++i) {
                c = __dadd_rn(c, s_n[i]);
                s_cdf[i] = c;
            }
        }
        __syncthreads();
        for (int i = tid; i < n; i += 1024) {
            const double t = floor(__dmul_rn(s_cdf[i], 4294967296.0));
            uint64_t T;
            if (!(t > 0.0)) T = 0;
            else if (t >= 4294967296.0) T = 4294967296ull;
            else T = (uint64_t)t;
            if (c0 + i == L - 1) T = 4294967296ull;
            if ((uint64_t)x < T) atomicMin(&s_found, c0 + i + 1);
        }
        __syncthreads();
        if (s_found != 0x7FFFFFFF) {   // uniform: the chunk holds the level, and s_n its probability
            level = s_found;
            pl = s_n[level - 1 - c0];
            break;
        }
    }
    if (tid == 0) {
        SRow* sr = a.srow + row;
        sr->level = level;
        sr->weight = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
        const int64_t lo = (int64_t)(level - 1) * a.s;
        sr->lo = lo;
        sr->count = lo + a.s < a.d ? a.s : a.d - lo;
        a.level[row] = level;
    }
}

__global__ __launch_bounds__(256) void k_sb_clear(uint4* p, size_t n16, int32_t* dev_status) {
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) p[i] = z;
    if (dev_status && blockIdx.x == 0 && threadIdx.x == 0) *dev_status = 0;
}

// The entries of the drawn segment, marked in the row's bitmap (bit j of the row: entry j is in the message) and counted
// per tile of 4096 indices.
__global__ __launch_bounds__(256) void k_sb_mark(StopkArgs a, const uint2* sorted) {
    const int row = blockIdx.y;
    const SRow sr = a.srow[row];
    uint32_t* bm = a.bitmap + (size_t)row * a.bm_words;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < sr.count; i += (int64_t)gridDim.x * 256) {
        const uint32_t j = sorted[(size_t)row * a.d + sr.lo + i].y;
        atomicOr(&bm[j >> 5], 1u << (j & 31u));
        atomicAdd(&a.tile_cnt[(size_t)row * a.ntiles + (j >> 12)], 1u);   // indices are distinct: an entry counts once
    }
}

// Per row: entries before every tile of 4096 indices, and where the row's message starts.
__global__ __launch_bounds__(1024) void k_sb_offsets(StopkArgs a) {
    __shared__ uint32_t s_scan[1024 / 64 + 1];
    const int row = blockIdx.x, tid = threadIdx.x;
    uint32_t* to = a.tile_off + (size_t)row * (a.ntiles + 1);
    const uint32_t* tc = a.tile_cnt + (size_t)row * a.ntiles;
    uint32_t carry = 0;
    for (int64_t j0 = 0; j0 < a.ntiles; j0 += 1024) {
        const int64_t t = j0 + tid;
        const uint32_t c = t < a.ntiles ? tc[t] : 0u;
        uint32_t round_total;
        const uint32_t ex = block_excl_scan<1024>(c, s_scan, round_total);
        if (t < a.ntiles) to[t] = carry + ex;
        carry += round_total;
    }
    const uint32_t total = carry;
    if (tid == 0) {
        to[a.ntiles] = total;
        if ((int64_t)total != a.srow[row].count) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        int64_t start = 0;
        for (int r = 0; r < row; ++r) start += a.srow[r].count;
        a.row_off[row] = start;
        if (row == a.M - 1) {
            a.row_off[a.M] = start + total;
            if (start + (int64_t)total > a.capacity) atomicOr(a.dev_status, MLMC_DEV_CAPACITY);
        }
    }
}

// The message of a row in index order: a wave takes a tile, a lane two words of its bitmap.
template <int DT>
__global__ __launch_bounds__(256) void k_sb_write(StopkArgs a) {
    const int row = blockIdx.y;
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
    if (tile >= a.ntiles) return;
    const uint32_t* bm = a.bitmap + (size_t)row * a.bm_words;
    const uint32_t* to = a.tile_off + (size_t)row * (a.ntiles + 1);
    if (to[tile + 1] == to[tile]) return;   // nothing of the segment in this tile
    RowLoader<DT, false> ld(a.g, a.ld, a.d, row);
    const float w = a.srow[row].weight;
    const int64_t w0 = tile * (TILE / 32) + lane * 2;
    uint32_t b0 = w0 < a.bm_words ? bm[w0] : 0u, b1 = w0 + 1 < a.bm_words ? bm[w0 + 1] : 0u;
    const uint32_t mine = (uint32_t)__popc(b0) + (uint32_t)__popc(b1);
    uint32_t inc = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(inc, o, 64);
        if (lane >= (uint32_t)o) inc += u;
    }
    int64_t at = a.row_off[row] + to[tile] + (inc - mine);
    auto emit = [&](uint32_t bits, int64_t jbase) {
        while (bits) {
            const int b = __builtin_ctz(bits);
            bits &= bits - 1u;
            const int64_t j = jbase + b;
            if (at < a.capacity) {
                a.idx[at] = (uint32_t)j;
                a.val[at] = __fmul_rn(__uint_as_float(ld.load1(j)), w);
            }
            ++at;
        }
    };
    emit(b0, w0 * 32);
    emit(b1, (w0 + 1) * 32);
}

// ---------------------------------------------------------------------------------------------------
template <int DT>
static mlmc_status launch_stopk(const mlmc_plan_t* pl, const StopkArgs& a, bool message, hipStream_t st) {
    const dim3 sgrid(a.nblk, pl->M);
    // bitmaps, tile counts and device status start at zero
    {
        const size_t n16 = a.clear_bytes / 16;   // the bitmaps and, right behind them, the tile counts
        int blocks = (int)((n16 + 255) / 256);
        if (blocks > 2048) blocks = 2048;
        MLMC_LAUNCH(K_ZERO, st, k_sb_clear<<<blocks, 256, 0, st>>>((uint4*)a.bitmap, n16, a.dev_status));
    }
    // sort: pass 0 reads the gradients; bf16 keys have their low 16 bits clear, so their two low digits are constant
    const int first_shift = pl->dtype == MLMC_BF16 ? 16 : 0;
    uint2* bufs[2] = {a.pa, a.pb};
    int cur = 0;   // the pass writes bufs[cur]
    for (int shift = first_shift; shift < 32; shift += 8) {
        const uint2* src = shift == first_shift ? nullptr : bufs[cur ^ 1];
        if (shift == first_shift) {
            MLMC_LAUNCH(K_RS_HIST, st, k_rs_hist<DT, true><<<sgrid, RS_THREADS, 0, st>>>(a, src, shift));
            MLMC_LAUNCH(K_RS_SCAN, st, k_rs_scan<<<dim3(256, pl->M), 1024, 0, st>>>(a));
            MLMC_LAUNCH(K_RS_SCATTER, st, k_rs_scatter<DT, true><<<sgrid, RS_THREADS, 0, st>>>(a, src, bufs[cur], shift));
        } else {
            MLMC_LAUNCH(K_RS_HIST, st, k_rs_hist<DT, false><<<sgrid, RS_THREADS, 0, st>>>(a, src, shift));
            MLMC_LAUNCH(K_RS_SCAN, st, k_rs_scan<<<dim3(256, pl->M), 1024, 0, st>>>(a));
            MLMC_LAUNCH(K_RS_SCATTER, st, k_rs_scatter<DT, false><<<sgrid, RS_THREADS, 0, st>>>(a, src, bufs[cur], shift));
        }
        cur ^= 1;
    }
    const uint2* sorted = bufs[cur ^ 1];
    {
        int64_t gx = (a.L + SN_WAVES - 1) / SN_WAVES;
        const int64_t cap = 8192 / pl->M > 0 ? 8192 / pl->M : 1;
        if (gx > cap) gx = cap;
        MLMC_LAUNCH(K_SB_NORMS, st, k_sb_norms<<<dim3((unsigned)gx, pl->M), SN_WAVES * 64, 0, st>>>(a, sorted));
    }
    if (!message) return MLMC_OK;
    MLMC_LAUNCH(K_SB_DRAW, st, k_sb_draw<<<pl->M, 1024, 0, st>>>(a));
    {
        int64_t gx = (a.s + 255) / 256;
        if (gx > 1024) gx = 1024;
        MLMC_LAUNCH(K_SB_MARK, st, k_sb_mark<<<dim3((unsigned)gx, pl->M), 256, 0, st>>>(a, sorted));
    }
    MLMC_LAUNCH(K_SB_OFFSETS, st, k_sb_offsets<<<pl->M, 1024, 0, st>>>(a));
    MLMC_LAUNCH(K_SB_WRITE, st, k_sb_write<DT><<<dim3((unsigned)((a.ntiles + 3) / 4), pl->M), 256, 0, st>>>(a));
    return MLMC_OK;
}

mlmc_status stopk_run(const mlmc_plan_t* pl, const StopkArgs& a, bool message, hipStream_t st) {
    if (pl->dtype == MLMC_F32) return launch_stopk<MLMC_F32>(pl, a, message, st);
    return launch_stopk<MLMC_BF16>(pl, a, message, st);
}

}  // namespace mlmc
