// Top-k MLMC on gfx950: exact multi-rank select on |g| keys, exact band sums of squares, level draw,
// index-ordered band message.  A row is normally read once (plus a sample); a second read happens only when
// the band that was set aside during the first read is not the band that is drawn.
//
// Pipeline per call (all rows at once):
//   k_hist       14-bit first-digit histogram (exponent + 6 mantissa bits) of a SAMPLE of every row: one
//                1024-element block out of 2^s (s = 0 for short rows: then the histogram is exact)
//   k_scan       per row: from the (scaled) sample histogram, a ZONE of buckets around every needed rank
//                threshold that holds it with overwhelming probability; the buckets between zones are REGIONS whose
//                elements lie wholly inside one band.  With known p the level is drawn here; with adaptive p it is
//                predicted from the histogram.  Writes the class table: bucket -> {region, sum group, stage flag | zone}.
//   k_main2      (k_main for short rows and the redo round) the selection read: per region exact element counts (per chunk and per row) and exact sums of
//                squared significands per (exponent, region); zone candidates and the members of the staged band
//                go to per-wave private lists, the candidates from there to per-zone lists
//   k_fhist      per (zone, slice): histogram of the candidates over the zone's own key range (that of its buckets,
//                cut at the largest key of the row)
//   k_finish<0>  per (zone, slice): the exact counts above the zone prove (or refute) that its thresholds lie
//                inside; candidates of the thresholds' bins are gathered, all others classified by their bin
//                (per-chunk counts of the zone's parts, exact sums per part and exponent)
//   k_finish<1>  per zone: gathered candidates ranked in LDS -> exact threshold key and index cut among equal keys
//                (radix select on an overflow list when the bins hold many: massive ties).
//                A refuted row is flagged and redone with an exact histogram (k_hist, k_scan, k_main, k_finish<1>
//                once more, for flagged rows only; these launches return at once otherwise).
//   k_norms      big-integer accumulation of group and part sums -> correctly rounded fp64 S_l -> Delta_l
//                (Lemma 3.4), then the adaptive level draw (Alg. 3)
//   k_msgplan    per row: where its message starts, message entries before every chunk, the three thresholds,
//                the row's place by message length (the two kernels below take the long rows first)
//   k_filter     rows whose staged band is the drawn one: base band + drawn band (Eq. (6)) from the staged lists,
//                ordered by index through a bitmap over the chunk
//   k_write      the other rows: second read, a workgroup owns a chunk whose output offset is known
#include <type_traits>

#include "mlmc_device.h"

namespace mlmc {

// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_zero(uint4* p, size_t n16, int32_t* dev_status) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    uint4 z = make_uint4(0, 0, 0, 0);
    for (; i < n16; i += stride) p[i] = z;
    if (dev_status && blockIdx.x == 0 && threadIdx.x == 0) *dev_status = 0;
}

// ---------------------------------------------------------------------------------------------------
// First-digit histogram of the sampled blocks (block b of 1024 elements is sampled when b % S == S / 2).
// exact_pass: only rows flagged for an exact redo are read, every block, into hist2.
constexpr int HIST_THREADS = 512;
template <int DT, bool VEC>
__global__ __launch_bounds__(HIST_THREADS) void k_hist(TopkArgs a, int exact_pass) {
    __shared__ uint32_t h[NB1];
    const int row = blockIdx.y;
    if (exact_pass && !a.rinfo[row].respec) return;
    const int shift = exact_pass ? 0 : a.sample_shift;
    const int64_t S = (int64_t)1 << shift, first = S >> 1;
    const int64_t nblk = (a.d + 1023) / 1024;
    const int64_t ns = nblk > first ? (nblk - first + S - 1) / S : 0;   // sampled blocks of the row
    const int64_t per = (ns + gridDim.x - 1) / gridDim.x;
    const int64_t i0 = (int64_t)blockIdx.x * per;
    const int64_t i1 = i0 + per < ns ? i0 + per : ns;
    if (i0 >= i1) return;
    for (int b = threadIdx.x; b < NB1; b += HIST_THREADS) h[b] = 0;
    __syncthreads();
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t maxkey = 0;
    auto count4 = [&](const uint32_t (&b)[4], int nv) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (c < nv) {
                const uint32_t key = key_of_bits(b[c]);
                atomicAdd(&h[key >> B1_SHIFT], 1u);
                maxkey = key > maxkey ? key : maxkey;
            }
        }
    };
    // A wave's whole blocks, the four loads of the next one in flight while the current one is counted; the row's last
    // block, when it is a partial one, comes after them (blocks ascend with i, so it is the last of its wave).
    const int64_t nwhole = a.d >> 10, wstep = HIST_THREADS / 64;
    auto fetch = [&](int64_t i, uint32_t (&b)[4][4]) {
        const int64_t base = (first + i * S) * 1024 + lane * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) ld.load4_full(base + q * 256, b[q]);
    };
    auto count = [&](const uint32_t (&b)[4][4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) count4(b[q], 4);
    };
    auto whole = [&](int64_t i) -> bool { return i < i1 && first + i * S < nwhole; };   // uniform
    uint32_t b0[4][4], b1[4][4];
    int64_t i = i0 + wave;
    bool have = whole(i);
    if (have) fetch(i, b0);
    while (have) {
        const bool more1 = whole(i + wstep);
        if (more1) fetch(i + wstep, b1);
        count(b0);
        i += wstep;
        if (!more1) break;
        const bool more2 = whole(i + wstep);
        if (more2) fetch(i + wstep, b0);
        count(b1);
        i += wstep;
        have = more2;
    }
    if (i < i1) {   // the partial last block of the row
        const int64_t base = (first + i * S) * 1024 + lane * 4;
        for (int q = 0; q < 4; ++q) {
            const int nv = ld.load4(base + q * 256, b0[q]);
            count4(b0[q], nv);
        }
    }
    __syncthreads();
    uint32_t* gh = (exact_pass ? a.hist2 : a.hist) + (size_t)row * NB1;
    for (int b = threadIdx.x; b < NB1; b += HIST_THREADS) {
        uint32_t v = h[b];
        if (v) atomicAdd(&gh[b], v);
    }
    if (__ballot(maxkey >= 0x7F800000u) && lane == 0) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
}

// ---------------------------------------------------------------------------------------------------
// Level draw of one row (Alg. 2 / Alg. 3 "Sample l ~ p"), run by one thread.
// `p` is LMAX doubles of LDS scratch: a thread-local array indexed by a loop variable would live in scratch memory.
__device__ void draw_row(const TopkArgs& a, int row, const double* norms_row, double* p) {
    const int L = a.L;
    if (a.draw_mode == 0) {
        for (int l = 0; l < L; ++l) p[l] = a.p_fixed[l];
    } else if (a.draw_mode == 1) {
        for (int l = 0; l < L; ++l) p[l] = a.p_dev[(size_t)row * L + l];
    } else {
        const double* n = a.draw_mode == 2 ? a.p_dev + (size_t)row * L : norms_row;
        double tot = 0.0;
        for (int l = 0; l < L; ++l) tot = __dadd_rn(tot, n[l]);
        for (int l = 0; l < L; ++l) p[l] = tot == 0.0 ? __ddiv_rn(1.0, (double)L) : __ddiv_rn(n[l], tot);
    }
    uint32_t x = philox_word0(a.seed, a.step, (uint32_t)row);
    int level = draw_from_p(p, L, x);
    double pl = p[level - 1];
    RowInfo* ri = a.rinfo + row;
    ri->level = level;
    ri->weight = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
    ri->draw_x = x;
    a.level[row] = level;
}

// ---------------------------------------------------------------------------------------------------
// Per row: zones and regions from the histogram, candidate list layout, the class table.
// How far (in standard deviations of the sampled count) a zone reaches on either side of the estimated rank.  The
// binomial model fits when every homogeneous stretch of a row contributes many sampled blocks; a small sample of a
// row made of segments with different scales is over-dispersed (whole blocks share a scale), hence the wide margin
// there.  A zone that misses its threshold only costs the exact redo of that row.
constexpr double ZONE_SIGMAS = 8.0;
constexpr double ZONE_SIGMAS_BIG = 5.0;         // samples of at least ZONE_BIG_SAMPLE elements
constexpr int64_t ZONE_BIG_SAMPLE = 1 << 20;
constexpr int64_t STAGE_MAX_BAND_INV = 8;   // bands wider than d / 8 are not staged

__global__ __launch_bounds__(1024) void k_scan(TopkArgs a, int exact_pass) {
    __shared__ __align__(16) uint32_t s_h[NB1];
    __shared__ uint32_t s_cum[NB1];          // sampled elements in buckets above b
    __shared__ uint32_t s_scan[17];
    __shared__ int32_t s_active[TMAX];
    __shared__ int64_t s_lo[TMAX], s_hi[TMAX];   // sample ranks (1-based) that bound the threshold's zone
    __shared__ uint32_t s_top[TMAX], s_bot[TMAX];
    __shared__ int32_t s_nz, s_lev;
    __shared__ uint32_t s_ztop[ZMAX], s_zbot[ZMAX];
    __shared__ int32_t s_label[RMAX];
    __shared__ float s_est[LMAX + 2];
    __shared__ double s_p[LMAX];
    __shared__ double s_kd[TMAX];
    __shared__ int64_t s_k[TMAX];            // the ladder (indexed by loop variables below: kept out of the argument block)
    __shared__ uint16_t s_gexp[GMAX], s_gband[GMAX];
    __shared__ uint32_t s_bmin, s_bmax;      // occupied buckets of the (sampled) histogram

    const int row = blockIdx.x, tid = threadIdx.x;
    RowInfo* ri = a.rinfo + row;
    RowAcc* ra = a.racc + row;
    const int L = a.L;
    if (exact_pass) {
        if (!ri->respec) return;
        if (tid == 0) atomicOr(a.dev_status, MLMC_DEV_REDONE);
        // the row starts over: clear what the first attempt accumulated
        uint32_t* z = (uint32_t*)ra;
        for (int i = tid; i < (int)(sizeof(RowAcc) / 4); i += 1024) z[i] = 0;
        z = a.zhist + (size_t)row * ZMAX * FH_BINS;
        for (int i = tid; i < ZMAX * FH_BINS; i += 1024) z[i] = 0;
        z = (uint32_t*)(a.zpacc + (size_t)row * ZMAX * PIECE_CLASSES * 2);
        for (int i = tid; i < ZMAX * PIECE_CLASSES * 4; i += 1024) z[i] = 0;
        z = a.chunk_zcnt + (size_t)row * a.cchunks_per_row * ZPMAX;
        for (int i = tid; i < a.cchunks_per_row * ZPMAX; i += 1024) z[i] = 0;
    }
    const bool exact = exact_pass || a.sample_shift == 0;
    const uint32_t* gh = (exact_pass ? a.hist2 : a.hist) + (size_t)row * NB1;

    if (tid == 0) {
        if (!exact_pass) {
            ri->respec = 0;
            if (!a.all_thresholds) draw_row(a, row, nullptr, s_p);  // p is known up front: draw before anything else
        }
        ri->exact = exact ? 1 : 0;
        s_lev = a.all_thresholds ? 0 : ri->level;
    }
    // descending buckets: rb = tid*16 + i  <->  b = NB1 - 1 - rb.  A thread fetches its sixteen buckets with four
    // loads issued together (a loop over strided single loads waits for every one of them in turn).
    uint32_t hv[16];
    {
        const uint4* src = (const uint4*)(gh + (NB1 - 16 - tid * 16));
        uint4 q[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) q[i] = src[i];
        uint4* dst = (uint4*)(s_h + (NB1 - 16 - tid * 16));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dst[i] = q[i];
            hv[15 - 4 * i] = q[i].x; hv[14 - 4 * i] = q[i].y; hv[13 - 4 * i] = q[i].z; hv[12 - 4 * i] = q[i].w;
        }
    }
    for (int g = tid; g < GMAX; g += 1024) { s_gband[g] = 0xFFFF; s_gexp[g] = 0; }
    if (tid <= L) { s_k[tid] = a.k[tid]; s_kd[tid] = (double)a.k[tid]; }
    if (tid == 0) { s_bmin = NB1; s_bmax = 0; }
    __syncthreads();
    const int lev = s_lev;

    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += hv[i];
    {   // range of the occupied buckets (the prediction below walks only that range): one pair of atomics per wave, from
        // its first and last thread with a non-empty run of buckets (a thousand threads on one LDS word take turns)
        const uint64_t occ = __ballot(sum != 0u);
        if (occ) {
            const int first = __builtin_ctzll(occ), last = 63 - __builtin_clzll(occ);
            const int l = (int)lane_id();
            if (l == last) atomicMin(&s_bmin, (uint32_t)(NB1 - 16 - tid * 16));   // buckets descend with the thread index
            if (l == first) atomicMax(&s_bmax, (uint32_t)(NB1 - 1 - tid * 16));
        }
    }
    uint32_t total;
    const uint32_t before = block_excl_scan<1024>(sum, s_scan, total);
    {
        uint32_t run = before;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            s_cum[NB1 - 1 - (tid * 16 + i)] = run;
            run += hv[i];
        }
    }
    const int64_t ns = total;  // sampled elements
    if (tid == 0 && exact && ns != a.d) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    if (tid <= L) {
        const int t = tid;
        const bool act = a.all_thresholds || t == 0 || t == lev - 1 || t == lev;
        s_active[t] = act;
        const int64_t kt = s_k[t];
        int64_t lo = kt, hi = kt;
        if (!exact) {
            const double m = (double)kt * (double)ns / (double)a.d;
            const double frac = 1.0 - (double)kt / (double)a.d;
            const double sd = sqrt(m * (frac > 0.0 ? frac : 0.0));
            const double zs = ns >= ZONE_BIG_SAMPLE ? ZONE_SIGMAS_BIG : ZONE_SIGMAS;
            lo = (int64_t)floor(m - zs * sd) - 2;
            hi = (int64_t)ceil(m + zs * sd) + 2;
        }
        if (lo < 1) lo = 0;            // the zone starts at the highest bucket
        if (hi > ns) hi = ns + 1;      // the zone reaches the lowest bucket
        s_lo[t] = lo;
        s_hi[t] = hi;
        s_top[t] = NB1 - 1;
        s_bot[t] = 0;
    }
    __syncthreads();
    // The bucket that holds sample rank r (counted from the top): the highest bucket b with at least r sampled
    // elements in buckets >= b.  One thread per (threshold, end of its zone), bisection over the scanned histogram;
    // r = 0 keeps the highest bucket, r > ns the lowest.
    if (tid < 2 * (L + 1) && s_active[tid >> 1]) {
        const int t = tid >> 1, which = tid & 1;
        const int64_t r = which ? s_hi[t] : s_lo[t];
        if (r >= 1 && r <= ns) {
            int lo = 0, hi = NB1 - 1;   // (elements in buckets >= lo) >= r holds throughout
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if ((int64_t)s_cum[mid] + s_h[mid] >= r) lo = mid;
                else hi = mid - 1;
            }
            if (which) s_bot[t] = (uint32_t)lo;
            else s_top[t] = (uint32_t)lo;
        }
    }
    __syncthreads();

    // Zones in descending key order, by the first wave: lane t holds what threshold t found, the uniform loop
    // fetches it with readlane, lane 0 writes.  Overlapping zones are merged.
    if (tid < 64) {
        const int tl = tid <= L ? tid : 0;
        const int my_act = s_active[tl];
        const uint32_t my_top = s_top[tl], my_bot0 = s_bot[tl];
        const uint32_t my_bot = my_bot0 < my_top ? my_bot0 : my_top;
        int nz = 0, lab = 0;
        uint32_t ztop = 0, zbot = 0;   // the open zone nz - 1
        for (int t = 0; t <= L; ++t) {
            const int act = __builtin_amdgcn_readlane(my_act, t);
            const uint32_t top = (uint32_t)__builtin_amdgcn_readlane((int)my_top, t);
            const uint32_t bot = (uint32_t)__builtin_amdgcn_readlane((int)my_bot, t);
            const int64_t kt = s_k[t];
            int tz;
            uint32_t tau = 0, jx = 0;
            bool set_thr = false;
            if (!act) {
                tz = THR_INACTIVE;
            } else if (kt <= 0) {
                tz = THR_NONE;
                tau = 0xFFFFFFFFu; jx = 0; set_thr = true;
                lab = t + 1;
            } else if (kt >= a.d) {
                tz = THR_ALL;
                tau = 0; jx = JX_ALL; set_thr = true;
            } else {
                if (nz > 0 && top >= zbot) {   // overlaps the previous zone: one zone for both
                    if (top > ztop) ztop = top;
                    if (bot < zbot) zbot = bot;
                    if (tid == 0) ri->zone_t1[nz - 1] = t;
                } else {
                    ztop = top;
                    zbot = bot;
                    if (tid == 0) {
                        ri->zone_t0[nz] = t;
                        ri->zone_t1[nz] = t;
                        s_label[nz] = lab;
                    }
                    ++nz;
                }
                if (tid == 0) { s_ztop[nz - 1] = ztop; s_zbot[nz - 1] = zbot; }
                tz = nz - 1;
                lab = t + 1;
            }
            if (tid == 0) {
                ri->thr_zone[t] = tz;
                if (set_thr) { ri->thr_tau[t] = tau; ri->thr_jx[t] = jx; }
            }
        }
        if (tid == 0) s_label[nz] = lab;
        wave_lds_sync();
        // candidate list layout: lane z sizes zone z, then the offsets in order
        const uint64_t S = exact ? 1ull : (1ull << a.sample_shift);
        uint32_t ltop = 0, lbot = 0;
        uint64_t mycap = 0;
        if (tid < nz) {
            ltop = s_ztop[tid];
            lbot = s_zbot[tid];
            const uint64_t c = (uint64_t)s_cum[lbot] + s_h[lbot] - s_cum[ltop];
            mycap = exact ? c : S * (c + (uint64_t)(8.0 * sqrt((double)c)) + 16);
        }
        uint64_t off = 0;
        for (int z = 0; z < nz; ++z) {
            uint64_t cap = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(mycap >> 32), z) << 32) |
                           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)mycap, z);
            if (off + cap > (uint64_t)a.d) cap = (uint64_t)a.d - off;
            if (tid == z) {
                ri->zone_top[z] = ltop;
                ri->zone_bot[z] = lbot;
                ri->zone_off[z] = (uint32_t)off;
                ri->zone_cap[z] = (uint32_t)cap;
            }
            off += cap;
        }
        if (tid <= nz) ri->region_label[tid] = s_label[tid];
        if (tid == 0) {
            ri->n_zones = nz;
            s_nz = nz;
        }
    }
    __syncthreads();

    // Which band will the message hold besides the base band?  With p known the level is already drawn.  With
    // adaptive p it is predicted: band energies estimated from the histogram (bucket count x squared bucket
    // midpoint), the same Philox word, the same inverse CDF.  The selection read stages the members of that band
    // so that the message can be assembled without a second read of the row; a wrong prediction only costs
    // that second read.
    const int nz = s_nz;
    if (a.all_thresholds && a.draw_mode == 3) {
        for (int l = tid; l < LMAX + 2; l += 1024) s_est[l] = 0.0f;
        __syncthreads();
        {
            // strided over the occupied range of buckets, so that the occupied ones (a few hundred in a row) spread
            // over the threads
            const double scale = (double)a.d / (double)(ns > 0 ? ns : 1);
            const int b1 = (int)s_bmax;
            for (int b = (int)s_bmin + tid; b <= b1; b += 1024) {
                const uint32_t h = s_h[b];
                if (h == 0 || (b >> 6) >= 255) continue;
                const double rank = ((double)s_cum[b] + 0.5 * (double)h) * scale;
                int band = 0;
                while (band <= L && rank >= s_kd[band]) ++band;   // first t with rank < k_t
                const double v = (double)__uint_as_float(((uint32_t)b << B1_SHIFT) | 0x10000u);
                atomicAdd(&s_est[band], (float)((double)h * scale * v * v));   // fp32: a native LDS atomic, ample for a prediction
            }
        }
        __syncthreads();
        if (tid < L) s_p[tid] = sqrt((double)s_est[tid + 1]);   // the square roots side by side, the rest in order
        __syncthreads();
        if (tid == 0) {
            double* p = s_p;
            double tot = 0.0;
            for (int l = 0; l < L; ++l) tot += p[l];
            for (int l = 0; l < L; ++l) p[l] = tot > 0.0 ? p[l] / tot : 1.0 / (double)L;
            s_lev = draw_from_p(p, L, philox_word0(a.seed, a.step, (uint32_t)row));
        }
        __syncthreads();
    }
    if (tid == 0) {
        int sl = ((a.all_thresholds && a.draw_mode != 3) || !a.staging) ? 0 : s_lev;   // norms only: nothing to stage
        // a wide band is cheaper to collect by a second read: the staged lists of such a row would keep its few
        // workgroups busy long after the other rows are done
        if (sl > 0 && (s_k[sl] - s_k[sl - 1]) * STAGE_MAX_BAND_INV > a.d) sl = 0;
        ri->spec_level = sl;
        ri->spec_ok = (sl > 0 && !(a.all_thresholds && a.draw_mode == 3)) ? 1 : 0;   // adaptive: decided after the draw
        s_lev = sl;
    }
    __syncthreads();
    const int spec = s_lev;

    // class table: thread tid writes its 16 buckets (descending), 64 bytes.  The zone bounds of the current zone
    // index stay in registers; a thread's buckets share their exponent, so their group changes only with the zone
    // index and the group tables are written once per change.
    uint32_t codes[16];
    int zi = 0;   // zones wholly above the current bucket
    uint32_t ztop_c = nz > 0 ? s_ztop[0] : 0u, zbot_c = nz > 0 ? s_zbot[0] : 0u;
    int lab_c = s_label[0];   // band of the region above zone zi (below the last zone when zi == nz)
    int last_gid = -1;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t b = (uint32_t)(NB1 - 1 - (tid * 16 + i));
        while (zi < nz && zbot_c > b) {
            ++zi;
            lab_c = s_label[zi];
            if (zi < nz) { ztop_c = s_ztop[zi]; zbot_c = s_zbot[zi]; }
        }
        if (zi < nz && b <= ztop_c) {
            codes[15 - i] = class_code((uint32_t)G_DUMMY, 64u + (uint32_t)zi, (uint32_t)zi, true);
        } else {
            const uint32_t E = b >> 6;
            const int gid = (int)(255 - E) + zi;
            if (gid != last_gid) {
                last_gid = gid;
                s_gexp[gid] = (uint16_t)(E ? E : 1);
                s_gband[gid] = (uint16_t)lab_c;
            }
            const bool member = spec > 0 && (lab_c == 0 || lab_c == spec);
            codes[15 - i] = class_code((uint32_t)gid, (uint32_t)zi, member ? TAG_MEMBER : 0u, member);
        }
    }
    {
        uint4* dst = (uint4*)(a.table + (size_t)row * NB1 + (NB1 - 16 - tid * 16));
#pragma unroll
        for (int i = 0; i < 4; ++i) dst[i] = make_uint4(codes[4 * i], codes[4 * i + 1], codes[4 * i + 2], codes[4 * i + 3]);
        // the same table in one byte per bucket (counter in bits 0..6, "stage" in bit 7), for the selection read that
        // rebuilds the rest from the key: the sum group of a region is (255 - exponent) + region, the tag of a zone its index
        uint32_t w8[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w8[i] = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t c = codes[4 * i + k];
                w8[i] |= (((c >> 6) & 0x7Fu) | ((c & CODE_STAGE) ? 0x80u : 0u)) << (8 * k);
            }
        }
        *(uint4*)(a.table8 + (size_t)row * NB1 + (NB1 - 16 - tid * 16)) = make_uint4(w8[0], w8[1], w8[2], w8[3]);
    }
    __syncthreads();
    for (int g = tid; g < GMAX; g += 1024) {
        ri->g_exp[g] = s_gexp[g];
        ri->g_band[g] = s_gband[g];
    }
}

// ---------------------------------------------------------------------------------------------------
// The selection read: region counts, group sums (SUMS), zone candidates.
constexpr int MAIN_THREADS = 1024;
constexpr int MAIN_WAVES = MAIN_THREADS / 64;

// LDS layout (bytes), all of the 160 KB.  The table sits at offset 0 so that the look-up needs no base; the sums
// at 64 KB and the counters at a multiple of 32 KB so that their bases can be OR-ed with the fields of the class
// code.  The counters exist once per count chunk of the workgroup's chunk.
constexpr int LM_TAB = 0;                                   // uint32 [NB1]
constexpr int LM_SUM = NB1 * 4;                             // uint64 [GMAX][REP_SUM]
constexpr int LM_ZCUR = LM_SUM + GMAX * REP_SUM * 8;        // uint32 [64] write cursor of every zone list
constexpr int LM_ROWMAX = LM_ZCUR + 64 * 4;                 // uint32 (16 bytes kept): largest key of the chunk
constexpr int LM_ZOFF = LM_ROWMAX + 16;                     // uint32 [64]
constexpr int LM_ZCAP = LM_ZOFF + 64 * 4;
constexpr int LM_MISC_END = LM_ZCAP + 64 * 4;
constexpr int LM_CNT = 4 * 32768;                           // uint32 [CSUB_MAX][128][REP_CNT]: regions 0..63, zones 64..127
constexpr int LM_END = LM_CNT + CSUB_MAX * 128 * REP_CNT * 4;
static_assert(LM_SUM == 65536 && LM_MISC_END <= LM_CNT && LM_CNT % 32768 == 0, "LDS layout");
static_assert(REP_SUM * 8 == 128 && REP_CNT * 4 == 64 && CSUB_MAX * 128 * REP_CNT * 4 == 32768, "field scaling of the class code");
template <bool SUMS> constexpr int lm_total() { return LM_END; }
static_assert(lm_total<true>() <= 160 * 1024, "LDS budget");
static_assert(ZMAX <= 64 && RMAX <= 64 && GMAX <= 512, "field widths of the class code");

// LOOPED: a workgroup takes the chunks blockIdx.x, blockIdx.x + gridDim.x, ... of its row.  The redo round is launched
// that way with a small grid, so that it costs little when, as nearly always, no row needs it; the first round has a
// workgroup per chunk and no loop.
template <int DT, bool VEC, bool SUMS, bool LOOPED>
__global__ __launch_bounds__(MAIN_THREADS) void k_main(TopkArgs a, int exact_pass) {
    __shared__ __align__(16) unsigned char lm[lm_total<SUMS>()];
    uint32_t* s_cnt = (uint32_t*)(lm + LM_CNT);
    uint32_t* s_zcur = (uint32_t*)(lm + LM_ZCUR);
    uint32_t* s_rowmax = (uint32_t*)(lm + LM_ROWMAX);   // largest key the workgroup met
    uint32_t* s_zoff = (uint32_t*)(lm + LM_ZOFF);
    uint32_t* s_zcap = (uint32_t*)(lm + LM_ZCAP);

    const int row = blockIdx.y, tid = threadIdx.x;
    const RowInfo* ri = a.rinfo + row;
    if (exact_pass && !ri->respec) return;
    const uint32_t lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: loop bounds and offsets stay in SGPRs
    RowAcc* ra = a.racc + row;
    const int nz = ri->n_zones;
    int chunk_id = blockIdx.x;
    do {
    if (LOOPED && chunk_id != (int)blockIdx.x) __syncthreads();   // the previous chunk is done with the shared arrays
    {
        const uint4* src = (const uint4*)(a.table + (size_t)row * NB1);
        uint4* dst = (uint4*)(lm + LM_TAB);
        for (int i = tid; i < NB1 * 4 / 16; i += MAIN_THREADS) dst[i] = src[i];
        uint4* z = (uint4*)(lm + LM_CNT);
        const uint4 zero = make_uint4(0, 0, 0, 0);
        for (int i = tid; i < (LM_END - LM_CNT) / 16; i += MAIN_THREADS) z[i] = zero;
        z = (uint4*)(lm + LM_ZCUR);
        for (int i = tid; i < (LM_ZOFF - LM_ZCUR) / 16; i += MAIN_THREADS) z[i] = zero;
        if (SUMS) {
            z = (uint4*)(lm + LM_SUM);
            for (int i = tid; i < GMAX * REP_SUM * 8 / 16; i += MAIN_THREADS) z[i] = zero;
        }
    }
    if (tid < 64) {
        s_zoff[tid] = tid < nz ? ri->zone_off[tid] : 0u;
        s_zcap[tid] = tid < nz ? ri->zone_cap[tid] : 0u;
    }
    __syncthreads();

    const int64_t c0 = (int64_t)chunk_id * a.chunk;
    const int64_t c1 = c0 + a.chunk < a.d ? c0 + a.chunk : a.d;
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    // this wave's private, worst-case sized part of the scratch list: its candidates in the order met
    // (room for twice the wave's even share of the chunk: the waves of k_main2 may take more than that share)
    uint2* priv = a.cand_priv + ((size_t)row * a.chunks_per_row + chunk_id) * (size_t)(2 * a.chunk) + (size_t)wave * (a.chunk / (MAIN_WAVES / 2));
    // per-lane byte addresses of the replicated accumulators
    const uint32_t cnt_lane = (uint32_t)LM_CNT + (lane & 15u) * 4u;
    const uint32_t sum_lane = (uint32_t)LM_SUM + (lane & 15u) * 8u;
    uint32_t head = 0;   // wave-uniform: entries staged so far
    uint32_t maxkey = 0;

    // four consecutive elements of every lane (bit c of vmask: element c is inside the chunk): table look-ups
    // first, then the accumulators (zone buckets carry a dummy group, elements past the end a dummy class, so
    // there is no branch), then the candidates
    auto lookup = [&](const uint32_t (&b)[4], uint32_t (&code)[4]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) code[c] = *(const uint32_t*)(lm + ((b[c] >> 15) & 0xFFFCu));
    };
    auto process = [&](const uint32_t (&b)[4], uint32_t (&code)[4], uint32_t rel0, uint32_t vmask, uint32_t cnt_base) {
        uint32_t anys = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (!((vmask >> c) & 1u)) code[c] = class_code((uint32_t)G_DUMMY, 63u, 0u, false);
            const uint32_t key = key_of_bits(b[c]);
            if (SUMS) {
                const uint32_t hid = (key & 0x7FFFFFu) | 0x800000u;
                const uint32_t sig = key < hid ? key : hid;   // exponent field 0: no hidden bit, sig = key
                atomicAdd((unsigned long long*)(lm + ((code[c] >> 16) | sum_lane)),
                          (unsigned long long)sig * (unsigned long long)sig);
            }
            atomicAdd((uint32_t*)(lm + ((code[c] & 0x1FC0u) | cnt_base)), 1u);
            maxkey = key > maxkey ? key : maxkey;
            anys |= code[c];
        }
        if (__ballot(anys & CODE_STAGE)) {
            const uint32_t relc = rel0 << 6;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint64_t m = __ballot(code[c] & CODE_STAGE);
                if (__builtin_amdgcn_inverse_ballot_w64(m))
                    priv[head + mbcnt(m)] = make_uint2(b[c], (relc + ((uint32_t)c << 6)) | (code[c] & 63u));
                head += (uint32_t)__popcll(m);
            }
        }
    };

    const int span = (int)(c1 - c0);
    const int tpc = a.cchunk / TILE;   // tiles per count chunk
    // the counters of the count chunk that tile t of the chunk lies in
    auto cnt_of = [&](int t) -> uint32_t {
        const uint32_t sub = (t >= tpc ? 1u : 0u) + (t >= 2 * tpc ? 1u : 0u) + (t >= 3 * tpc ? 1u : 0u);
        return cnt_lane + (a.csub > 1 ? sub : 0u) * (uint32_t)(128 * REP_CNT * 4);
    };
    uint32_t buf[8][4];
    uint32_t cc[4], cn[4];
    // Load n of a wave covers the 256 elements at c0 + (16 n + wave) * 256: the 16 waves read 16 KB side by
    // side.  Eight loads per lane stay in flight: a slot is refilled as soon as it has been processed.
    const int woff = (int)wave * 256;
    const int nfull = span >= woff + 256 ? (span - woff - 256) / 4096 + 1 : 0;   // loads with all 256 elements
    auto issue = [&](int n, uint32_t (&b)[4]) { ld.load4_stream(c0 + (int64_t)((n * 16 + (int)wave) * 256) + (int64_t)lane * 4, b); };
    auto rel_of = [&](int n) -> uint32_t { return (uint32_t)((n * 16 + (int)wave) * 256) + lane * 4; };
    // load round n covers tile n of the chunk
    // The table look-ups of the next load are issued before the accumulators of the current one are updated, so
    // that their latency is covered.
    int n = 0;
    if (nfull >= 8) {
#pragma unroll
        for (int q = 0; q < 8; ++q) issue(q, buf[q]);
        lookup(buf[0], cn);
        for (; n + 16 <= nfull; n += 8) {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
#pragma unroll
                for (int c = 0; c < 4; ++c) cc[c] = cn[c];
                lookup(buf[(q + 1) & 7], cn);   // q = 7: load n + 8, issued at q = 0 of this iteration
                process(buf[q], cc, rel_of(n + q), 15u, cnt_of(n + q));
                issue(n + q + 8, buf[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
#pragma unroll
            for (int c = 0; c < 4; ++c) cc[c] = cn[c];
            if (q < 7) lookup(buf[q + 1], cn);
            process(buf[q], cc, rel_of(n + q), 15u, cnt_of(n + q));
        }
        n += 8;
    }
    for (; n < nfull; ++n) {
        issue(n, buf[0]);
        lookup(buf[0], cc);
        process(buf[0], cc, rel_of(n), 15u, cnt_of(n));
    }
    if (c0 + (int64_t)((nfull * 16 + (int)wave) * 256) < c1) {   // the ragged end of the chunk: at most one partial load per wave
        const int64_t j = c0 + (int64_t)((nfull * 16 + (int)wave) * 256) + (int64_t)lane * 4;
        const int nv = j < c1 ? ld.load4(j, buf[0]) : 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) if (c >= nv) buf[0][c] = 0u;
        lookup(buf[0], cc);
        process(buf[0], cc, rel_of(nfull), (1u << nv) - 1u, cnt_of(nfull));
    }
    if (__ballot(maxkey >= 0x7F800000u) && lane == 0) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
    maxkey = wave_max(maxkey);
    if (lane == 0) atomicMax(s_rowmax, maxkey);

    // ---- the workgroup's candidates move from the private lists to the zones' lists: one reservation per zone.
    //      The wave's list comes back from memory while the reservations are made and the sums and counts, which
    //      need nothing from it, go out. ----
    constexpr int EP_KEEP = 16;
    uint2 ent[EP_KEEP];
    __threadfence_block();   // the wave reads back what it stored
    if (head) {   // uniform
#pragma unroll
        for (int u = 0; u < EP_KEEP; ++u) {
            const uint32_t i = lane + 64u * (uint32_t)u;
            ent[u] = priv[i < head ? i : head - 1u];
        }
    }
    if (lane == 0) a.priv_cnt[((size_t)row * a.chunks_per_row + chunk_id) * MAIN_WAVES + wave] = head;
    __syncthreads();
    if (tid < nz) {
        uint32_t total = 0;
        for (int r = 0; r < CSUB_MAX * REP_CNT; ++r)
            total += s_cnt[(r / REP_CNT) * (128 * REP_CNT) + (64 + tid) * REP_CNT + ((r + tid) & (REP_CNT - 1))];
        s_zcur[tid] = total ? atomicAdd(&ra->zone_fill[tid], total) : 0u;
    }
    if (tid == 64) atomicMax(&ra->rowmax_key, s_rowmax[0]);
    if (SUMS && tid >= 64) {   // the waves after the first: the first is waiting for its reservations
        const unsigned long long* s_sum = (const unsigned long long*)(lm + LM_SUM);
        for (int g = tid - 64; g < G_DUMMY; g += MAIN_THREADS - 64) {
            unsigned long long lo = 0, hi = 0;
#pragma unroll
            for (int r = 0; r < REP_SUM; ++r) {
                const unsigned long long v = s_sum[g * REP_SUM + ((r + tid) & (REP_SUM - 1))];
                lo += v & 0xFFFFFFFFull;
                hi += v >> 32;
            }
            if (lo) atomicAdd((unsigned long long*)&ra->gsum[g][0], lo);
            if (hi) atomicAdd((unsigned long long*)&ra->gsum[g][1], hi);
        }
    }
    if (tid >= MAIN_THREADS - RMAX * CSUB_MAX) {   // per count chunk: the counters of region t % RMAX (the last waves)
        const int t = tid - (MAIN_THREADS - RMAX * CSUB_MAX);
        const int r = t % RMAX, sub = t / RMAX;
        uint32_t cnt = 0;
        for (int k = 0; k < REP_CNT; ++k) cnt += s_cnt[sub * (128 * REP_CNT) + r * REP_CNT + ((k + t) & (REP_CNT - 1))];
        const int64_t cc = (int64_t)chunk_id * a.csub + sub;
        if (sub < a.csub && cc < a.cchunks_per_row) a.chunk_cnt[((size_t)row * RMAX + r) * a.cchunks_per_row + cc] = cnt;
        if (cnt) atomicAdd(&ra->region_cnt[r], cnt);
    }
    __syncthreads();
    uint2* cl = a.cand + (size_t)row * (size_t)a.d;
    bool dropped = false;
    auto move = [&](uint2 e) {
        const uint32_t z = e.y & 63u;
        if (z == TAG_MEMBER) return;   // staged for the message only
        const uint32_t pos = atomicAdd(&s_zcur[z], 1u);
        if (pos < s_zcap[z]) {
            cl[(size_t)s_zoff[z] + pos] = make_uint2(e.x, (uint32_t)c0 + (e.y >> 6));
        } else {
            dropped = true;
        }
    };
    if (head) {
#pragma unroll
        for (int u = 0; u < EP_KEEP; ++u)
            if (lane + 64u * (uint32_t)u < head) move(ent[u]);
    }
    batched_loop<16, 64>(64u * EP_KEEP, head, lane, [&](uint32_t i) { return priv[i]; }, [&](uint32_t, uint2 e) { move(e); });
    if (__ballot(dropped) && lane == 0) {
        // a candidate list overflowed its estimated capacity: redo the row exactly (exact capacities cannot overflow)
        if (ri->exact) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        else atomicOr((int32_t*)&a.rinfo[row].respec, 1);
    }
    } while (LOOPED && (chunk_id += (int)gridDim.x) < a.chunks_per_row);
}

// ---------------------------------------------------------------------------------------------------
constexpr int MAIN_GROUP = 2048;   // elements a wave takes at a time: its eight loads in flight
// The selection read with two workgroups per CU (plans whose chunks have four count chunks): a chunk is read by two
// workgroups of 512 threads, two count chunks each, so that the table load, the flush and the move of the candidates of
// one workgroup run beside the streaming of the other (with one workgroup per CU they overlap nothing: a tenth to a
// quarter of its time).  What makes two fit: the class table in one byte per bucket (16 KB instead of 64: the sum
// group and the tag follow from the key and the counter), counters for two count chunks.  Everything the workgroup
// writes has the layout of k_main: sixteen private lists per chunk (this workgroup's eight waves use lists 8 h .. 8 h + 7),
// entries {bits, offset in the CHUNK << 6 | tag}, counts per count chunk.
// The waves take their workgroup's elements in groups of MAIN_GROUP consecutive ones handed out by an LDS counter, not in
// fixed interleaved shares: the waves of a SIMD are served oldest first, so with fixed shares the oldest is done when the
// youngest still has a third of its share left and the workgroup ends at a fraction of its wave slots; with the counter
// all waves end within one group of each other.
constexpr int M2_THREADS = 512;
constexpr int M2_WAVES = M2_THREADS / 64;
constexpr int M2_CSUB = 2;                                   // count chunks per workgroup
constexpr int M2_TAB = 0;                                    // uint8 [NB1]
constexpr int M2_SUM = NB1;                                  // uint64 [GMAX][REP_SUM]
constexpr int M2_ZCUR = M2_SUM + GMAX * REP_SUM * 8;         // uint32 [64]
constexpr int M2_ROWMAX = M2_ZCUR + 64 * 4;                  // uint32 largest key, uint32 (at + 8) group counter
constexpr int M2_ZOFF = M2_ROWMAX + 16;
constexpr int M2_ZCAP = M2_ZOFF + 64 * 4;
constexpr int M2_MISC_END = M2_ZCAP + 64 * 4;
constexpr int M2_CNT = 56 * 1024;                            // uint32 [M2_CSUB][128][REP_CNT]
constexpr int M2_END = M2_CNT + M2_CSUB * 128 * REP_CNT * 4;
static_assert(M2_MISC_END <= M2_CNT && 2 * M2_END <= 160 * 1024 && M2_SUM % 16 == 0 && M2_ZCUR % 16 == 0, "LDS layout: two workgroups per CU");

template <int DT, bool VEC, bool SUMS>
__global__ __launch_bounds__(M2_THREADS, 4) void k_main2(TopkArgs a) {
    __shared__ __align__(16) unsigned char lm[M2_END];
    uint32_t* s_cnt = (uint32_t*)(lm + M2_CNT);
    uint32_t* s_zcur = (uint32_t*)(lm + M2_ZCUR);
    uint32_t* s_rowmax = (uint32_t*)(lm + M2_ROWMAX);
    uint32_t* s_next = (uint32_t*)(lm + M2_ROWMAX + 8);
    uint32_t* s_zoff = (uint32_t*)(lm + M2_ZOFF);
    uint32_t* s_zcap = (uint32_t*)(lm + M2_ZCAP);

    const int row = blockIdx.y, tid = threadIdx.x;
    const RowInfo* ri = a.rinfo + row;
    const uint32_t lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    RowAcc* ra = a.racc + row;
    const int nz = ri->n_zones;
    const int chunk_id = blockIdx.x >> 1, half = blockIdx.x & 1;
    {
        const uint4* src = (const uint4*)(a.table8 + (size_t)row * NB1);
        uint4* dst = (uint4*)(lm + M2_TAB);
        for (int i = tid; i < NB1 / 16; i += M2_THREADS) dst[i] = src[i];
        const uint4 zero = make_uint4(0, 0, 0, 0);
        uint4* z = (uint4*)(lm + M2_CNT);
        for (int i = tid; i < (M2_END - M2_CNT) / 16; i += M2_THREADS) z[i] = zero;
        z = (uint4*)(lm + M2_ZCUR);
        for (int i = tid; i < (M2_ZOFF - M2_ZCUR) / 16; i += M2_THREADS) z[i] = zero;
        if (SUMS) {
            z = (uint4*)(lm + M2_SUM);
            for (int i = tid; i < GMAX * REP_SUM * 8 / 16; i += M2_THREADS) z[i] = zero;
        }
    }
    if (tid < 64) {
        s_zoff[tid] = tid < nz ? ri->zone_off[tid] : 0u;
        s_zcap[tid] = tid < nz ? ri->zone_cap[tid] : 0u;
    }
    __syncthreads();

    const int hlen = a.chunk / 2;   // elements of a workgroup: two count chunks
    const int64_t cbase = (int64_t)chunk_id * a.chunk;
    const int64_t c0 = cbase + (int64_t)half * hlen;
    const int64_t c1 = c0 + hlen < a.d ? c0 + hlen : a.d;
    const int span = c1 > c0 ? (int)(c1 - c0) : 0;   // the second half of a row's last chunk may be empty
    const uint32_t relh = (uint32_t)(half * hlen);   // offsets in the entries count from the start of the chunk
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    uint2* priv = a.cand_priv + ((size_t)row * a.chunks_per_row + chunk_id) * (size_t)(2 * a.chunk) +
                  (size_t)(half * M2_WAVES + (int)wave) * (a.chunk / 8);
    const uint32_t cnt_lane = (uint32_t)M2_CNT + (lane & 15u) * 4u;
    const uint32_t sum_lane = (uint32_t)M2_SUM + (lane & 15u) * 8u;
    uint32_t head = 0;
    uint32_t maxkey = 0;

    auto lookup = [&](const uint32_t (&b)[4], uint32_t (&code)[4]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) code[c] = lm[(b[c] >> B1_SHIFT) & (uint32_t)(NB1 - 1)];
    };
    auto process = [&](const uint32_t (&b)[4], uint32_t (&code)[4], uint32_t rel0, uint32_t vmask, uint32_t cnt_base) {
        uint32_t anys = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (!((vmask >> c) & 1u)) code[c] = 0x7Fu;   // past the end: an unused zone's counter, the dummy group, not staged
            const uint32_t key = key_of_bits(b[c]);
            const uint32_t cnt7 = code[c] & 0x7Fu;
            if (SUMS) {
                const uint32_t hid = (key & 0x7FFFFFu) | 0x800000u;
                const uint32_t sig = key < hid ? key : hid;   // exponent field 0: no hidden bit, sig = key
                const uint32_t gid = cnt7 < 64u ? 255u - (key >> 23) + cnt7 : (uint32_t)G_DUMMY;
                atomicAdd((unsigned long long*)(lm + (gid * (uint32_t)(REP_SUM * 8) + sum_lane)),
                          (unsigned long long)sig * (unsigned long long)sig);
            }
            atomicAdd((uint32_t*)(lm + (cnt7 * (uint32_t)(REP_CNT * 4) + cnt_base)), 1u);
            maxkey = key > maxkey ? key : maxkey;
            anys |= code[c];
        }
        if (__ballot(anys & 0x80u)) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint64_t m = __ballot(code[c] & 0x80u);
                if (__builtin_amdgcn_inverse_ballot_w64(m)) {
                    const uint32_t cnt7 = code[c] & 0x7Fu;
                    const uint32_t tag = cnt7 >= 64u ? cnt7 & 63u : TAG_MEMBER;
                    priv[head + mbcnt(m)] = make_uint2(b[c], ((rel0 + (uint32_t)c) << 6) | tag);
                }
                head += (uint32_t)__popcll(m);
            }
        }
    };

    const int tpc = a.cchunk / TILE;   // tiles per count chunk
    auto cnt_of = [&](int t) -> uint32_t { return cnt_lane + (t >= tpc ? 1u : 0u) * (uint32_t)(128 * REP_CNT * 4); };
    uint32_t buf[8][4];
    uint32_t cc[4], cn[4];
    {
        // Groups of MAIN_GROUP elements from the counter; a wave holds the group it works on and the next one, whose
        // loads refill the ring as those of the current one are consumed (no condition on a load of the steady-state
        // loop, so that the waits can count them).  A wave takes at most gmax groups, which with one piece of the ragged
        // end is what its private list has room for; together the waves have room for twice their elements.
        const int ngroups = span / MAIN_GROUP;
        const int gmax = (a.chunk / 8 - 256) / MAIN_GROUP;
        int taken = 0;
        auto grab = [&]() -> int {   // uniform
            if (taken >= gmax) return -1;
            uint32_t v = 0;
            if (lane == 0) v = atomicAdd(s_next, 1u);
            const int g = __builtin_amdgcn_readfirstlane((int)v);
            if (g >= ngroups) return -1;
            ++taken;
            return g;
        };
        auto gissue = [&](int g, int q, uint32_t (&b)[4]) { ld.load4_stream(c0 + (int64_t)(g * MAIN_GROUP + q * 256) + (int64_t)lane * 4, b); };
        int gc = grab(), gn = gc >= 0 ? grab() : -1;
        if (gc >= 0) {
#pragma unroll
            for (int q = 0; q < 8; ++q) gissue(gc, q, buf[q]);
            lookup(buf[0], cn);
            while (gn >= 0) {   // uniform
                const uint32_t cb = cnt_of(gc / (TILE / MAIN_GROUP));
                const uint32_t rel0 = relh + (uint32_t)(gc * MAIN_GROUP) + lane * 4;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) cc[c] = cn[c];
                    lookup(buf[(q + 1) & 7], cn);
                    process(buf[q], cc, rel0 + (uint32_t)(q * 256), 15u, cb);
                    gissue(gn, q, buf[q]);
                }
                gc = gn;
                gn = grab();
            }
            {
                const uint32_t cb = cnt_of(gc / (TILE / MAIN_GROUP));
                const uint32_t rel0 = relh + (uint32_t)(gc * MAIN_GROUP) + lane * 4;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) cc[c] = cn[c];
                    if (q < 7) lookup(buf[q + 1], cn);
                    process(buf[q], cc, rel0 + (uint32_t)(q * 256), 15u, cb);
                }
            }
        }
        const int tbase = ngroups * MAIN_GROUP;   // up to eight pieces of 256 elements are left, the last one ragged: wave w takes piece w
        if (tbase + (int)wave * 256 < span) {
            const int pos = tbase + (int)wave * 256;
            const int64_t j = c0 + pos + (int64_t)lane * 4;
            const int nv = j < c1 ? ld.load4(j, buf[0]) : 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) if (c >= nv) buf[0][c] = 0u;
            lookup(buf[0], cc);
            process(buf[0], cc, relh + (uint32_t)pos + lane * 4, (1u << nv) - 1u, cnt_of(pos / TILE));
        }
    }
    if (__ballot(maxkey >= 0x7F800000u) && lane == 0) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
    maxkey = wave_max(maxkey);
    if (lane == 0) atomicMax(s_rowmax, maxkey);

    // ---- flush and move, as in k_main ----
    constexpr int EP_KEEP = 16;
    uint2 ent[EP_KEEP];
    __threadfence_block();
    if (head) {   // uniform
#pragma unroll
        for (int u = 0; u < EP_KEEP; ++u) {
            const uint32_t i = lane + 64u * (uint32_t)u;
            ent[u] = priv[i < head ? i : head - 1u];
        }
    }
    if (lane == 0) a.priv_cnt[((size_t)row * a.chunks_per_row + chunk_id) * MAIN_WAVES + half * M2_WAVES + wave] = head;
    __syncthreads();
    if (tid < nz) {
        uint32_t total = 0;
        for (int r = 0; r < M2_CSUB * REP_CNT; ++r)
            total += s_cnt[(r / REP_CNT) * (128 * REP_CNT) + (64 + tid) * REP_CNT + ((r + tid) & (REP_CNT - 1))];
        s_zcur[tid] = total ? atomicAdd(&ra->zone_fill[tid], total) : 0u;
    }
    if (tid == 64) atomicMax(&ra->rowmax_key, s_rowmax[0]);
    if (SUMS && tid >= 64) {
        const unsigned long long* s_sum = (const unsigned long long*)(lm + M2_SUM);
        for (int g = tid - 64; g < G_DUMMY; g += M2_THREADS - 64) {
            unsigned long long lo = 0, hi = 0;
#pragma unroll
            for (int r = 0; r < REP_SUM; ++r) {
                const unsigned long long v = s_sum[g * REP_SUM + ((r + tid) & (REP_SUM - 1))];
                lo += v & 0xFFFFFFFFull;
                hi += v >> 32;
            }
            if (lo) atomicAdd((unsigned long long*)&ra->gsum[g][0], lo);
            if (hi) atomicAdd((unsigned long long*)&ra->gsum[g][1], hi);
        }
    }
    if (tid >= M2_THREADS - RMAX * M2_CSUB) {   // per count chunk: the counters of region t % RMAX
        const int t = tid - (M2_THREADS - RMAX * M2_CSUB);
        const int r = t % RMAX, sub = t / RMAX;
        uint32_t cnt = 0;
        for (int k = 0; k < REP_CNT; ++k) cnt += s_cnt[sub * (128 * REP_CNT) + r * REP_CNT + ((k + t) & (REP_CNT - 1))];
        const int64_t ccx = (int64_t)chunk_id * 4 + half * M2_CSUB + sub;
        if (ccx < a.cchunks_per_row) a.chunk_cnt[((size_t)row * RMAX + r) * a.cchunks_per_row + ccx] = cnt;
        if (cnt) atomicAdd(&ra->region_cnt[r], cnt);
    }
    __syncthreads();
    uint2* cl = a.cand + (size_t)row * (size_t)a.d;
    bool dropped = false;
    auto move = [&](uint2 e) {
        const uint32_t z = e.y & 63u;
        if (z == TAG_MEMBER) return;   // staged for the message only
        const uint32_t pos = atomicAdd(&s_zcur[z], 1u);
        if (pos < s_zcap[z]) {
            cl[(size_t)s_zoff[z] + pos] = make_uint2(e.x, (uint32_t)cbase + (e.y >> 6));
        } else {
            dropped = true;
        }
    };
    if (head) {
#pragma unroll
        for (int u = 0; u < EP_KEEP; ++u)
            if (lane + 64u * (uint32_t)u < head) move(ent[u]);
    }
    batched_loop<16, 64>(64u * EP_KEEP, head, lane, [&](uint32_t i) { return priv[i]; }, [&](uint32_t, uint2 e) { move(e); });
    if (__ballot(dropped) && lane == 0) {
        if (ri->exact) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        else atomicOr((int32_t*)&a.rinfo[row].respec, 1);
    }
}

// ---------------------------------------------------------------------------------------------------
// One workgroup per (zone, row): resolve every threshold of the zone on its candidate list.
constexpr int FN_THREADS = 1024;

// Descending search in a histogram held by one wave: lane l owns bins [BPL*l, BPL*l + BPL).  For the 1-based
// rank r (counted from the top bin) returns the bin that contains it, the rank inside that bin, and the bin count.
template <int BPL>
__device__ __forceinline__ void wave_rank_search(const uint32_t* h, uint32_t r, int& bin, uint32_t& rin, uint32_t& cnt) {
    const uint32_t lane = lane_id();
    uint32_t v[BPL];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < BPL; ++i) { v[i] = h[BPL * lane + i]; sum += v[i]; }
    // suffix sums: elements in bins above this lane's bins = total - inclusive prefix
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t u = __shfl_up(inc, o, 64);
        if (lane >= (uint32_t)o) inc += u;
    }
    const uint32_t total = __shfl(inc, 63, 64);
    uint32_t above = total - inc;  // count in bins of higher lanes
    int fb = -1;
    uint32_t fr = 0, fc = 0;
#pragma unroll
    for (int i = BPL - 1; i >= 0; --i) {
        if (fb < 0 && above < r && r <= above + v[i]) { fb = BPL * (int)lane + i; fr = r - above; fc = v[i]; }
        above += v[i];
    }
    uint64_t m = __ballot(fb >= 0);
    int src = m ? (int)__builtin_ctzll(m) : 0;
    bin = __shfl(fb, src, 64);
    rin = __shfl(fr, src, 64);
    cnt = __shfl(fc, src, 64);
    if (!m) { bin = 0; rin = r; cnt = 0; }
}

constexpr int ZC_CAP = 8192;         // (parts of the zone) x (chunks of the row) counters

// A zone's candidate list is split over up to a.fin_slices workgroups, a.fin_slice candidates or more each.
__device__ __forceinline__ int finish_slices(const TopkArgs& a, uint32_t n) {
    const uint32_t s = (n + (uint32_t)a.fin_slice - 1u) / (uint32_t)a.fin_slice;
    return s < 1u ? 1 : (s > (uint32_t)a.fin_slices ? a.fin_slices : (int)s);
}
// Key range of a zone: its buckets, cut at the largest key of the row (the top zone of a small sample reaches up to
// the highest bucket, which would otherwise stretch the zone over every exponent above the data).
__device__ __forceinline__ void zone_key_range(const RowInfo* ri, const RowAcc* ra, int z, uint32_t& kmin, uint32_t& kmax) {
    kmin = ri->zone_bot[z] << B1_SHIFT;
    kmax = ((ri->zone_top[z] + 1u) << B1_SHIFT) - 1u;
    const uint32_t rmax = ra->rowmax_key;
    if (kmax > rmax) kmax = rmax;
}
// Key range of a zone -> shift of the zone-relative histogram.
__device__ __forceinline__ int finish_shift(uint32_t kmin, uint32_t kmax) {
    const uint32_t range = kmax - kmin;
    return range < (uint32_t)FH_BINS ? 0 : (32 - __clz(range)) - 11;   // (range >> shift) < FH_BINS
}

// The work of the finish kernels is a list of items (zone, slice) per row; the workgroups of a row take them in
// turn.  Fills s_fill / s_rcnt (zone list lengths, region counts) and s_first (first item of every zone).
__device__ __forceinline__ int finish_items(const TopkArgs& a, const RowInfo* ri, const RowAcc* ra, bool sliced, uint32_t* s_fill,
                                            uint32_t* s_rcnt, int32_t* s_first) {
    const int tid = threadIdx.x, nz = ri->n_zones;
    if (tid < nz) s_fill[tid] = ra->zone_fill[tid];
    if (tid >= 64 && tid - 64 <= nz) s_rcnt[tid - 64] = ra->region_cnt[tid - 64];
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int z = 0; z < nz; ++z) {
            s_first[z] = run;
            run += sliced ? finish_slices(a, s_fill[z]) : 1;
        }
        s_first[nz] = run;
    }
    __syncthreads();
    return s_first[nz];
}

// Ranking by counting in LDS for a workgroup of FN_THREADS threads and n <= 2 * FN_THREADS distinct values v[0..n)
// (16-byte aligned): r0 / r1 = how many values are greater than v[t] / v[t + FN_THREADS].  Every thread walks the
// whole list once for both of its values, two list entries per (broadcast) LDS read.
__device__ __forceinline__ void count_greater2(const unsigned long long* v, uint32_t n, uint32_t t, uint32_t& r0, uint32_t& r1) {
    const unsigned long long c0 = t < n ? v[t] : ~0ull;
    const unsigned long long c1 = t + (uint32_t)FN_THREADS < n ? v[t + (uint32_t)FN_THREADS] : ~0ull;
    r0 = 0;
    r1 = 0;
    const ulonglong2* v2 = (const ulonglong2*)v;
    const uint32_t n2 = n >> 1;
    if (t >= n) return;   // waves past the end of the list do not load the LDS pipe
    if (n <= (uint32_t)FN_THREADS) {   // uniform: one value per thread
#pragma unroll 8
        for (uint32_t f = 0; f < n; ++f) r0 += v[f] > c0 ? 1u : 0u;
        return;
    }
#pragma unroll 8
    for (uint32_t f = 0; f < n2; ++f) {
        const ulonglong2 x = v2[f];
        r0 += (x.x > c0 ? 1u : 0u) + (x.y > c0 ? 1u : 0u);
        r1 += (x.x > c1 ? 1u : 0u) + (x.y > c1 ? 1u : 0u);
    }
    if (n & 1u) {
        const unsigned long long x = v[n - 1u];
        r0 += x > c0 ? 1u : 0u;
        r1 += x > c1 ? 1u : 0u;
    }
}

// Bitonic sort in LDS, descending, of n values (n a power of two, at most 2 * FN_THREADS) by a whole workgroup: a thread
// takes one compare-exchange per stage.  (Ranking by counting costs n broadcast reads per thread, which the LDS serves no
// faster than distinct ones: at 2048 values it took ten times as long.)
__device__ __forceinline__ void bitonic_sort_desc(unsigned long long* v, uint32_t n, uint32_t t) {
    __syncthreads();   // the values were written by other waves
    for (uint32_t k = 2; k <= n; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            // With a stride below 64 the pairs of a wave's 64 threads lie inside the wave's own 128 values: such a stage
            // needs the other waves only if the stage before it had a longer stride.
            if (j >= 64u || (j == 32u && k >= 128u)) __syncthreads();
            else wave_lds_sync();
            if (t < (n >> 1)) {
                const uint32_t i = ((t & ~(j - 1u)) << 1) | (t & (j - 1u));   // bit j clear
                const uint32_t l = i | j;
                const unsigned long long x = v[i], y = v[l];
                const bool desc = (i & k) == 0u;
                if ((x < y) == desc) { v[i] = y; v[l] = x; }
            }
        }
    }
    __syncthreads();
}

// Read 1 of a candidate list, one item per (zone, slice): histogram of (key - kmin) >> shift.
__global__ __launch_bounds__(FN_THREADS) void k_fhist(TopkArgs a, int exact_pass) {
    // four lane-interleaved copies: keys with few distinct values (16-bit inputs) put many lanes on one bin, and LDS
    // atomics of many lanes on one word take a turn each
    __shared__ uint32_t s_fh[4 * FH_BINS];
    __shared__ uint32_t s_fill[ZMAX], s_rcnt[RMAX];
    __shared__ int32_t s_first[ZMAX + 1];
    const int row = blockIdx.y, tid = threadIdx.x;
    const RowInfo* ri = a.rinfo + row;
    const RowAcc* ra = a.racc + row;
    if (exact_pass && !ri->respec) return;
    if (!exact_pass && ri->respec) return;
    const int nz = ri->n_zones;
    const int nitems = finish_items(a, ri, ra, true, s_fill, s_rcnt, s_first);
    for (int item = blockIdx.x; item < nitems; item += gridDim.x) {
        int z = 0;
        while (z + 1 < nz && s_first[z + 1] <= item) ++z;
        const int slice = item - s_first[z];
        if (slice == 0) {   // what the sliced launch accumulates for a zone with massive ties: index histogram, key range
            uint32_t* zi = (uint32_t*)(a.zcol + ((size_t)row * ZMAX + z) * COLLECT_CAP);
            for (int i = tid; i < FH_BINS + 2; i += FN_THREADS) zi[i] = 0;
        }
        const uint32_t n = s_fill[z];
        if (n == 0 || n > ri->zone_cap[z]) continue;   // the finish kernel reports it
        const int S = finish_slices(a, n);
        uint32_t kmin, kmax;
        zone_key_range(ri, ra, z, kmin, kmax);
        if (kmin > kmax) continue;
        const int sh = finish_shift(kmin, kmax);
        const uint2* kl = a.cand + (size_t)row * (size_t)a.d + ri->zone_off[z];
        const uint32_t per = (n + S - 1) / S;
        const uint32_t i0 = (uint32_t)slice * per, i1 = i0 + per < n ? i0 + per : n;
        __syncthreads();
        for (int i = tid; i < 4 * FH_BINS; i += FN_THREADS) s_fh[i] = 0;
        __syncthreads();
        batched_loop<8, FN_THREADS>(i0, i1, (uint32_t)tid, [&](uint32_t i) { return kl[i].x; }, [&](uint32_t, uint32_t bits) {
            const uint32_t b = (key_of_bits(bits) - kmin) >> sh;
            atomicAdd(&s_fh[((b < (uint32_t)FH_BINS ? b : (uint32_t)FH_BINS - 1) << 2) | (lane_id() & 3u)], 1u);
        });
        __syncthreads();
        uint32_t* zh = a.zhist + ((size_t)row * ZMAX + z) * FH_BINS;
        for (int i = tid; i < FH_BINS; i += FN_THREADS) {
            const uint32_t v = s_fh[4 * i] + s_fh[4 * i + 1] + s_fh[4 * i + 2] + s_fh[4 * i + 3];
            if (v) atomicAdd(&zh[i], v);
        }
    }
}

// Read 2, one workgroup per (slice, zone, row): from the zone's histogram the bin of every threshold; the
// candidates of those bins are gathered (a few hundred) and ranked by the workgroup that finishes last, every other
// candidate is classified by its bin: per-chunk counts of the zone's parts and exact sums per (part, exponent).
// When a threshold bin is too full to rank in LDS (massive ties) slice 0 resolves the zone alone by radix select.
constexpr int ZC0_CAP = 8192;        // the sliced pass takes zones whose (parts x chunks) counters fit this

template <bool SUMS, int PHASE>
__global__ __launch_bounds__(FN_THREADS, PHASE == 0 ? 8 : 4) void k_finish(TopkArgs a, int exact_pass) {
    // phase 0 (many workgroups per zone) keeps its LDS small so that several workgroups share a CU
    constexpr int UN_WORDS = PHASE == 0 ? COLLECT_CAP * 2 : TMAX * 256;
    constexpr int ZC = PHASE == 0 ? ZC0_CAP : ZC_CAP;
    constexpr int PREP = PHASE == 0 ? 8 : REP;   // lane replicas of the part sum accumulators
    __shared__ __align__(16) uint32_t s_un[UN_WORDS];   // slow path: digit histograms; else: candidates of the threshold bins
    __shared__ uint32_t s_fh[FH_BINS];
    __shared__ uint8_t s_bincls[FH_BINS];
    __shared__ uint32_t s_zc[ZC];
    __shared__ unsigned long long s_pacc[SUMS ? PIECE_CLASSES * PREP : 1][2];
    __shared__ int32_t s_n, s_ok, s_nsub, s_any, s_fast;
    __shared__ int32_t s_t[TMAX], s_sub[TMAX];
    __shared__ uint32_t s_res[TMAX], s_pfx[TMAX], s_tau[TMAX], s_q[TMAX], s_eq[TMAX], s_jx[TMAX];
    __shared__ uint32_t s_subpfx[TMAX], s_subtau[TMAX];
    __shared__ uint32_t s_bin[TMAX], s_rin[TMAX], s_bcnt[TMAX], s_pos[TMAX];
    __shared__ uint32_t s_ncollect;
    uint32_t (*s_hist)[256] = (uint32_t(*)[256])s_un;
    unsigned long long* s_col = (unsigned long long*)s_un;    // [COLLECT_CAP] as collected
    unsigned long long* s_srt = s_col + COLLECT_CAP;          // [COLLECT_CAP] in descending order (phase 1)
    static_assert(PHASE == 0 || sizeof(s_un) >= 2 * COLLECT_CAP * sizeof(unsigned long long), "candidate buffers must fit");

    __shared__ uint32_t s_fill[ZMAX], s_rcnt[RMAX];
    __shared__ int32_t s_first[ZMAX + 1];
    const int row = blockIdx.y, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6), lrep = lane & (uint32_t)(PREP - 1);
    RowInfo* ri = a.rinfo + row;
    RowAcc* ra = a.racc + row;
    if (exact_pass && !ri->respec) return;
    if (!exact_pass && ri->respec) return;   // already refuted (candidate overflow): the row is redone anyway
    const int L = a.L;
    const int nzones = ri->n_zones;
    const int fail_bit = ri->exact ? 1 : 0;   // what a refuted check means: 1 internal error, 0 redo the row
    auto fail = [&]() {   // called by one thread
        if (fail_bit) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        else atomicOr((int32_t*)&ri->respec, 1);
    };
    const int nitems = finish_items(a, ri, ra, PHASE == 0, s_fill, s_rcnt, s_first);

    auto run_item = [&](const int z, const int slice) {
    const uint32_t n = s_fill[z];
    const int S = finish_slices(a, n);
    const uint2* kl = a.cand + (size_t)row * (size_t)a.d + ri->zone_off[z];   // {bits, index}

    if (tid == 0) {
        // elements strictly above the zone: regions 0..z and zones 0..z-1
        int64_t above = 0;
        for (int i = 0; i <= z; ++i) above += s_rcnt[i];
        for (int i = 0; i < z; ++i) above += s_fill[i];
        bool ok = n <= ri->zone_cap[z];
        int m = 0;
        for (int t = ri->zone_t0[z]; t <= ri->zone_t1[z] && t <= L; ++t) {
            if (ri->thr_zone[t] != z) continue;
            const int64_t r = a.k[t] - above;
            if (r < 1 || r > (int64_t)n) ok = false;
            s_t[m] = t;
            s_res[m] = (uint32_t)(r > 0 ? r : 1);
            s_pfx[m] = 0;
            ++m;
        }
        if (z == nzones - 1) {   // the last zone also checks that nothing was lost
            int64_t tot = above + n + s_rcnt[z + 1];
            if (tot != a.d) ok = false;
        }
        if (m == 0) ok = false;
        if (!ok && slice == 0) fail();
        s_n = m;
        s_ok = ok ? 1 : 0;
    }
    __syncthreads();
    if (!s_ok) return;
    const int nthr = s_n;
    const int nparts = nthr + 1;
    const int nchunks = a.cchunks_per_row;   // count chunks
    const bool count_fits = nparts * nchunks <= ZC;
    // Neighbours in a candidate list mostly come from the same chunk, and 64 lanes adding to one LDS word take 64
    // turns: the counters are kept in as many lane-interleaved copies (1, 2, 4 or 8) as the LDS array holds.
    const int zrep_shift = nparts * nchunks * 8 <= ZC ? 3 : nparts * nchunks * 4 <= ZC ? 2 : nparts * nchunks * 2 <= ZC ? 1 : 0;
    const uint32_t zrep_lane = lane & ((1u << zrep_shift) - 1u);
    const uint32_t cmagic = (uint32_t)(0x100000000ull / (uint32_t)(a.cchunk >> 12)) + 1u;   // count chunk = multiple of 4096, >= 4 * 4096
    auto chunk_of = [&](uint32_t j) -> uint32_t { return __umulhi(j >> 12, cmagic); };

    // range of the keys in the list, exponents for the part sums
    uint32_t kmin, kmax;
    zone_key_range(ri, ra, z, kmin, kmax);
    const int Elo = (int)(kmin >> 23) ? (int)(kmin >> 23) : 1;
    const int Ehi = (int)(kmax >> 23) ? (int)(kmax >> 23) : 1;
    const int span = Ehi - Elo + 1;
    const int nclass = nparts * span;
    if (kmin > kmax || (SUMS && nclass > PIECE_CLASSES)) {
        if (tid == 0 && slice == 0) fail();
        return;
    }
    const int sh = finish_shift(kmin, kmax);
    uint32_t* zc = a.chunk_zcnt + (size_t)row * nchunks * ZPMAX;
    unsigned long long* zp = a.zpacc + ((size_t)row * ZMAX + z) * (PIECE_CLASSES * 2);
    unsigned long long* zcol = a.zcol + ((size_t)row * ZMAX + z) * COLLECT_CAP;
    auto slot_of = [&](int part) -> int { return part < nthr ? s_t[part] : TMAX + z; };

    if (PHASE == 1 && exact_pass) {
        // the redo round has no launches of its own for the histogram and the sliced pass: this workgroup makes the
        // zone's histogram here (a zone of an exact histogram is one bucket) and resolves the zone alone
        for (int i = tid; i < FH_BINS; i += FN_THREADS) s_fh[i] = 0;
        __syncthreads();
        batched_loop<8, FN_THREADS>(0u, n, (uint32_t)tid, [&](uint32_t i) { return kl[i].x; }, [&](uint32_t, uint32_t bits) {
            const uint32_t b = (key_of_bits(bits) - kmin) >> sh;
            atomicAdd(&s_fh[b < (uint32_t)FH_BINS ? b : (uint32_t)FH_BINS - 1], 1u);
        });
    } else {
        const uint32_t* zh = a.zhist + ((size_t)row * ZMAX + z) * FH_BINS;
        for (int i = tid; i < FH_BINS; i += FN_THREADS) s_fh[i] = zh[i];
    }
    if (count_fits) for (int i = tid; i < (nparts * nchunks) << zrep_shift; i += FN_THREADS) s_zc[i] = 0;
    if (SUMS) for (int i = tid; i < PIECE_CLASSES * PREP * 2; i += FN_THREADS) (&s_pacc[0][0])[i] = 0ull;
    __syncthreads();

    // what every candidate contributes once its part (number of the zone's thresholds it is NOT inside) is known
    const bool whole_adds = (PHASE == 0 ? (n + (uint32_t)S - 1u) / (uint32_t)S : n) <= 32768u;   // candidates this workgroup classifies
    auto classify = [&](int part, uint32_t key, uint32_t j) {
        if (count_fits) atomicAdd(&s_zc[(((uint32_t)(part * nchunks) + chunk_of(j)) << zrep_shift) | zrep_lane], 1u);
        if (SUMS) {
            const int E = (int)(key >> 23) ? (int)(key >> 23) : 1;
            const int cls = part * span + (E - Elo);
            const unsigned long long sq = sig_square(key);
            if (whole_adds) {   // uniform: at most 2^15 squares below 2^48 cannot overflow one 64-bit accumulator
                atomicAdd(&s_pacc[cls * PREP + lrep][0], sq);
            } else {
                atomicAdd(&s_pacc[cls * PREP + lrep][0], sq & 0xFFFFFFFFull);
                atomicAdd(&s_pacc[cls * PREP + lrep][1], sq >> 32);
            }
        }
    };
    // LDS counters and sums -> the zone's totals
    auto flush_totals = [&](bool with_sums) {
        __syncthreads();
        if (count_fits) {
            for (int i = tid; i < nparts * nchunks; i += FN_THREADS) {
                uint32_t v = 0;
                for (int r = 0; r < (1 << zrep_shift); ++r) v += s_zc[(i << zrep_shift) + r];
                if (v) {
                    const int part = i / nchunks, c = i - part * nchunks;
                    atomicAdd(&zc[(size_t)slot_of(part) * nchunks + c], v);
                }
            }
        }
        if (SUMS && with_sums && tid < nclass) {
            unsigned long long lo = 0, hi = 0;
            for (int r = 0; r < PREP; ++r) {
                const unsigned long long v = s_pacc[tid * PREP + r][0];
                lo += v & 0xFFFFFFFFull;
                hi += (v >> 32) + s_pacc[tid * PREP + r][1];
            }
            if (lo) atomicAdd(&zp[tid * 2], lo);
            if (hi) atomicAdd(&zp[tid * 2 + 1], hi);
        }
    };

    for (int u = wave; u < nthr; u += FN_THREADS / 64) {
        int bin;
        uint32_t rin, cnt;
        wave_rank_search<FH_BINS / 64>(s_fh, s_res[u], bin, rin, cnt);
        if (lane == 0) { s_bin[u] = (uint32_t)bin; s_rin[u] = rin; s_bcnt[u] = cnt; }
    }
    __syncthreads();
    if (tid == 0) {
        // the candidates of the thresholds' bins, in descending key order, form segments (one per distinct bin)
        uint32_t run = 0, seg = 0;
        bool ok = true;
        for (int u = 0; u < nthr; ++u) {
            if (u == 0 || s_bin[u] != s_bin[u - 1]) { seg = run; run += s_bcnt[u]; }
            if (s_rin[u] < 1 || s_rin[u] > s_bcnt[u]) ok = false;
            s_pos[u] = seg + s_rin[u] - 1;
        }
        if (!ok && slice == 0) fail();
        s_ok = ok ? 1 : 0;
        s_fast = run <= (uint32_t)COLLECT_CAP ? 1 : 0;
        s_ncollect = run;
    }
    __syncthreads();
    if (!s_ok) return;
    // Zones that the sliced pass (phase 0) takes: those whose per-chunk counters fit its LDS.  When the thresholds'
    // bins hold few candidates (par_ok) they are gathered for ranking in LDS; when they hold many (massive ties,
    // e.g. bf16 keys: par_big) they are moved to the zone's overflow list, on which phase 1 runs a radix select.
    // Every other zone is resolved by one workgroup in phase 1.
    const bool fits0 = !exact_pass && nparts * nchunks <= ZC0_CAP;   // the redo round: phase 1 only
    const bool par_ok = s_fast && fits0;
    const bool par_big = !s_fast && fits0;
    if (PHASE == 0 && !par_ok && !par_big) return;
    const int Seff = PHASE == 0 ? S : 1;
    const uint32_t per = (n + Seff - 1) / Seff;
    const uint32_t i0 = (uint32_t)slice * per, i1 = i0 + per < n ? i0 + per : n;
    const uint32_t ncollect_zone = s_ncollect;   // candidates in the thresholds' bins, all slices together
    uint2* c2l = a.cand2 + (size_t)row * (size_t)a.d + ri->zone_off[z];
    const uint32_t zcap = ri->zone_cap[z];
    __syncthreads();
    if (s_fast || (PHASE == 0 && par_big)) {
        if (tid == 0) s_ncollect = 0;
        for (int b = tid; b < FH_BINS; b += FN_THREADS) {
            int part = 0;
            bool isthr = false;
            for (int u = 0; u < nthr; ++u) {
                part += (uint32_t)b < s_bin[u] ? 1 : 0;
                isthr |= (uint32_t)b == s_bin[u];
            }
            s_bincls[b] = isthr ? (uint8_t)0xFF : (uint8_t)part;
        }
        __syncthreads();
    }
    if (PHASE == 0 && par_big) {
        // ---- read 2, massive ties: the thresholds' bins go to the overflow list.  First everything else is
        //      classified and the slice's share counted, then one reservation per workgroup, then the copy ----
        auto bin_class = [&](uint32_t key) -> uint32_t {
            uint32_t b = (key - kmin) >> sh;
            b = b < (uint32_t)FH_BINS ? b : (uint32_t)FH_BINS - 1;
            return s_bincls[b];
        };
        batched_loop<8, FN_THREADS>(i0, i1, (uint32_t)tid, [&](uint32_t i) { return kl[i]; },
                                    [&](uint32_t, uint2 e) {
            const uint32_t key = key_of_bits(e.x);
            const uint32_t cls = bin_class(key);
            const bool col = cls == 0xFFu;
            const uint64_t m = __ballot(col);
            if (m && (int)lane == __builtin_ctzll(m)) atomicAdd(&s_ncollect, (uint32_t)__popcll(m));
            if (!col) classify((int)cls, key, e.y);
        });
        __syncthreads();
        const uint32_t mine = s_ncollect;
        __syncthreads();
        if (tid == 0) s_ncollect = mine ? atomicAdd(&ra->zone_colcnt[z], mine) : 0u;   // becomes the write cursor
        __syncthreads();
        if (mine) {
            // With the copy: the key range of what is copied and the histogram of its indices, for the zone as a whole
            // (in the zone's gather buffer, unused on this path and cleared by the histogram launch).  When the range
            // is a single key, the usual case, the ranking launch needs no pass of its own for them.
            uint32_t* s_ih = s_un;   // FH_BINS words: free on this path
            int ish = 0;
            while (((uint32_t)(a.d - 1) >> ish) >= (uint32_t)FH_BINS) ++ish;
            const bool chunk_bins = nchunks <= FH_BINS;   // the bins are the row's count chunks when there are few enough
            for (int i = tid; i < FH_BINS; i += FN_THREADS) s_ih[i] = 0;
            if (tid == 0) { s_q[0] = 0u; s_eq[0] = 0u; }   // largest ~key, largest key
            __syncthreads();
            uint32_t kmx = 0, kmn_inv = 0;
            batched_loop<8, FN_THREADS>(i0, i1, (uint32_t)tid, [&](uint32_t i) { return kl[i]; },
                                        [&](uint32_t, uint2 e) {
                const uint32_t key = key_of_bits(e.x);
                const bool col = bin_class(key) == 0xFFu;
                const uint64_t m = __ballot(col);
                if (m) {
                    const int first = __builtin_ctzll(m);
                    uint32_t base = 0;
                    if ((int)lane == first) base = atomicAdd(&s_ncollect, (uint32_t)__popcll(m));
                    base = __shfl(base, first, 64);
                    if (col) {
                        const uint32_t pos = base + mbcnt(m);
                        if (pos < zcap) c2l[pos] = e;
                        atomicAdd(&s_ih[chunk_bins ? chunk_of(e.y) : e.y >> ish], 1u);
                        kmx = key > kmx ? key : kmx;
                        kmn_inv = ~key > kmn_inv ? ~key : kmn_inv;
                    }
                }
            });
            kmx = wave_max(kmx);
            kmn_inv = wave_max(kmn_inv);
            if (lane == 0 && kmn_inv) { atomicMax(&s_eq[0], kmx); atomicMax(&s_q[0], kmn_inv); }
            __syncthreads();
            uint32_t* zi = (uint32_t*)zcol;
            for (int i = tid; i < FH_BINS; i += FN_THREADS) {
                const uint32_t v = s_ih[i];
                if (v) atomicAdd(&zi[i], v);
            }
            if (tid == 0 && s_q[0]) { atomicMax(&zi[FH_BINS], s_q[0]); atomicMax(&zi[FH_BINS + 1], s_eq[0]); }
        }
        flush_totals(true);
        return;
    }
    if (s_fast) {
        // ---- read 2: candidates of the thresholds' bins are gathered in LDS, every other one is classified ----
        if (PHASE == 0 || !par_ok) {
            batched_loop<8, FN_THREADS>(i0, i1, (uint32_t)tid, [&](uint32_t i) { return kl[i]; },
                                        [&](uint32_t, uint2 e) {
                const uint32_t key = key_of_bits(e.x);
                const uint32_t j = e.y;
                uint32_t b = (key - kmin) >> sh;
                b = b < (uint32_t)FH_BINS ? b : (uint32_t)FH_BINS - 1;
                const uint32_t cls = s_bincls[b];
                if (cls == 0xFFu) {
                    const uint32_t at = atomicAdd(&s_ncollect, 1u);
                    if (at < (uint32_t)COLLECT_CAP) s_col[at] = ((unsigned long long)key << 32) | (uint32_t)~j;
                } else {
                    classify((int)cls, key, j);
                }
            });
            __syncthreads();
        }
        if constexpr (PHASE == 0) {
            // one reservation in the zone's list per workgroup; phase 1 (the next launch) ranks the gathered candidates
            const uint32_t mine = s_ncollect;   // <= COLLECT_CAP: the zone's threshold bins hold no more
            __syncthreads();
            if (tid == 0) s_ncollect = mine ? atomicAdd(&ra->zone_colcnt[z], mine) : 0u;
            __syncthreads();
            const uint32_t at0 = s_ncollect;
            for (uint32_t e = tid; e < mine; e += FN_THREADS)
                if (at0 + e < (uint32_t)COLLECT_CAP) zcol[at0 + e] = s_col[e];
            flush_totals(true);
            return;
        }
        const uint32_t ncol = ncollect_zone;
        if (par_ok) {
            if (ra->zone_colcnt[z] != ncol) {
                if (tid == 0) fail();
                return;
            }
            for (uint32_t e = tid; e < ncol; e += FN_THREADS) s_col[e] = zcol[e];
        } else if (s_ncollect != ncol) {
            if (tid == 0) fail();
            return;
        }
        __syncthreads();
        // descending order of (key, lower index first): composites are distinct and non-zero, zeros pad the end
        if (ncol <= 256u) {   // few: ranking by counting (a thread per value, every thread walks the list) is quicker than sorting
            uint32_t r0, r1;
            count_greater2(s_col, ncol, (uint32_t)tid, r0, r1);
            if ((uint32_t)tid < ncol) s_srt[r0] = s_col[tid];
            __syncthreads();
        } else {
            uint32_t np2 = 512;
            while (np2 < ncol) np2 <<= 1;   // <= COLLECT_CAP = 2 * FN_THREADS
            for (uint32_t e = tid; e < np2; e += FN_THREADS) s_srt[e] = e < ncol ? s_col[e] : 0ull;
            bitonic_sort_desc(s_srt, np2, (uint32_t)tid);
        }
        if (tid < nthr) {
            const unsigned long long c = s_srt[s_pos[tid]];
            s_tau[tid] = (uint32_t)(c >> 32);
            // inside: equal key and index <= that of the threshold element; when it is the last of its key
            // (every equal key sits in this bin, hence in this list) the index plays no part
            const bool last = s_pos[tid] + 1 >= ncol || (uint32_t)(s_srt[s_pos[tid] + 1] >> 32) != s_tau[tid];
            s_jx[tid] = last ? JX_ALL : ~(uint32_t)c + 1u;
        }
        __syncthreads();
        for (uint32_t e = tid; e < ncol; e += FN_THREADS) {
            int part = 0;
            for (int u = 0; u < nthr; ++u) part += e > s_pos[u] ? 1 : 0;
            const unsigned long long c = s_srt[e];
            classify(part, (uint32_t)(c >> 32), ~(uint32_t)c);
        }
        flush_totals(false);   // the sums stay in LDS and are added to the zone's totals below
    } else if constexpr (PHASE == 1) {
        // ---- slow path (a threshold bin too full to rank in LDS, e.g. massive ties): radix select on the
        //      keys, digits of 8, 8, 8, 7 bits from the top, then on the indices of the entries equal to the key.
        //      It runs on the overflow list (the thresholds' bins only) when phase 0 built one, else on the whole list ----
        const uint2* xl = par_big ? c2l : kl;
        const uint32_t xn = par_big ? ncollect_zone : n;
        if (par_big) {
            if (ra->zone_colcnt[z] != ncollect_zone || ncollect_zone > zcap) {
                if (tid == 0) fail();
                return;
            }
            if (tid < nthr) { s_res[tid] = s_pos[tid] + 1u; s_pfx[tid] = 0; }   // rank inside the overflow list
        }
        // One threshold and a single distinct key in the overflow list (the usual case for 16-bit inputs): the key is
        // the threshold, only the index cut is left: histogram of the indices, then the one bin ranked in LDS.
        if (tid == 0) { s_any = 0; s_nsub = 0; }
        __syncthreads();
        // Bins of the index histogram that the sliced launch made: the row's count chunks when they are few enough.  Then
        // the overflow list is not read here at all: the chunk that holds the index cut is read from the row itself
        // (its entries equal to the key, in index order), and every other chunk lies wholly on one side of the cut.
        const bool chunk_bins = nchunks <= FH_BINS;
        bool single_key = false;
        uint32_t cut_chunk = (uint32_t)nchunks, cut_inside = 0;   // count chunk of the cut, entries of it inside the top k
        if (par_big && nthr == 1) {
            // key range and index histogram of the overflow list: made by the sliced launch while it copied
            const uint32_t* zi = (const uint32_t*)zcol;
            int ish = 0;
            while (((uint32_t)(a.d - 1) >> ish) >= (uint32_t)FH_BINS) ++ish;
            for (int i = tid; i < FH_BINS; i += FN_THREADS) s_fh[i] = zi[i];
            if (tid == 0) { s_q[0] = ~zi[FH_BINS]; s_eq[0] = zi[FH_BINS + 1]; s_ncollect = 0; }
            __syncthreads();
            const uint32_t key1 = s_q[0];
            const bool single = key1 == s_eq[0];
            single_key = single;
            __syncthreads();
            if (single) {
                const uint32_t q = s_res[0];   // the threshold is the q-th entry of the list by ascending index
                if (q < xn) {
                    if (wave == 0) {
                        int bin;
                        uint32_t rin, cnt;
                        wave_rank_search<FH_BINS / 64>(s_fh, xn - q + 1u, bin, rin, cnt);   // q-th smallest = (n - q + 1)-th largest
                        if (lane == 0) { s_bin[0] = (uint32_t)bin; s_rin[0] = rin; s_bcnt[0] = cnt; }
                    }
                    __syncthreads();
                    if (chunk_bins) {
                        const uint32_t cnt = s_bcnt[0], rin = s_rin[0];
                        const uint32_t target = cnt - rin + 1u;   // the cut is the target-th of the chunk's entries equal to the key, by index
                        cut_chunk = s_bin[0];
                        cut_inside = target;
                        const int64_t e0 = (int64_t)cut_chunk * a.cchunk;
                        const int64_t e1 = e0 + a.cchunk < a.d ? e0 + a.cchunk : a.d;
                        // wave w takes a run of whole 64-element groups of the chunk, in order
                        const int64_t per = ((e1 - e0 + FN_THREADS - 1) / FN_THREADS) * 64;
                        const int64_t w0 = e0 + (int64_t)wave * per, w1 = w0 + per < e1 ? w0 + per : e1;
                        // sixteen groups at a time, their loads issued together (a load per group in turn would cost a
                        // memory latency per 64 elements); a lane past the end of the wave's run reads the run's last element
                        // (the element type is a compile-time tag: a run-time test inside the loop would split the loads up again)
                        auto equal_masks = [&](auto is_bf16, int64_t j0, uint64_t (&m)[16]) {
                            constexpr bool BF = decltype(is_bf16)::value;
                            uint32_t v[16];
#pragma unroll
                            for (int u = 0; u < 16; ++u) {
                                const int64_t j = j0 + u * 64 + lane;
                                const int64_t jc = (int64_t)row * a.ld + (j < w1 ? j : w1 - 1);
                                if (BF) v[u] = (uint32_t)((const uint16_t*)a.g)[jc] << 16;
                                else v[u] = ((const uint32_t*)a.g)[jc];
                            }
#pragma unroll
                            for (int u = 0; u < 16; ++u) m[u] = __ballot(j0 + u * 64 + lane < w1 && key_of_bits(v[u]) == key1);
                        };
                        auto scan_chunk = [&](auto is_bf16) {
                        uint32_t mine = 0;
                        for (int64_t j0 = w0; j0 < w1; j0 += 1024) {
                            uint64_t m[16];
                            equal_masks(is_bf16, j0, m);
#pragma unroll
                            for (int u = 0; u < 16; ++u) mine += (uint32_t)__popcll(m[u]);
                        }
                        if (lane == 0) s_subpfx[wave] = mine;
                        __syncthreads();
                        uint32_t before = 0, total = 0;
                        for (uint32_t w2 = 0; w2 < (uint32_t)(FN_THREADS / 64); ++w2) {
                            const uint32_t v = s_subpfx[w2];
                            before += w2 < wave ? v : 0u;
                            total += v;
                        }
                        // total != cnt cannot happen (every entry equal to the key is in the overflow list); if it did the
                        // zone would be resolved the long way below
                        if (total == cnt && rin >= 1u && rin <= cnt && before < target && target <= before + mine) {
                            uint32_t run = before;
                            bool found = false;
                            for (int64_t j0 = w0; j0 < w1 && !found; j0 += 1024) {
                                uint64_t m[16];
                                equal_masks(is_bf16, j0, m);
#pragma unroll
                                for (int u = 0; u < 16; ++u) {
                                    const uint32_t c = (uint32_t)__popcll(m[u]);
                                    if (!found && run + c >= target) {
                                        if (((m[u] >> lane) & 1ull) && run + mbcnt(m[u]) + 1u == target) {
                                            s_tau[0] = key1;
                                            s_jx[0] = (uint32_t)(j0 + u * 64 + lane) + 1u;
                                            s_any = 1;
                                        }
                                        found = true;
                                    }
                                    run += c;
                                }
                            }
                        }
                        };   // scan_chunk
                        if (a.dtype == MLMC_BF16) scan_chunk(std::true_type{});
                        else scan_chunk(std::false_type{});
                    } else if (s_bcnt[0] <= (uint32_t)COLLECT_CAP && s_bcnt[0] > 0) {
                        const uint32_t ibin = s_bin[0];
                        batched_loop<16, FN_THREADS>(0u, xn, (uint32_t)tid, [&](uint32_t i) { return xl[i].y; }, [&](uint32_t, uint32_t j) {
                            if ((j >> ish) == ibin) {
                                const uint32_t at = atomicAdd(&s_ncollect, 1u);
                                if (at < (uint32_t)COLLECT_CAP) s_col[at] = j;
                            }
                        });
                        __syncthreads();
                        const uint32_t nc2 = s_ncollect < (uint32_t)COLLECT_CAP ? s_ncollect : (uint32_t)COLLECT_CAP;
                        {   // the entries are indices (distinct), held in 64-bit slots
                            uint32_t r0, r1;
                            count_greater2(s_col, nc2, (uint32_t)tid, r0, r1);
                            if ((uint32_t)tid < nc2 && r0 + 1u == s_rin[0]) { s_tau[0] = key1; s_jx[0] = (uint32_t)s_col[tid] + 1u; s_any = 1; }
                            if ((uint32_t)tid + FN_THREADS < nc2 && r1 + 1u == s_rin[0]) { s_tau[0] = key1; s_jx[0] = (uint32_t)s_col[tid + FN_THREADS] + 1u; s_any = 1; }
                        }
                    }
                } else if (tid == 0) {   // every entry of the list is inside
                    s_tau[0] = key1;
                    s_jx[0] = JX_ALL;
                    s_any = 1;
                }
                __syncthreads();
            }
        }
        const bool resolved = s_any != 0;
        __syncthreads();
        if (!resolved) {
            for (int pass = 0; pass < 4; ++pass) {
                const int shift = pass == 0 ? 23 : pass == 1 ? 15 : pass == 2 ? 7 : 0;
                const uint32_t mask = pass == 3 ? 127u : 255u;
                const int hb = pass == 3 ? 7 : shift + 8;   // unresolved low bits before this pass (31 for pass 0)
                __syncthreads();
                if (tid == 0) {
                    int ns = 0;
                    for (int u = 0; u < nthr; ++u) {
                        if (u == 0 || s_pfx[u] != s_pfx[u - 1]) { s_subpfx[ns] = s_pfx[u]; ++ns; }
                        s_sub[u] = ns - 1;
                    }
                    s_nsub = ns;
                }
                for (int i = tid; i < TMAX * 256; i += FN_THREADS) (&s_hist[0][0])[i] = 0;
                __syncthreads();
                const int nsub = s_nsub;
                if (pass == 0) {
                    batched_loop<8, FN_THREADS>(0u, xn, (uint32_t)tid, [&](uint32_t i) { return xl[i].x; }, [&](uint32_t, uint32_t bits) {
                        atomicAdd(&s_hist[0][(key_of_bits(bits) >> 23) & 255u], 1u);
                    });
                } else if (nsub == 1) {
                    const uint32_t pf = s_subpfx[0] >> hb;
                    batched_loop<8, FN_THREADS>(0u, xn, (uint32_t)tid, [&](uint32_t i) { return xl[i].x; }, [&](uint32_t, uint32_t bits) {
                        const uint32_t key = key_of_bits(bits);
                        if ((key >> hb) == pf) atomicAdd(&s_hist[0][(key >> shift) & mask], 1u);
                    });
                } else {
                    batched_loop<8, FN_THREADS>(0u, xn, (uint32_t)tid, [&](uint32_t i) { return xl[i].x; }, [&](uint32_t, uint32_t bits) {
                        const uint32_t key = key_of_bits(bits);
                        const uint32_t kp = key >> hb;
                        for (int s2 = 0; s2 < nsub; ++s2)
                            if (kp == (s_subpfx[s2] >> hb)) atomicAdd(&s_hist[s2][(key >> shift) & mask], 1u);
                    });
                }
                __syncthreads();
                for (int u = wave; u < nthr; u += FN_THREADS / 64) {
                    int bin;
                    uint32_t rin, cnt;
                    wave_rank_search<4>(s_hist[s_sub[u]], s_res[u], bin, rin, cnt);
                    if (lane == 0) {
                        s_pfx[u] |= (uint32_t)bin << shift;
                        s_res[u] = rin;
                        if (pass == 3) { s_tau[u] = s_pfx[u]; s_q[u] = rin; s_eq[u] = cnt; }
                    }
                }
            }
            __syncthreads();
            // index cut among the entries equal to the threshold key: the q-th smallest index + 1
            if (tid < nthr) {
                s_jx[tid] = JX_ALL;
                s_pfx[tid] = 0;
                s_res[tid] = s_eq[tid] - s_q[tid] + 1;   // the q-th smallest is the (eq - q + 1)-th largest
                if (s_q[tid] < 1 || s_q[tid] > s_eq[tid]) fail();
            }
            if (tid == 0) {
                int any = 0;
                for (int u = 0; u < nthr; ++u) any |= s_q[u] < s_eq[u] ? 1 : 0;
                s_any = any;
            }
            __syncthreads();
            if (s_any) {
                for (int pass = 0; pass < 4; ++pass) {
                    const int shift = 24 - 8 * pass;
                    const int hb = shift + 8;   // 32 for pass 0: no prefix yet
                    if (tid == 0) {
                        int ns = 0;
                        for (int u = 0; u < nthr; ++u) {
                            if (s_q[u] >= s_eq[u]) { s_sub[u] = -1; continue; }
                            int found = -1;
                            for (int s2 = 0; s2 < ns; ++s2)
                                if (s_subtau[s2] == s_tau[u] && s_subpfx[s2] == s_pfx[u]) found = s2;
                            if (found < 0) { s_subtau[ns] = s_tau[u]; s_subpfx[ns] = s_pfx[u]; found = ns++; }
                            s_sub[u] = found;
                        }
                        s_nsub = ns;
                    }
                    for (int i = tid; i < TMAX * 256; i += FN_THREADS) (&s_hist[0][0])[i] = 0;
                    __syncthreads();
                    const int nsub = s_nsub;
                    batched_loop<8, FN_THREADS>(0u, xn, (uint32_t)tid, [&](uint32_t i) { return xl[i]; },
                                                [&](uint32_t, uint2 e) {
                        const uint32_t key = key_of_bits(e.x), j = e.y;
                        for (int s2 = 0; s2 < nsub; ++s2) {
                            if (key != s_subtau[s2]) continue;
                            if (pass == 0 || (j >> hb) == (s_subpfx[s2] >> hb)) atomicAdd(&s_hist[s2][(j >> shift) & 255u], 1u);
                        }
                    });
                    __syncthreads();
                    for (int u = wave; u < nthr; u += FN_THREADS / 64) {
                        if (s_sub[u] < 0) continue;
                        int bin;
                        uint32_t rin, cnt;
                        wave_rank_search<4>(s_hist[s_sub[u]], s_res[u], bin, rin, cnt);
                        if (lane == 0) {
                            s_pfx[u] |= (uint32_t)bin << shift;
                            s_res[u] = rin;
                            if (pass == 3) s_jx[u] = s_pfx[u] + 1u;
                        }
                    }
                    __syncthreads();
                }
            }
        }
        // every candidate's part from the exact thresholds
        if (resolved && single_key && chunk_bins) {
            // one key, bins = count chunks: the histogram says how many entries every chunk has, the cut says which side
            // they are on; their squares are all the same
            const uint32_t key1 = s_tau[0];
            const uint32_t inside_all = s_res[0] < xn ? s_res[0] : xn;   // entries of the list inside the top k
            for (int c = tid; c < nchunks; c += FN_THREADS) {
                const uint32_t h = s_fh[c];
                const uint32_t p0 = (uint32_t)c < cut_chunk ? h : (uint32_t)c > cut_chunk ? 0u : cut_inside;
                if (p0) atomicAdd(&zc[(size_t)slot_of(0) * nchunks + c], p0);
                if (h - p0) atomicAdd(&zc[(size_t)slot_of(1) * nchunks + c], h - p0);
            }
            if (SUMS && tid < 2) {
                const unsigned long long cntp = tid == 0 ? inside_all : xn - inside_all;
                const int E = (int)(key1 >> 23) ? (int)(key1 >> 23) : 1;
                const int cls = tid * span + (E - Elo);
                const unsigned long long sq = sig_square(key1);
                if (cntp) {
                    atomicAdd(&zp[cls * 2], (sq & 0xFFFFFFFFull) * cntp);
                    atomicAdd(&zp[cls * 2 + 1], (sq >> 32) * cntp);
                }
            }
        } else if (count_fits || SUMS) {
            batched_loop<8, FN_THREADS>(0u, xn, (uint32_t)tid, [&](uint32_t i) { return xl[i]; },
                                        [&](uint32_t, uint2 e) {
                const uint32_t key = key_of_bits(e.x), j = e.y;
                int part = 0;
                for (int u = 0; u < nthr; ++u) {
                    const uint32_t tau = s_tau[u];
                    part += (key > tau || (key == tau && j < s_jx[u])) ? 0 : 1;
                }
                classify(part, key, j);
            });
        }
        flush_totals(true);
        __syncthreads();
        if (SUMS) for (int i = tid; i < PIECE_CLASSES * PREP * 2; i += FN_THREADS) (&s_pacc[0][0])[i] = 0ull;
    }
    __syncthreads();
    if (PHASE == 0) return;
    if (tid < nthr) {
        ri->thr_tau[s_t[tid]] = s_tau[tid];
        ri->thr_jx[s_t[tid]] = s_jx[tid];
    }
    if (!count_fits) {
        // long rows with many thresholds in one zone: a few parts at a time, one more read of the list each
        const int ppp = ZC_CAP / nchunks;   // >= 1: a row has at most CHUNKS_MAX = ZC_CAP chunks
        for (int p0 = 0; p0 < nparts; p0 += ppp) {
            const int p1 = p0 + ppp < nparts ? p0 + ppp : nparts;
            __syncthreads();
            for (int i = tid; i < (p1 - p0) * nchunks; i += FN_THREADS) s_zc[i] = 0;
            __syncthreads();
            batched_loop<8, FN_THREADS>(0u, n, (uint32_t)tid, [&](uint32_t i) { return kl[i]; },
                                        [&](uint32_t, uint2 e) {
                const uint32_t key = key_of_bits(e.x), j = e.y;
                int part = 0;
                for (int u = 0; u < nthr; ++u) {
                    const uint32_t tau = s_tau[u];
                    part += (key > tau || (key == tau && j < s_jx[u])) ? 0 : 1;
                }
                if (part >= p0 && part < p1) atomicAdd(&s_zc[(part - p0) * nchunks + (int)chunk_of(j)], 1u);
            });
            __syncthreads();
            for (int i = tid; i < (p1 - p0) * nchunks; i += FN_THREADS) {
                const int part = p0 + i / nchunks, c = i % nchunks;
                zc[(size_t)slot_of(part) * nchunks + c] = s_zc[i];
            }
        }
    }
    if (!SUMS) return;

    // ---- exact sums of the parts: one piece per (part, exponent): the zone's totals of the earlier launch plus
    //      what the ranked candidates added here ----
    __syncthreads();
    if (tid < nclass) {
        unsigned long long lo = zp[tid * 2], hi = zp[tid * 2 + 1];
        for (int r = 0; r < PREP; ++r) {
            const unsigned long long v = s_pacc[tid * PREP + r][0];
            lo += v & 0xFFFFFFFFull;
            hi += (v >> 32) + s_pacc[tid * PREP + r][1];
        }
        hi += lo >> 32;
        lo &= 0xFFFFFFFFull;
        if (lo | hi) {
            const int part = tid / span, e = Elo + tid % span;
            const uint32_t at = atomicAdd(&ra->n_pieces, 1u);
            if (at >= (uint32_t)PMAX) {
                fail();
            } else {
                Piece* pc = &ra->pieces[at];
                pc->exp = e;
                pc->lo = lo;
                pc->hi = hi;
                pc->band_plus1 = (part < nthr ? s_t[part] : s_t[nthr - 1] + 1) + 1;
            }
        }
    }
    };   // run_item

    for (int item = blockIdx.x; item < nitems; item += gridDim.x) {
        int z = 0;
        while (z + 1 < nzones && s_first[z + 1] <= item) ++z;
        __syncthreads();   // the previous item is done with the shared arrays
        run_item(z, item - s_first[z]);
    }
}

// ---------------------------------------------------------------------------------------------------
// Delta_l (Lemma 3.4) from the exact group and part sums, then the adaptive draw.  One workgroup per row; the
// 640-bit sums live in LDS.
__global__ __launch_bounds__(256) void k_norms(TopkArgs a) {
    __shared__ uint32_t s_big[TMAX][20];
    __shared__ unsigned long long s_wide[TMAX][20];   // per 32-bit word position: sum of the addends' words, carries not yet propagated
    __shared__ double s_norm[LMAX];
    __shared__ double s_p[LMAX];
    const int row = blockIdx.x, tid = threadIdx.x;
    const RowInfo* ri = a.rinfo + row;
    const RowAcc* ra = a.racc + row;
    for (int i = tid; i < TMAX * 20; i += 256) (&s_wide[0][0])[i] = 0ull;
    __syncthreads();
    // Every non-zero group or part sum goes to its band: v << shift is split into three 32-bit words that are added
    // (LDS atomics, any order) to 64-bit counters of their word positions; a few hundred addends cannot overflow them.
    auto add = [&](int band, uint64_t v, int shift) {
        if (!v) return;
        const int wi = shift >> 5, bs = shift & 31;
        uint32_t parts[3];
        parts[0] = (uint32_t)(v << bs);
        parts[1] = (uint32_t)(bs ? v >> (32 - bs) : v >> 32);
        parts[2] = bs ? (uint32_t)(v >> (64 - bs)) : 0u;
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (parts[i] && wi + i < 20) atomicAdd(&s_wide[band][wi + i], (unsigned long long)parts[i]);
    };
    const int np = ra->n_pieces < (uint32_t)PMAX ? (int)ra->n_pieces : PMAX;
    for (int g = tid; g < GMAX + np; g += 256) {
        int band, sh;
        uint64_t lo, hi;
        if (g < GMAX) {
            band = ri->g_band[g];
            sh = 2 * ((int)ri->g_exp[g] - 1);
            lo = ra->gsum[g][0];
            hi = ra->gsum[g][1];
        } else {
            const Piece pc = ra->pieces[g - GMAX];
            band = pc.band_plus1 - 1;
            sh = 2 * (pc.exp - 1);
            lo = pc.lo;
            hi = pc.hi;
        }
        if (band >= 1 && band <= a.L && sh >= 0) {
            add(band, lo, sh);
            add(band, hi, sh + 32);
        }
    }
    __syncthreads();
    const int l = tid;
    if (l >= 1 && l <= a.L) {
        uint64_t wide[20];
#pragma unroll
        for (int i = 0; i < 20; ++i) wide[i] = s_wide[l][i];
        uint64_t carry = 0;
#pragma unroll
        for (int i = 0; i < 20; ++i) {
            const uint64_t t = wide[i] + carry;
            s_big[l][i] = (uint32_t)t;
            carry = t >> 32;
        }
        BigAcc acc;
        acc.w = s_big[l];
        double nrm = __dsqrt_rn(acc.to_double());
        s_norm[l - 1] = nrm;
        a.norms[(size_t)row * a.L + (l - 1)] = nrm;
        if (a.norms_user) a.norms_user[(size_t)row * a.L + (l - 1)] = nrm;
    }
    __syncthreads();
    if (tid == 0 && a.draw_mode == 3) {
        draw_row(a, row, s_norm, s_p);
        RowInfo* rw = a.rinfo + row;
        rw->spec_ok = (rw->spec_level > 0 && rw->spec_level == rw->level) ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------------------------------
// Membership tests of the message (Eq. (6)): base band = top k_0; drawn band = top k_l without top k_{l-1}.
struct Thr3 {
    uint32_t tau[3], jx[3];
};
__device__ __forceinline__ Thr3 load_thr3(const RowInfo* ri) {
    Thr3 t;
    const int lev = ri->level;
    const int ts[3] = {0, lev - 1, lev};
#pragma unroll
    for (int i = 0; i < 3; ++i) { t.tau[i] = ri->thr_tau[ts[i]]; t.jx[i] = ri->thr_jx[ts[i]]; }
    return t;
}
__device__ __forceinline__ bool inside_top(const Thr3& th, int i, uint32_t key, uint32_t j) {
    return key > th.tau[i] || (key == th.tau[i] && j < th.jx[i]);
}

// ---------------------------------------------------------------------------------------------------
// Per row, once the level is drawn and the thresholds are exact: where the row's message starts, how many of its
// entries lie before every chunk (regions of band 0 and band l plus the parts of the zones of thresholds 0, l-1, l
// that belong to those bands), and the three thresholds, so that the kernels that write the message start from
// one small record.
constexpr int MP_THREADS = 1024;
__global__ __launch_bounds__(MP_THREADS) void k_msgplan(TopkArgs a) {
    __shared__ uint32_t s_scan[MP_THREADS / 64 + 1];
    __shared__ uint32_t s_carry;
    __shared__ int64_t s_k[TMAX];   // the ladder, indexed per lane below
    const int row = blockIdx.x, tid = threadIdx.x;
    if (tid < TMAX) s_k[tid] = tid <= a.L ? a.k[tid] : 0;
    RowInfo* ri = a.rinfo + row;
    const int lev = ri->level;
    const int nzn = ri->n_zones;
    const int nc = a.cchunks_per_row;   // count chunks
    // the regions of band 0 and of band l (the last one with that label): lane r looks at region r
    int r0, rl;
    {
        const uint32_t lane = lane_id();
        const int lab = (int)lane <= nzn ? ri->region_label[lane] : -1;
        const uint64_t m0 = __ballot(lab == 0), ml = __ballot(lab == lev);
        r0 = m0 ? 63 - __builtin_clzll(m0) : -1;
        rl = ml ? 63 - __builtin_clzll(ml) : -1;
    }
    int zs[3] = {-1, -1, -1};
    {
        const int z0 = ri->thr_zone[0], za = ri->thr_zone[lev - 1], zb = ri->thr_zone[lev];
        if (z0 >= 0) zs[0] = 0;                                   // inside the top k_0
        if (za >= 0) zs[1] = zb == za ? lev : TMAX + za;          // just below threshold l-1, in its zone
        if (zb >= 0 && zb != za) zs[2] = lev;                     // above threshold l, in a zone of its own
    }
    // message entries before every count chunk: a thread takes a run of consecutive count chunks (their counts are
    // fetched together), one scan over the threads' sums
    uint32_t* cbase = a.chunk_base + (size_t)row * (nc + 1);
    constexpr int MP_RUN = CHUNKS_MAX / MP_THREADS;   // a row has at most CHUNKS_MAX count chunks
    const int per = (nc + MP_THREADS - 1) / MP_THREADS;
    uint32_t v[MP_RUN];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < MP_RUN; ++i) {
        const int c = tid * per + i;
        v[i] = 0;
        if (i < per && c < nc) {
            // both tables are laid out [region or part][count chunk]: a thread's run is contiguous
            const uint32_t* cc = a.chunk_cnt + (size_t)row * RMAX * nc + c;
            const uint32_t* zc = a.chunk_zcnt + (size_t)row * ZPMAX * nc + c;
            if (r0 >= 0) v[i] += cc[(size_t)r0 * nc];
            if (rl >= 0) v[i] += cc[(size_t)rl * nc];
#pragma unroll
            for (int q = 0; q < 3; ++q)
                if (zs[q] >= 0) v[i] += zc[(size_t)zs[q] * nc];
        }
        mine += v[i];
    }
    uint32_t total;
    uint32_t run = block_excl_scan<MP_THREADS>(mine, s_scan, total);
#pragma unroll
    for (int i = 0; i < MP_RUN; ++i) {
        const int c = tid * per + i;
        if (i < per && c < nc) cbase[c] = run;
        run += v[i];
    }
    if (tid == 0) s_carry = total;
    __syncthreads();
    // The messages of the rows before this one, and this row's place among all rows by descending message length
    // (the message kernels take the rows in that order, so that the long ones are not left for the end): lanes
    // of the first wave take rows in turn.
    int64_t start = 0;
    if (tid < 64) {
        const int64_t mine = a.k[0] + s_k[lev] - s_k[lev - 1];
        uint32_t ahead = 0;
        for (int i = tid; i < a.M; i += 64) {
            const int li = a.rinfo[i].level;
            const int64_t ni = a.k[0] + s_k[li] - s_k[li - 1];
            if (i < row) start += ni;
            ahead += (ni > mine || (ni == mine && i < row)) ? 1u : 0u;
        }
        ahead = wave_sum(ahead);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)start, o, 64), hi = __shfl_xor((uint32_t)((uint64_t)start >> 32), o, 64);
            start += (int64_t)(((uint64_t)hi << 32) | lo);
        }
        if (tid == 0) a.row_order[ahead] = row;
    }
    if (tid == 0) {
        const int64_t nnz = a.k[0] + a.k[lev] - a.k[lev - 1];
        cbase[nc] = s_carry;
        if ((int64_t)s_carry != nnz) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        MsgPlan m;
        m.rowstart = start;
        m.rownnz = nnz;
        const int ts[3] = {0, lev - 1, lev};
        for (int i = 0; i < 3; ++i) { m.tau[i] = ri->thr_tau[ts[i]]; m.jx[i] = ri->thr_jx[ts[i]]; }
        m.weight = ri->weight;
        m.level = lev;
        ri->msg = m;
        a.row_off[row] = start;
        a.tile_off[(size_t)row * (a.ntiles + 1) + a.ntiles] = (uint32_t)nnz;
        if (row == a.M - 1) {
            a.row_off[a.M] = start + nnz;
            if (start + nnz > a.capacity) atomicOr(a.dev_status, MLMC_DEV_CAPACITY);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// The message read.  One workgroup per (chunk, row), one tile per step.
constexpr int WR_THREADS = 512;
constexpr int WR_WAVES = WR_THREADS / 64;
constexpr int WR_LINES = TILE / (WR_WAVES * 64);   // 64-element lines of a wave per step
constexpr int WR_STAGE = 1024;   // entries of one step that are gathered in LDS and written densely
constexpr int WR_DIRECT = 1024;  // steps with more entries write them straight from the lanes (at most WR_STAGE)

template <int DT, bool VEC>
__global__ __launch_bounds__(WR_THREADS, 4) void k_write(TopkArgs a) {
    __shared__ uint32_t s_wemit[2][WR_WAVES];
    __shared__ uint2 s_out[2][WR_STAGE];
    const int row = a.row_order[blockIdx.y], chunk_id = blockIdx.x, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    const RowInfo* ri = a.rinfo + row;
    if (ri->spec_ok) return;   // the message of this row comes from the staged lists (k_filter)
    const int nc = a.cchunks_per_row;   // one workgroup per count chunk
    const int64_t nt = a.ntiles;
    const MsgPlan mp = ri->msg;
    const int64_t rowstart = mp.rowstart;
    Thr3 th;
#pragma unroll
    for (int i = 0; i < 3; ++i) { th.tau[i] = mp.tau[i]; th.jx[i] = mp.jx[i]; }
    const float w = mp.weight;
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    const int64_t c0 = (int64_t)chunk_id * a.cchunk;
    const int64_t c1 = c0 + a.cchunk < a.d ? c0 + a.cchunk : a.d;
    const uint32_t base = a.chunk_base[(size_t)row * (nc + 1) + chunk_id];
    const uint32_t next_base = a.chunk_base[(size_t)row * (nc + 1) + chunk_id + 1];
    uint32_t run = base;   // entries of this row before the current step

    // Thresholds as signed "key > tau" wherever the index plays no part (keys are 31-bit, so -1 admits every
    // key and 0x7FFFFFFF none): all entries equal to the key inside -> tau - 1; none of them -> tau.  "cut"
    // marks a threshold whose equal keys are split by index.
    int32_t tau[3];
    bool cut[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t t = th.tau[i] > 0x7FFFFFFFu ? 0x7FFFFFFFu : th.tau[i];
        cut[i] = th.jx[i] != 0u && th.jx[i] != JX_ALL;
        tau[i] = th.jx[i] == JX_ALL ? (int32_t)t - 1 : (int32_t)t;
    }
    const bool any_cut = cut[0] || cut[1] || cut[2];

    // One step = one tile of 4096 elements; a wave covers 512 consecutive elements as 8 lines of 64, one element
    // per lane and load, so that the order of the lanes is the order of the indices.  Membership is one wave-wide
    // mask per line, combined with scalar logic.  The step's entries are gathered in LDS (s_out[par]) and written
    // densely after the barrier of the next step; a step with more than WR_STAGE entries writes them straight
    // from the lanes that hold them.
    uint32_t par = 0;
    uint32_t prev_first = 0, prev_count = 0;   // a finished step whose entries still wait in s_out[par ^ 1]
    // s_out holds {index, input bits}: the weight is applied here, once per entry
    auto write_out = [&](uint32_t buf_id, uint32_t first, uint32_t count) {
        for (uint32_t i = tid; i < count; i += WR_THREADS) {
            const uint2 e = s_out[buf_id][i];
            const int64_t at = rowstart + first + i;
            const uint32_t key = key_of_bits(e.y);
            const bool base = (int32_t)key > tau[0] || (cut[0] && key == th.tau[0] && e.x < th.jx[0]);
            const float v = __uint_as_float(e.y);
            if (at < a.capacity) { a.idx[at] = e.x; a.val[at] = base ? v : __fmul_rn(v, w); }
        }
    };
    auto step = [&](auto with_cuts, auto is_ragged, const uint32_t (&b)[WR_LINES], int64_t sb) {
        constexpr bool CUTS = decltype(with_cuts)::value;
        constexpr bool RAGGED = decltype(is_ragged)::value;
        const uint32_t jbase = (uint32_t)(sb + (int64_t)wave * (64 * WR_LINES)) + lane;
        auto inside = [&](int i, uint32_t key, uint32_t j) -> bool {
            bool g = (int32_t)key > tau[i];
            if (CUTS) g = g || (cut[i] && key == th.tau[i] && j < th.jx[i]);
            return g;
        };
        uint64_t em[WR_LINES];
        uint32_t wcount = 0;
#pragma unroll
        for (int q = 0; q < WR_LINES; ++q) {
            const uint32_t key = key_of_bits(b[q]);
            const uint32_t j = jbase + (uint32_t)q * 64u;
            bool m = inside(0, key, j) || (inside(2, key, j) && !inside(1, key, j));
            if (RAGGED) m = m && (int64_t)j < c1;
            em[q] = __ballot(m);
            wcount += (uint32_t)__popcll(em[q]);
        }
        if (lane == 0) s_wemit[par][wave] = wcount;
        __syncthreads();
        if (prev_count) write_out(par ^ 1u, prev_first, prev_count);   // every wave is past its staging of that step
        uint32_t wave_pre = 0, step_total = 0;
#pragma unroll
        for (int w2 = 0; w2 < WR_WAVES; ++w2) {
            const uint32_t v = s_wemit[par][w2];
            if ((uint32_t)w2 < wave) wave_pre += v;
            step_total += v;
        }
        if (tid == 0) a.tile_off[(size_t)row * (nt + 1) + sb / TILE] = run;
        if (step_total > (uint32_t)WR_DIRECT) {
            // a dense step: every lane writes its own entry (emitting neighbours write neighbouring positions)
            uint32_t pos0 = run + wave_pre;
#pragma unroll
            for (int q = 0; q < WR_LINES; ++q) {
                const uint64_t m = em[q];
                if (m == 0) continue;   // uniform: nobody in the wave emits from this line
                const uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, pos0));
                if (__builtin_amdgcn_inverse_ballot_w64(m)) {
                    const uint32_t j = jbase + (uint32_t)q * 64u;
                    const uint32_t key = key_of_bits(b[q]);
                    const int64_t at = rowstart + pos;
                    const bool base = (int32_t)key > tau[0] || (cut[0] && key == th.tau[0] && j < th.jx[0]);
                    const float v = __uint_as_float(b[q]);
                    if (at < a.capacity) { a.idx[at] = j; a.val[at] = base ? v : __fmul_rn(v, w); }
                }
                pos0 += (uint32_t)__popcll(m);
            }
        } else {
            uint32_t pos0 = wave_pre;
#pragma unroll
            for (int q = 0; q < WR_LINES; ++q) {
                const uint64_t m = em[q];
                if (m == 0) continue;   // uniform: nobody in the wave emits from this line
                const uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, pos0));
                if (__builtin_amdgcn_inverse_ballot_w64(m)) s_out[par][pos] = make_uint2(jbase + (uint32_t)q * 64u, b[q]);
                pos0 += (uint32_t)__popcll(m);
            }
        }
        prev_first = run;
        prev_count = step_total > (uint32_t)WR_DIRECT ? 0u : step_total;
        run += step_total;
        par ^= 1u;
    };
    // `ragged` and any_cut are uniform over the workgroup (every variant holds barriers)
    auto run_step = [&](const uint32_t (&b)[WR_LINES], int64_t sb, bool ragged) {
        if (ragged) step(std::true_type{}, std::true_type{}, b, sb);
        else if (any_cut) step(std::true_type{}, std::false_type{}, b, sb);
        else step(std::false_type{}, std::false_type{}, b, sb);
    };
    // two steps (sixteen loads per lane) are in flight: the loads of step s + 2 are issued as soon as step s is done
    const int64_t nfull = (c1 - c0) / TILE;
    auto issue = [&](int64_t s2, uint32_t (&b)[WR_LINES]) {
        const int64_t j = c0 + s2 * TILE + (int64_t)wave * (64 * WR_LINES) + lane;
#pragma unroll
        for (int q = 0; q < WR_LINES; ++q) b[q] = ld.load1_stream(j + q * 64);
    };
    uint32_t buf[2][WR_LINES];
    int64_t s2 = 0;
    if (nfull >= 2) {
        issue(0, buf[0]);
        issue(1, buf[1]);
        for (; s2 + 4 <= nfull; s2 += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                run_step(buf[u], c0 + (s2 + u) * TILE, false);
                issue(s2 + u + 2, buf[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) run_step(buf[u], c0 + (s2 + u) * TILE, false);
        s2 += 2;
    }
    for (; s2 < nfull; ++s2) {
        issue(s2, buf[0]);
        run_step(buf[0], c0 + s2 * TILE, false);
    }
    if (c0 + nfull * TILE < c1) {   // the ragged last tile of the row
        const int64_t sb = c0 + nfull * TILE;
#pragma unroll
        for (int q = 0; q < WR_LINES; ++q) {
            const int64_t j = sb + (int64_t)wave * (64 * WR_LINES) + q * 64 + lane;
            buf[0][q] = j < c1 ? ld.load1(j) : 0u;
        }
        run_step(buf[0], sb, true);
    }
    __syncthreads();
    if (prev_count) write_out(par ^ 1u, prev_first, prev_count);
    // consistency: the chunk ends where the per-chunk counts say the next one starts
    if (tid == 0 && run != next_base) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
}

// ---------------------------------------------------------------------------------------------------
// The message without a second read of the row, for rows whose drawn band was staged by the selection read.
// One workgroup per (chunk, row): the chunk's staged entries (16 private lists: zone candidates and band
// members, in the order the waves met them) are tested against the exact thresholds; a bitmap over the chunk's
// elements turns the members' offsets into ranks, i.e. into positions of the index-ordered message.
constexpr int FL_THREADS = 1024;

__global__ __launch_bounds__(FL_THREADS) void k_filter(TopkArgs a) {
    extern __shared__ uint32_t s_dyn[];     // two arrays of chunk / 32 words
    uint32_t* s_bits = s_dyn;               // bit rel: element c0 + rel is in the message
    uint32_t* s_pre = s_dyn + a.chunk / 32; // members in the words before
    __shared__ uint32_t s_scan[FL_THREADS / 64 + 1];
    const int row = a.row_order[blockIdx.y], chunk_id = blockIdx.x, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6);
    const RowInfo* ri = a.rinfo + row;
    if (!ri->spec_ok) return;   // k_write reads the row again
    const int nc = a.chunks_per_row;
    const int64_t nt = a.ntiles;
    const int64_t c0 = (int64_t)chunk_id * a.chunk;
    const int64_t c1 = c0 + a.chunk < a.d ? c0 + a.chunk : a.d;
    const int nwords = (int)((c1 - c0 + 31) / 32);
    // wave w of this workgroup reads the private list of wave w of the selection read
    const uint2* priv = a.cand_priv + ((size_t)row * nc + chunk_id) * (size_t)(2 * a.chunk) + (size_t)wave * (a.chunk / 8);
    const uint32_t cnt = a.priv_cnt[((size_t)row * nc + chunk_id) * 16 + wave];
    // The first FL_KEEP entries of every lane stay in registers for the second pass (a wave's list rarely holds
    // more than 64 * FL_KEEP).  They are loaded without waiting for the list's length: the list's memory is there
    // whatever it holds, and what lies past the end is ignored.
    constexpr int FL_KEEP = 8;
    uint2 ent[FL_KEEP];
#pragma unroll
    for (int u = 0; u < FL_KEEP; ++u) ent[u] = priv[lane + 64u * (uint32_t)u];
    static_assert(64 * FL_KEEP <= 4 * TILE / MAIN_WAVES, "a wave's list has room for at least chunk / 16 >= 1024 entries");
    for (int i = tid; i < nwords; i += FL_THREADS) s_bits[i] = 0;
    const MsgPlan mp = ri->msg;
    const int64_t rowstart = mp.rowstart;
    Thr3 th;
#pragma unroll
    for (int i = 0; i < 3; ++i) { th.tau[i] = mp.tau[i]; th.jx[i] = mp.jx[i]; }
    const float w = mp.weight;
    const int ncc = a.cchunks_per_row;
    const int cc0 = chunk_id * a.csub, cc1 = cc0 + a.csub < ncc ? cc0 + a.csub : ncc;   // the chunk's count chunks
    const uint32_t base = a.chunk_base[(size_t)row * (ncc + 1) + cc0];
    const uint32_t next_base = a.chunk_base[(size_t)row * (ncc + 1) + cc1];
    __syncthreads();
    auto member = [&](uint32_t key, uint32_t j, bool& in0) -> bool {
        in0 = inside_top(th, 0, key, j);
        return in0 || (inside_top(th, 2, key, j) && !inside_top(th, 1, key, j));
    };
    auto mark = [&](uint2 e) {
        const uint32_t rel = e.y >> 6;
        bool in0;
        if (member(key_of_bits(e.x), (uint32_t)c0 + rel, in0)) atomicOr(&s_bits[rel >> 5], 1u << (rel & 31u));
    };
    if (cnt) {
#pragma unroll
        for (int u = 0; u < FL_KEEP; ++u)
            if (lane + 64u * (uint32_t)u < cnt) mark(ent[u]);
    }
    batched_loop<8, 64>(64u * FL_KEEP, cnt, lane, [&](uint32_t i) { return priv[i]; }, [&](uint32_t, uint2 e) { mark(e); });
    __syncthreads();
    // exclusive prefix of the word popcounts
    {
        const int per = (nwords + FL_THREADS - 1) / FL_THREADS;
        const int w0 = tid * per, w1 = w0 + per < nwords ? w0 + per : nwords;
        uint32_t mysum = 0;
        for (int i = w0; i < w1; ++i) mysum += (uint32_t)__popc(s_bits[i]);
        uint32_t total;
        uint32_t run = block_excl_scan<FL_THREADS>(mysum, s_scan, total);
        for (int i = w0; i < w1; ++i) {
            s_pre[i] = run;
            run += (uint32_t)__popc(s_bits[i]);
        }
        if (tid == 0 && base + total != next_base) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    }
    __syncthreads();
    for (int64_t t = c0 / TILE + tid; t * TILE < c1; t += FL_THREADS)
        a.tile_off[(size_t)row * (nt + 1) + t] = base + s_pre[(t * TILE - c0) >> 5];
    auto emit = [&](uint2 e) {
        const uint32_t rel = e.y >> 6, j = (uint32_t)c0 + rel;
        bool in0;
        if (member(key_of_bits(e.x), j, in0)) {
            const uint32_t wd = rel >> 5;
            const uint32_t rank = s_pre[wd] + (uint32_t)__popc(s_bits[wd] & ((1u << (rel & 31u)) - 1u));
            const int64_t at = rowstart + base + rank;
            const float v = __uint_as_float(e.x);
            if (at < a.capacity) { a.idx[at] = j; a.val[at] = in0 ? v : __fmul_rn(v, w); }
        }
    };
    if (cnt) {
#pragma unroll
        for (int u = 0; u < FL_KEEP; ++u)
            if (lane + 64u * (uint32_t)u < cnt) emit(ent[u]);
    }
    batched_loop<8, 64>(64u * FL_KEEP, cnt, lane, [&](uint32_t i) { return priv[i]; }, [&](uint32_t, uint2 e) { emit(e); });
}

// ---------------------------------------------------------------------------------------------------
// host-side launchers
template <int DT, bool VEC>
static mlmc_status launch_select(const mlmc_plan_t* pl, const TopkArgs& a, bool sums, hipStream_t st) {
    const dim3 fgrid(a.fin_wgs, pl->M);
    const int rounds = pl->sample_shift > 0 ? 2 : 1;   // second round: rows whose sampled zones were refuted
    for (int exact_pass = 0; exact_pass < rounds; ++exact_pass) {
        // histogram workgroups per row: enough to spread the row, few enough that the 64 KB flushes stay cheap
        const int64_t nblk = (pl->d + 1023) / 1024;
        const int64_t ns = exact_pass ? nblk : ((nblk >> pl->sample_shift) > 0 ? (nblk >> pl->sample_shift) : 1);
        int64_t hw = ns / 32 > 0 ? ns / 32 : 1;
        // at most two workgroups per CU in all (what the 64 KB of LDS a workgroup holds allow at a time)
        const int64_t hcap = 512 / pl->M > 0 ? 512 / pl->M : 1;
        if (hw > hcap) hw = hcap;
        if (exact_pass && hw > 16) hw = 16;   // the redo round: small grids, they nearly always return at once
        const dim3 hgrid((unsigned)hw, pl->M);
        const dim3 mgrid(exact_pass && pl->chunks_per_row > 32 ? 32 : pl->chunks_per_row, pl->M);
        // the kernels of the redo round exit at once for rows that need none: they are timed as one entry
        const int kh = exact_pass ? K_REDO : K_HIST, ks = exact_pass ? K_REDO : K_SCAN;
        const int km = exact_pass ? K_REDO : K_MAIN;
        MLMC_LAUNCH(kh, st, k_hist<DT, VEC><<<hgrid, HIST_THREADS, 0, st>>>(a, exact_pass));
        MLMC_LAUNCH(ks, st, k_scan<<<pl->M, 1024, 0, st>>>(a, exact_pass));
        if (exact_pass) {
            if (sums) MLMC_LAUNCH(km, st, k_main<DT, VEC, true, true><<<mgrid, MAIN_THREADS, 0, st>>>(a, exact_pass));
            else MLMC_LAUNCH(km, st, k_main<DT, VEC, false, true><<<mgrid, MAIN_THREADS, 0, st>>>(a, exact_pass));
        } else {
            // chunks of 64 K elements or more in four count chunks: two workgroups per chunk, two per CU
            if (pl->chunk >= 65536 && pl->csub == 4) {
                const dim3 grid2(2 * pl->chunks_per_row, pl->M);
                if (sums) MLMC_LAUNCH(km, st, k_main2<DT, VEC, true><<<grid2, M2_THREADS, 0, st>>>(a));
                else MLMC_LAUNCH(km, st, k_main2<DT, VEC, false><<<grid2, M2_THREADS, 0, st>>>(a));
            } else if (sums) {
                MLMC_LAUNCH(km, st, k_main<DT, VEC, true, false><<<mgrid, MAIN_THREADS, 0, st>>>(a, exact_pass));
            } else {
                MLMC_LAUNCH(km, st, k_main<DT, VEC, false, false><<<mgrid, MAIN_THREADS, 0, st>>>(a, exact_pass));
            }
        }
        // the redo round resolves every zone in the ranking launch alone (two launches fewer to pay for when, as
        // nearly always, no row needs it)
        if (!exact_pass) MLMC_LAUNCH(K_FHIST, st, k_fhist<<<fgrid, FN_THREADS, 0, st>>>(a, exact_pass));
        const dim3 rgrid(pl->L + 1 < FIN_WGS ? pl->L + 1 : FIN_WGS, pl->M);
        const int k0 = exact_pass ? K_REDO : K_FINISH, k1 = exact_pass ? K_REDO : K_FINISH1;
        if (sums) {
            if (!exact_pass) MLMC_LAUNCH(k0, st, k_finish<true, 0><<<fgrid, FN_THREADS, 0, st>>>(a, exact_pass));
            MLMC_LAUNCH(k1, st, k_finish<true, 1><<<rgrid, FN_THREADS, 0, st>>>(a, exact_pass));
        } else {
            if (!exact_pass) MLMC_LAUNCH(k0, st, k_finish<false, 0><<<fgrid, FN_THREADS, 0, st>>>(a, exact_pass));
            MLMC_LAUNCH(k1, st, k_finish<false, 1><<<rgrid, FN_THREADS, 0, st>>>(a, exact_pass));
        }
    }
    if (sums) MLMC_LAUNCH(K_NORMS, st, k_norms<<<pl->M, 256, 0, st>>>(a));
    return MLMC_OK;
}

// The plan's side stream and its two events, created on first use (one plan is used from one host thread at a time).
static bool side_stream_ready(const mlmc_plan_t* pl) {
    if (!pl->side_enable || pl->side_state < 0) return false;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (pl->side_state == 1) return dev == pl->side_device;   // a call on another device runs on one stream
    pl->side_state = -1;
    if (hipStreamCreateWithFlags(&pl->side_stream, hipStreamNonBlocking) != hipSuccess) { pl->side_stream = nullptr; return false; }
    if (hipEventCreateWithFlags(&pl->side_fork, hipEventDisableTiming) != hipSuccess) { pl->side_fork = nullptr; return false; }
    if (hipEventCreateWithFlags(&pl->side_join, hipEventDisableTiming) != hipSuccess) { pl->side_join = nullptr; return false; }
    pl->side_device = dev;
    pl->side_state = 1;
    return true;
}

template <int DT, bool VEC>
static mlmc_status launch_compact(const mlmc_plan_t* pl, const TopkArgs& a, hipStream_t st) {
    const dim3 grid(pl->chunks_per_row, pl->M), wgrid(pl->cchunks_per_row, pl->M);
    // rows whose drawn band was staged get their message from the staged lists, the others from a second read
    MLMC_LAUNCH(K_MSGPLAN, st, k_msgplan<<<pl->M, MP_THREADS, 0, st>>>(a));
    // the bitmap and its prefix: chunk / 32 words each, up to 64 KB for the largest chunk; a workgroup may need the
    // limit on dynamic LDS raised for that (static arrays come on top)
    const size_t fl_lds = (size_t)pl->chunk / 32 * 8;
    if (fl_lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)k_filter, hipFuncAttributeMaxDynamicSharedMemorySize, (int)fl_lds) != hipSuccess)
        return MLMC_EHIP;
    // The two message kernels serve disjoint sets of rows and write disjoint parts of the message, and neither fills
    // the machine for its whole run (the second read has the workgroups of one or two rows, the assembly is bound by
    // latency): the second read goes to the plan's side stream, forked from and joined to the caller's stream with
    // events, so the caller still sees one in-order stream.
    hipStream_t sw = st;
    const bool fork = pl->M > 1 && side_stream_ready(pl);
    if (fork) {
        if (hipEventRecord(pl->side_fork, st) != hipSuccess || hipStreamWaitEvent(pl->side_stream, pl->side_fork, 0) != hipSuccess)
            return MLMC_EHIP;
        sw = pl->side_stream;
    }
    MLMC_LAUNCH(K_WRITE, sw, k_write<DT, VEC><<<wgrid, WR_THREADS, 0, sw>>>(a));
    MLMC_LAUNCH(K_FILTER, st, k_filter<<<grid, FL_THREADS, fl_lds, st>>>(a));
    if (fork) {
        if (hipEventRecord(pl->side_join, sw) != hipSuccess || hipStreamWaitEvent(st, pl->side_join, 0) != hipSuccess)
            return MLMC_EHIP;
    }
    return MLMC_OK;
}

mlmc_status topk_zero(const mlmc_plan_t* pl, void* ws, int32_t* dev_status, hipStream_t st) {
    size_t n16 = pl->zero_bytes / 16;
    int blocks = (int)((n16 + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    MLMC_LAUNCH(K_ZERO, st, k_zero<<<blocks, 256, 0, st>>>((uint4*)ws, n16, dev_status));
    return MLMC_OK;
}

mlmc_status topk_select(const mlmc_plan_t* pl, const TopkArgs& a, bool sums, bool vec, hipStream_t st) {
    if (pl->dtype == MLMC_F32)
        return vec ? launch_select<MLMC_F32, true>(pl, a, sums, st) : launch_select<MLMC_F32, false>(pl, a, sums, st);
    return vec ? launch_select<MLMC_BF16, true>(pl, a, sums, st) : launch_select<MLMC_BF16, false>(pl, a, sums, st);
}

mlmc_status topk_compact(const mlmc_plan_t* pl, const TopkArgs& a, bool vec, hipStream_t st) {
    if (pl->dtype == MLMC_F32)
        return vec ? launch_compact<MLMC_F32, true>(pl, a, st) : launch_compact<MLMC_F32, false>(pl, a, st);
    return vec ? launch_compact<MLMC_BF16, true>(pl, a, st) : launch_compact<MLMC_BF16, false>(pl, a, st);
}

}  // namespace mlmc
