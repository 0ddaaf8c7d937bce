// Top-k MLMC on gfx950: exact multi-rank radix select on |g| keys, exact band sums of squares,
// level draw, index-ordered band compaction.
//
// Pipeline per call (all rows at once, one row per blockIdx.y or per workgroup):
//   k_hist1    first-digit histogram of the keys (14 bits: exponent + 6 mantissa bits), LDS atomics
//   k_scan1    per row: bucket of every needed rank threshold, class table bucket -> {sum group | candidate slot}
//   k_pass2    second read: exact sums of squared significands per (exponent, band) group; keys of the
//              boundary buckets are appended to per-slot candidate lists
//   k_finish   per boundary bucket: remaining 17 key bits from the candidate list -> exact threshold key,
//              tie quota, and the exact split of the bucket's sum between the bands it straddles
//   k_norms    big-integer accumulation of the group sums -> correctly rounded fp64 S_l -> Delta_l (Lemma 3.4),
//              then the adaptive level draw (Alg. 3); with known p the draw happens at the start of k_scan1
//   k_compact  index-ordered compaction of base band + drawn band (Eq. (6)) in one read of the rows:
//              per-unit counts chained across workgroups by decoupled look-back
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
// First-digit histogram.  One workgroup = one contiguous chunk of one row.
template <int DT, bool VEC>
__global__ __launch_bounds__(512) void k_hist1(TopkArgs a) {
    __shared__ uint32_t h[NB1];
    const int row = blockIdx.y;
    const int64_t c0 = (int64_t)blockIdx.x * a.chunk;
    const int64_t c1 = c0 + a.chunk < a.d ? c0 + a.chunk : a.d;
    for (int b = threadIdx.x; b < NB1; b += 512) h[b] = 0;
    __syncthreads();
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    uint32_t maxkey = 0;
#pragma unroll 4
    for (int64_t j = c0 + (int64_t)threadIdx.x * 4; j < c1; j += 512 * 4) {
        uint32_t b[4];
        int nv = ld.load4(j, b);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (c < nv) {
                uint32_t key = key_of_bits(b[c]);
                atomicAdd(&h[key >> B1_SHIFT], 1u);
                maxkey = key > maxkey ? key : maxkey;
            }
        }
    }
    __syncthreads();
    uint32_t* gh = a.hist1 + (size_t)row * NB1;
    for (int b = threadIdx.x; b < NB1; b += 512) {
        uint32_t v = h[b];
        if (v) atomicAdd(&gh[b], v);
    }
    if (__ballot(maxkey >= 0x7F800000u) && lane_id() == 0) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
}

// ---------------------------------------------------------------------------------------------------
// Level draw of one row (Alg. 2 / Alg. 3 "Sample l ~ p"), run by one thread.
__device__ void draw_row(const TopkArgs& a, int row, const double* norms_row) {
    double p[LMAX];
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
// Per row: locate thresholds at bucket resolution, assign candidate slots and sum groups, write the table.
__global__ __launch_bounds__(1024) void k_scan1(TopkArgs a) {
    __shared__ uint32_t s_h[NB1];
    __shared__ uint32_t s_scan[17];
    __shared__ uint32_t s_bmask[NB1 / 32];   // bit per bucket: holds a threshold (boundary bucket)
    __shared__ uint32_t s_pmask[NB1 / 32];   // bit per bucket: populated
    __shared__ int32_t s_active[TMAX];
    __shared__ int64_t s_k[TMAX];
    __shared__ uint32_t s_tb[TMAX];          // bucket of threshold t; 0xFFFFFFFF none, 0xFFFFFFFE all
    __shared__ uint32_t s_tr[TMAX];
    __shared__ int32_t s_ng[256];
    __shared__ int32_t s_gbase[256];
    __shared__ int32_t s_nslots, s_lev;
    __shared__ uint32_t s_slotb[SMAX];

    const int row = blockIdx.x, tid = threadIdx.x;
    RowInfo* ri = a.rinfo + row;
    const uint32_t* gh = a.hist1 + (size_t)row * NB1;
    const int L = a.L;

    if (tid == 0) {
        if (!a.all_thresholds) draw_row(a, row, nullptr);  // p is known up front: draw before anything else
        s_lev = a.all_thresholds ? 0 : ri->level;
    }
    for (int b = tid; b < NB1; b += 1024) s_h[b] = gh[b];
    for (int w = tid; w < NB1 / 32; w += 1024) { s_bmask[w] = 0; s_pmask[w] = 0; }
    __syncthreads();
    const int lev = s_lev;
    if (tid <= L) {
        bool act = a.all_thresholds || tid == 0 || tid == lev - 1 || tid == lev;
        s_active[tid] = act;
        int64_t kt = a.k[tid];
        s_k[tid] = kt;
        s_tb[tid] = kt <= 0 ? 0xFFFFFFFFu : 0xFFFFFFFEu;  // overwritten below when 0 < k_t < d
        s_tr[tid] = 0;
    }

    // descending buckets: rb = tid*16 + i  <->  b = NB1 - 1 - rb
    uint32_t hv[16];
    uint32_t sum = 0, pbits = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        hv[i] = s_h[NB1 - 1 - (tid * 16 + i)];
        sum += hv[i];
        pbits |= (hv[i] ? 1u : 0u) << (15 - i);   // bit position = bucket offset inside the aligned 16-block
    }
    if (pbits) {
        const int b0 = NB1 - 16 - tid * 16;        // lowest bucket of this thread's block (multiple of 16)
        atomicOr(&s_pmask[b0 >> 5], pbits << (b0 & 31));
    }
    uint32_t total;
    const uint32_t before = block_excl_scan<1024>(sum, s_scan, total);   // also orders the LDS writes above
    if (tid == 0 && (int64_t)total != a.d) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    if (sum) {
        for (int t = 0; t <= L; ++t) {
            const int64_t kt = s_k[t];
            if (!s_active[t] || kt <= 0 || kt >= a.d) continue;
            if (kt <= (int64_t)before || kt > (int64_t)before + sum) continue;   // not in this thread's 16 buckets
            uint32_t run = before;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if ((int64_t)run < kt && kt <= (int64_t)run + hv[i]) {
                    s_tb[t] = (uint32_t)(NB1 - 1 - (tid * 16 + i));
                    s_tr[t] = (uint32_t)(kt - run);
                }
                run += hv[i];
            }
        }
    }
    __syncthreads();

    if (tid == 0) {
        int ns = 0;
        uint32_t off = 0;
        for (int t = 0; t <= L; ++t) {
            if (!s_active[t]) {
                ri->thr_slot[t] = THR_INACTIVE;
                continue;
            }
            uint32_t b = s_tb[t];
            if (b == 0xFFFFFFFFu) {
                ri->thr_slot[t] = THR_NONE;
                ri->thr_tau[t] = 0xFFFFFFFFu;
                ri->thr_q[t] = 0;
            } else if (b == 0xFFFFFFFEu) {
                ri->thr_slot[t] = THR_ALL;
                ri->thr_tau[t] = 0;
                ri->thr_q[t] = 0xFFFFFFFFu;
            } else {
                if (ns == 0 || s_slotb[ns - 1] != b) {
                    s_slotb[ns] = b;
                    ri->slot_bucket[ns] = b;
                    ri->slot_cnt[ns] = s_h[b];
                    ri->slot_off[ns] = off;
                    off += s_h[b];
                    s_bmask[b >> 5] |= 1u << (b & 31);
                    ++ns;
                }
                ri->thr_slot[t] = ns - 1;
                ri->thr_resid[t] = s_tr[t];
            }
        }
        ri->n_slots = ns;
        s_nslots = ns;
    }
    __syncthreads();

    // One thread per exponent (64 buckets, bit i of the masks <-> bucket 64 E + i).  Boundary buckets cut the
    // exponent into segments; a populated segment lies wholly inside one band and is one sum group:
    // band = number of thresholds whose bucket lies above the segment ("none" thresholds always do).
    const int E = tid;
    uint64_t pm = 0, bm = 0;
    int band_top = 0;
    if (tid < 256) {
        pm = (uint64_t)s_pmask[2 * E] | ((uint64_t)s_pmask[2 * E + 1] << 32);
        bm = (uint64_t)s_bmask[2 * E] | ((uint64_t)s_bmask[2 * E + 1] << 32);
        for (int t = 0; t <= L; ++t) {
            uint32_t tb = s_tb[t];
            band_top += (tb == 0xFFFFFFFFu || (tb != 0xFFFFFFFEu && (int)tb > E * 64 + 63)) ? 1 : 0;
        }
    }
    auto thresholds_in = [&](int b) -> int {
        int n = 0;
        for (int t = 0; t <= L; ++t) n += s_tb[t] == (uint32_t)b ? 1 : 0;
        return n;
    };
    // walks the segments from the top; calls f(segment mask, band, boundary bit below it or -1)
    auto walk = [&](auto&& f) {
        uint64_t rem = bm;
        int hi = 63, band = band_top;
        while (hi >= 0) {
            const int bpos = rem ? 63 - __builtin_clzll(rem) : -1;
            const uint64_t upto_hi = hi == 63 ? ~0ull : ((1ull << (hi + 1)) - 1ull);
            const uint64_t below = bpos < 0 ? 0ull : ((bpos == 63) ? ~0ull : ((1ull << (bpos + 1)) - 1ull));
            f(upto_hi & ~below, band, bpos);
            if (bpos < 0) break;
            band += thresholds_in(E * 64 + bpos);
            rem &= ~(1ull << bpos);
            hi = bpos - 1;
        }
    };
    if (a.all_thresholds) {
        if (tid < 256) {
            int ng = 0;
            walk([&](uint64_t seg, int, int) { ng += (pm & ~bm & seg) ? 1 : 0; });
            s_ng[tid] = ng;
        }
        __syncthreads();
        if (tid < 64) {  // exclusive scan over exponents, highest first: lane l owns exponents 255-4l .. 252-4l
            int v[4], sum4 = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[i] = s_ng[255 - (tid * 4 + i)]; sum4 += v[i]; }
            int inc = sum4;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                int u = __shfl_up(inc, o, 64);
                if (tid >= o) inc += u;
            }
            int run = inc - sum4;
#pragma unroll
            for (int i = 0; i < 4; ++i) { s_gbase[255 - (tid * 4 + i)] = run; run += v[i]; }
            if (tid == 63) {
                ri->n_groups = run;
                ri->rep_shift = run <= 32 ? 6 : run <= 64 ? 5 : run <= 128 ? 4 : run <= 256 ? 3 : 2;
            }
        }
        __syncthreads();
    }
    if (tid < 256) {
        uint16_t* tab = a.table + (size_t)row * NB1 + E * 64;
        if (bm == 0) {  // whole exponent in one band (or unpopulated / not needed)
            uint16_t code = CODE_IGNORE;
            if (a.all_thresholds && pm) {
                int gid = s_gbase[E];
                if (gid < GMAX) {
                    ri->g_exp[gid] = (uint16_t)(E ? E : 1);
                    ri->g_band[gid] = (uint16_t)band_top;
                    code = (uint16_t)gid;
                }
            }
            uint32_t c2 = (uint32_t)code | ((uint32_t)code << 16);
            uint4 v = make_uint4(c2, c2, c2, c2);
            uint4* dst = (uint4*)tab;
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[i] = v;
        } else {
            int gid = a.all_thresholds ? s_gbase[E] : 0;
            const int ns = s_nslots;
            walk([&](uint64_t seg, int band, int bpos) {
                uint16_t gcode = CODE_IGNORE;
                if (a.all_thresholds && (pm & ~bm & seg)) {
                    if (gid < GMAX) {
                        ri->g_exp[gid] = (uint16_t)(E ? E : 1);
                        ri->g_band[gid] = (uint16_t)band;
                        gcode = (uint16_t)gid;
                    }
                    ++gid;
                }
                uint64_t sm = seg;
                while (sm) {
                    const int i = __builtin_ctzll(sm);
                    sm &= sm - 1;
                    tab[i] = ((pm >> i) & 1ull) ? gcode : CODE_IGNORE;
                }
                if (bpos >= 0) {
                    int sl = 0;
                    for (int u = 0; u < ns; ++u) if (s_slotb[u] == (uint32_t)(E * 64 + bpos)) sl = u;
                    tab[bpos] = (uint16_t)(CODE_CAND | sl);
                }
            });
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Second read of the rows: band sums (SUMS) and candidate extraction.
constexpr int P2_THREADS = 1024;
constexpr int P2_WAVES = P2_THREADS / 64;
constexpr int P2_CAP = 512;  // staged candidates per wave

template <int DT, bool VEC, bool SUMS>
__global__ __launch_bounds__(P2_THREADS) void k_pass2(TopkArgs a) {
    __shared__ uint16_t s_tab[NB1];
    __shared__ unsigned long long s_acc[SUMS ? ACC_SLOTS : 1];
    __shared__ uint32_t s_key[P2_WAVES][P2_CAP];
    __shared__ uint32_t s_meta[P2_WAVES][P2_CAP];
    __shared__ uint32_t s_cnt[P2_WAVES][SMAX];
    __shared__ uint32_t s_base[P2_WAVES][SMAX];
    __shared__ uint32_t s_slot_off[SMAX];

    const int row = blockIdx.y, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = tid >> 6;
    const RowInfo* ri = a.rinfo + row;
    RowAcc* ra = a.racc + row;
    const int nslots = ri->n_slots;
    const int rep_shift = SUMS ? ri->rep_shift : 0;
    const int G = SUMS ? ri->n_groups : 0;
    {
        const uint4* src = (const uint4*)(a.table + (size_t)row * NB1);
        uint4* dst = (uint4*)s_tab;
        for (int i = tid; i < NB1 * 2 / 16; i += P2_THREADS) dst[i] = src[i];
    }
    if (SUMS) for (int i = tid; i < ACC_SLOTS; i += P2_THREADS) s_acc[i] = 0ull;
    if (tid < SMAX) s_slot_off[tid] = tid < nslots ? ri->slot_off[tid] : 0u;
    if (lane < SMAX) s_cnt[wave][lane] = 0;
    __syncthreads();

    const int64_t c0 = (int64_t)blockIdx.x * a.chunk;
    const int64_t c1 = c0 + a.chunk < a.d ? c0 + a.chunk : a.d;
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    uint32_t* cand_row = a.cand + (size_t)row * (size_t)a.d;
    const uint32_t rep_mask = (1u << rep_shift) - 1u;
    uint32_t nst = 0;  // wave-uniform: staged candidates

    auto flush = [&]() {
        wave_lds_sync();
        if ((int)lane < nslots) {
            uint32_t n = s_cnt[wave][lane];
            uint32_t base = 0;
            if (n) base = atomicAdd(&ra->slot_fill[lane], n);
            s_base[wave][lane] = s_slot_off[lane] + base;
            s_cnt[wave][lane] = 0;
        }
        wave_lds_sync();
        for (uint32_t i = lane; i < nst; i += 64) {
            uint32_t meta = s_meta[wave][i];
            uint32_t pos = s_base[wave][meta >> 24] + (meta & 0xFFFFFFu);
            if ((int64_t)pos < a.d) cand_row[pos] = s_key[wave][i];
            else atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        }
        wave_lds_sync();
        nst = 0;
    };

    // every lane of a wave runs the same number of iterations (lanes past the chunk end load nothing)
    for (int64_t jw = c0 + (int64_t)wave * 256; jw < c1; jw += P2_THREADS * 4) {
        const int64_t j = jw + (int64_t)lane * 4;
        uint32_t b[4];
        int nv = j < c1 ? ld.load4(j, b) : 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t key = key_of_bits(b[c]);
            uint16_t code = c < nv ? s_tab[key >> B1_SHIFT] : CODE_IGNORE;
            if (SUMS && code < CODE_IGNORE)
                atomicAdd(&s_acc[((uint32_t)code << rep_shift) + (lane & rep_mask)], (unsigned long long)sig_square(key));
            bool is_cand = (code & CODE_CAND) != 0;
            uint64_t m = __ballot(is_cand);
            if (m) {
                if (is_cand) {
                    uint32_t s = code & 0xFFu;
                    uint32_t pos = nst + mbcnt(m);
                    uint32_t lr = atomicAdd(&s_cnt[wave][s], 1u);
                    s_key[wave][pos] = key;
                    s_meta[wave][pos] = (s << 24) | lr;
                }
                nst += (uint32_t)__popcll(m);
            }
        }
        if (nst > P2_CAP - 256) flush();
    }
    flush();
    if (SUMS) {
        __syncthreads();
        if (tid < G) {
            unsigned long long lo = 0, hi = 0;
            const int R = 1 << rep_shift;
            for (int r = 0; r < R; ++r) {
                unsigned long long v = s_acc[(tid << rep_shift) + r];
                lo += v & 0xFFFFFFFFull;
                hi += v >> 32;
            }
            if (lo) atomicAdd((unsigned long long*)&ra->gsum[tid][0], lo);
            if (hi) atomicAdd((unsigned long long*)&ra->gsum[tid][1], hi);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// One workgroup per (boundary bucket, row): resolve the remaining 17 key bits on the candidate list.
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

template <bool SUMS>
__global__ __launch_bounds__(FN_THREADS) void k_finish(TopkArgs a) {
    __shared__ uint32_t hA[512];
    __shared__ uint32_t hB[TMAX][256];
    __shared__ unsigned long long pacc[SUMS ? TMAX + 1 : 1][64][2];
    __shared__ int32_t s_n;
    __shared__ int32_t s_t[TMAX];
    __shared__ uint32_t s_res[TMAX], s_sb[TMAX], s_tau[TMAX], s_q[TMAX], s_eq[TMAX];
    __shared__ int32_t s_sub[TMAX];
    __shared__ uint8_t s_sub_of_sb[512];

    const int s = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = tid >> 6;
    RowInfo* ri = a.rinfo + row;
    RowAcc* ra = a.racc + row;
    if (s >= ri->n_slots) return;
    const uint32_t n = ri->slot_cnt[s];
    const uint32_t bucket = ri->slot_bucket[s];
    const uint32_t* list = a.cand + (size_t)row * (size_t)a.d + ri->slot_off[s];
    const int L = a.L;

    for (int i = tid; i < 512; i += FN_THREADS) { hA[i] = 0; s_sub_of_sb[i] = 0xFF; }
    for (int i = tid; i < TMAX * 256; i += FN_THREADS) (&hB[0][0])[i] = 0;
    if (SUMS) for (int i = tid; i < (TMAX + 1) * 64 * 2; i += FN_THREADS) (&pacc[0][0][0])[i] = 0ull;
    if (tid == 0) {
        int m = 0;
        for (int t = 0; t <= L; ++t)
            if (ri->thr_slot[t] == s) { s_t[m] = t; s_res[m] = ri->thr_resid[t]; ++m; }
        s_n = m;
        if (ra->slot_fill[s] != n) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    }
    __syncthreads();
    const int nthr = s_n;

    // A: bits 16..8
#pragma unroll 4
    for (uint32_t i = tid; i < n; i += FN_THREADS) atomicAdd(&hA[(list[i] >> 8) & 511u], 1u);
    __syncthreads();
    if (wave == 0) {
        for (int u = 0; u < nthr; ++u) {
            int sb;
            uint32_t rin, cnt;
            wave_rank_search<8>(hA, s_res[u], sb, rin, cnt);
            if (lane == 0) { s_sb[u] = (uint32_t)sb; s_res[u] = rin; }
        }
        wave_lds_sync();
        if (lane == 0) {
            int nsub = 0;
            for (int u = 0; u < nthr; ++u) {
                if (u == 0 || s_sb[u] != s_sb[u - 1]) { s_sub_of_sb[s_sb[u]] = (uint8_t)nsub; ++nsub; }
                s_sub[u] = nsub - 1;
            }
        }
    }
    __syncthreads();

    // B: bits 7..0 of the keys in the thresholds' sub-bins
#pragma unroll 4
    for (uint32_t i = tid; i < n; i += FN_THREADS) {
        uint32_t key = list[i];
        uint32_t u = s_sub_of_sb[(key >> 8) & 511u];
        if (u != 0xFF) atomicAdd(&hB[u][key & 255u], 1u);
    }
    __syncthreads();
    for (int u = wave; u < nthr; u += FN_THREADS / 64) {
        int lb;
        uint32_t rin, cnt;
        wave_rank_search<4>(hB[s_sub[u]], s_res[u], lb, rin, cnt);
        if (lane == 0) {
            uint32_t tau = (bucket << B1_SHIFT) | (s_sb[u] << 8) | (uint32_t)lb;
            s_tau[u] = tau;
            s_q[u] = rin;
            s_eq[u] = cnt;
            ri->thr_tau[s_t[u]] = tau;
            ri->thr_q[s_t[u]] = rin;
            if (rin > cnt || rin == 0) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        }
    }
    if (!SUMS) return;
    __syncthreads();

    // C: exact sums of the parts the thresholds cut the bucket into (piece j: keys strictly between
    // threshold j-1 and threshold j; entries equal to a threshold key are added arithmetically)
#pragma unroll 4
    for (uint32_t i = tid; i < n; i += FN_THREADS) {
        uint32_t key = list[i];
        int j = 0;
        bool eq = false;
        for (int u = 0; u < nthr; ++u) {
            uint32_t tau = s_tau[u];
            j += tau > key ? 1 : 0;
            eq |= tau == key;
        }
        if (!eq) {
            unsigned long long sq = sig_square(key);
            atomicAdd(&pacc[j][lane][0], sq & 0xFFFFFFFFull);
            atomicAdd(&pacc[j][lane][1], sq >> 32);
        }
    }
    __syncthreads();
    if (tid <= nthr) {
        const int j = tid;
        unsigned long long lo = 0, hi = 0;
        for (int l = 0; l < 64; ++l) { lo += pacc[j][l][0]; hi += pacc[j][l][1]; }
        hi += lo >> 32;
        lo &= 0xFFFFFFFFull;
        // entries equal to threshold key tau_u: q_u of them are within the top k_{t_u}
        auto add_ties = [&](uint32_t tau, unsigned long long cnt) {
            unsigned long long sq = sig_square(tau);
            lo += cnt * (sq & 0xFFFFFFFFull);
            hi += cnt * (sq >> 32);
            hi += lo >> 32;
            lo &= 0xFFFFFFFFull;
        };
        if (j < nthr) {
            unsigned long long prevq = (j > 0 && s_tau[j - 1] == s_tau[j]) ? s_q[j - 1] : 0ull;
            add_ties(s_tau[j], (unsigned long long)s_q[j] - prevq);
        }
        if (j > 0 && (j == nthr || s_tau[j] != s_tau[j - 1]))
            add_ties(s_tau[j - 1], (unsigned long long)s_eq[j - 1] - s_q[j - 1]);
        const int pidx = s_t[0] + s + j;
        if (pidx >= PMAX) { atomicOr(a.dev_status, MLMC_DEV_INTERNAL); return; }
        Piece* pc = &ra->pieces[pidx];
        uint32_t E = bucket >> 6;
        pc->exp = (int32_t)(E ? E : 1u);
        pc->lo = lo;
        pc->hi = hi;
        pc->band_plus1 = (j < nthr ? s_t[j] : s_t[nthr - 1] + 1) + 1;
    }
}

// ---------------------------------------------------------------------------------------------------
// Delta_l (Lemma 3.4) from the exact group and piece sums, then the adaptive draw.  One workgroup per row,
// one thread per band; the 640-bit accumulators live in LDS.
struct BigAcc {
    uint32_t* w;  // 20 words
    __device__ void clear() { for (int i = 0; i < 20; ++i) w[i] = 0; }
    __device__ void add(uint64_t v, int shift) {  // += v << shift
        if (!v) return;
        int wi = shift >> 5, bs = shift & 31;
        uint32_t parts[3];
        if (bs == 0) {
            parts[0] = (uint32_t)v;
            parts[1] = (uint32_t)(v >> 32);
            parts[2] = 0;
        } else {
            parts[0] = (uint32_t)(v << bs);
            parts[1] = (uint32_t)(v >> (32 - bs));
            parts[2] = (uint32_t)(v >> (64 - bs));
        }
        uint64_t carry = 0;
        for (int i = 0; i < 3 || carry; ++i) {
            if (wi + i >= 20) break;
            uint64_t sum = (uint64_t)w[wi + i] + (i < 3 ? parts[i] : 0u) + carry;
            w[wi + i] = (uint32_t)sum;
            carry = sum >> 32;
        }
    }
    // value * 2^-298 rounded to nearest-even fp64
    __device__ double to_double() const {
        int top = -1;
        for (int i = 19; i >= 0; --i) if (w[i]) { top = i; break; }
        if (top < 0) return 0.0;
        const int P = top * 32 + 31 - __clz(w[top]);  // index of the most significant set bit
        auto word = [&](int i) -> uint64_t { return (i < 0 || i >= 20) ? 0ull : (uint64_t)w[i]; };
        if (P <= 52) {  // fits the significand exactly
            uint64_t v = word(0) | (word(1) << 32);
            return ldexp((double)v, -298);
        }
        // bits P .. P-52 as the significand, bit P-53 as guard, anything below as sticky
        const int g = P - 53;                       // guard bit index (>= 0)
        const int wi = g >> 5, bs = g & 31;         // window starting at the guard bit: 54 bits needed
        uint64_t win = (word(wi) >> bs) | (word(wi + 1) << (32 - bs));
        if (bs > 0) win |= word(wi + 2) << (64 - bs);
        const uint32_t guard = (uint32_t)(win & 1ull);
        uint64_t mant = (win >> 1) & ((1ull << 53) - 1ull);
        bool sticky = bs ? (w[wi] & ((1u << bs) - 1u)) != 0 : false;
        for (int i = wi - 1; i >= 0 && !sticky; --i) sticky = w[i] != 0;
        if (guard && (sticky || (mant & 1ull))) ++mant;
        return ldexp((double)mant, P - 52 - 298);
    }
};

__global__ __launch_bounds__(256) void k_norms(TopkArgs a) {
    __shared__ uint32_t s_big[TMAX][20];
    __shared__ unsigned long long s_glo[GMAX], s_ghi[GMAX];
    __shared__ uint16_t s_gexp[GMAX], s_gband[GMAX];
    __shared__ Piece s_pc[PMAX];
    __shared__ double s_norm[LMAX];
    const int row = blockIdx.x, tid = threadIdx.x;
    const RowInfo* ri = a.rinfo + row;
    const RowAcc* ra = a.racc + row;
    const int G = ri->n_groups;
    for (int g = tid; g < G; g += 256) {
        s_glo[g] = ra->gsum[g][0];
        s_ghi[g] = ra->gsum[g][1];
        s_gexp[g] = ri->g_exp[g];
        s_gband[g] = ri->g_band[g];
    }
    for (int p = tid; p < PMAX; p += 256) s_pc[p] = ra->pieces[p];
    __syncthreads();
    const int l = tid;
    if (l >= 1 && l <= a.L) {
        BigAcc acc;
        acc.w = s_big[l];
        acc.clear();
        for (int g = 0; g < G; ++g) {
            if (s_gband[g] == l) {
                int sh = 2 * ((int)s_gexp[g] - 1);
                acc.add(s_glo[g], sh);
                acc.add(s_ghi[g], sh + 32);
            }
        }
        for (int p = 0; p < PMAX; ++p) {
            if (s_pc[p].band_plus1 == l + 1) {
                int sh = 2 * (s_pc[p].exp - 1);
                acc.add(s_pc[p].lo, sh);
                acc.add(s_pc[p].hi, sh + 32);
            }
        }
        double nrm = __dsqrt_rn(acc.to_double());
        s_norm[l - 1] = nrm;
        a.norms[(size_t)row * a.L + (l - 1)] = nrm;
        if (a.norms_user) a.norms_user[(size_t)row * a.L + (l - 1)] = nrm;
    }
    __syncthreads();
    if (tid == 0 && a.draw_mode == 3) draw_row(a, row, s_norm);
}

// ---------------------------------------------------------------------------------------------------
// Level draw for all rows of the bit-wise path (one workgroup).
__global__ __launch_bounds__(1024) void k_draw(DrawArgs a) {
    const int r = threadIdx.x;
    if (r < a.M) {
        double p[LMAX];
        const int L = a.L;
        for (int l = 0; l < L; ++l) p[l] = a.p_fixed[l];
        uint32_t x = philox_word0(a.seed, a.step, (uint32_t)r);
        int level = draw_from_p(p, L, x);
        double pl = p[level - 1];
        RowInfo* ri = a.rinfo + r;
        ri->level = level;
        ri->weight = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
        ri->draw_x = x;
        a.level[r] = level;
    }
}

// ---------------------------------------------------------------------------------------------------
// Compaction in one read.  A unit = CW waves x 1024 consecutive elements of one row.  Workgroups take units
// from a ticket counter (rows interleaved, so every unit's predecessor in its row has an earlier ticket
// and is already running); each unit publishes its counts (three tie counts, one output count) as
// 64-bit descriptors and obtains its exclusive prefixes by decoupled look-back over its predecessors.
struct Thr3 {
    uint32_t tau[3], q[3];
};
__device__ __forceinline__ Thr3 load_thr3(const RowInfo* ri) {
    Thr3 t;
    const int lev = ri->level;
    const int ts[3] = {0, lev - 1, lev};
#pragma unroll
    for (int i = 0; i < 3; ++i) { t.tau[i] = ri->thr_tau[ts[i]]; t.q[i] = ri->thr_q[ts[i]]; }
    return t;
}

constexpr unsigned long long DESC_AGG = 1ull << 62;   // value = this unit's own count
constexpr unsigned long long DESC_PRE = 2ull << 62;   // value = inclusive prefix up to and including this unit
constexpr unsigned long long DESC_VAL = 0xFFFFFFFFull;
constexpr uint32_t LOOKBACK_SPIN_MAX = 1u << 22;      // bounded wait: about a second of polling

__device__ __forceinline__ void desc_store(unsigned long long* p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long desc_load(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Run by one whole wave.  drow: descriptors of this row, [units][4]; chain c.  Publishes the unit's count,
// returns the sum of the counts of units 0..unit-1, then publishes the inclusive prefix.
__device__ uint32_t lookback(unsigned long long* drow, int c, int64_t unit, uint32_t agg, int32_t* dev_status) {
    const uint32_t lane = lane_id();
    unsigned long long* mine = drow + unit * 4 + c;
    if (unit == 0) {
        if (lane == 0) desc_store(mine, DESC_PRE | agg);
        return 0;
    }
    if (lane == 0) desc_store(mine, DESC_AGG | agg);
    uint32_t excl = 0;
    int64_t pos = unit - 1;  // the window is units pos, pos-1, ..., pos-63 (lane 0 = nearest)
    uint32_t spin = 0;
    bool done = false;
    while (!done) {
        const int64_t u = pos - (int64_t)lane;
        unsigned long long v = u >= 0 ? desc_load(drow + u * 4 + c) : DESC_PRE;
        const uint32_t flag = (uint32_t)(v >> 62);
        const uint64_t m_inv = __ballot(flag == 0);
        const uint64_t m_pre = __ballot(flag == 2);
        const int first_inv = m_inv ? (int)__builtin_ctzll(m_inv) : 64;
        const int first_pre = m_pre ? (int)__builtin_ctzll(m_pre) : 64;
        if (first_pre < first_inv) {          // a prefix is reachable through published counts
            uint32_t part = (int)lane <= first_pre ? (uint32_t)(v & DESC_VAL) : 0u;
            excl += wave_sum(part);
            done = true;
        } else if (first_inv == 64) {         // 64 published counts, no prefix yet: take them, look further back
            excl += wave_sum((uint32_t)(v & DESC_VAL));
            pos -= 64;
        } else {                              // a predecessor has not published yet: poll again
            __builtin_amdgcn_s_sleep(8);
            if (++spin >= LOOKBACK_SPIN_MAX) {
                if (lane == 0) atomicOr(dev_status, MLMC_DEV_INTERNAL);
                done = true;
            }
        }
    }
    if (lane == 0) desc_store(mine, DESC_PRE | (unsigned long long)(excl + agg));
    return excl;
}

template <int DT, bool VEC, int CW>
__global__ __launch_bounds__(CW * 64) void k_compact(TopkArgs a) {
    constexpr int NT = CW * 64;
    constexpr int UNIT = CW * 1024;
    __shared__ int64_t s_rowoff[MLMC_MAX_WORKERS + 1];
    __shared__ uint32_t s_ticket;
    __shared__ uint32_t s_wtie[3][CW];
    __shared__ uint32_t s_wemit[CW];
    __shared__ uint32_t s_pre[4];
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = tid >> 6;
    const int64_t nt = a.ntiles;

    // row offsets of the messages from the drawn levels (every workgroup keeps a copy; workgroup 0 writes them)
    for (int i = tid; i < a.M; i += NT) {
        const int lev = a.rinfo[i].level;
        s_rowoff[i + 1] = a.k[0] + a.k[lev] - a.k[lev - 1];
    }
    __syncthreads();
    if (tid == 0) {
        int64_t run = 0;
        s_rowoff[0] = 0;
        for (int i = 0; i < a.M; ++i) { int64_t n = s_rowoff[i + 1]; s_rowoff[i] = run; run += n; }
        s_rowoff[a.M] = run;
        if (blockIdx.x == 0 && run > a.capacity) atomicOr(a.dev_status, MLMC_DEV_CAPACITY);
    }
    __syncthreads();
    if (blockIdx.x == 0)
        for (int i = tid; i <= a.M; i += NT) a.row_off[i] = s_rowoff[i];

    const uint32_t total_units = (uint32_t)(a.units_per_row * a.M);
    while (true) {
        if (tid == 0) s_ticket = atomicAdd(a.ticket, 1u);
        __syncthreads();
        const uint32_t ticket = s_ticket;
        if (ticket >= total_units) break;
        const int row = (int)(ticket % (uint32_t)a.M);
        const int64_t unit = ticket / (uint32_t)a.M;
        const RowInfo* ri = a.rinfo + row;
        const Thr3 th = load_thr3(ri);
        const float w = ri->weight;
        RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
        const int64_t wbase = unit * UNIT + (int64_t)wave * 1024;  // this wave's 1024 elements

        uint32_t bits[16];
        uint32_t valid = 0;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            uint32_t b[4];
            int nv = ld.load4(wbase + it * 256 + lane * 4, b);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                bits[it * 4 + c] = b[c];
                if (c < nv) valid |= 1u << (it * 4 + c);
            }
        }
        uint32_t above[3] = {0, 0, 0}, equal[3] = {0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            uint32_t key = key_of_bits(bits[e]);
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                above[k] |= (key > th.tau[k] ? 1u : 0u) << e;
                equal[k] |= (key == th.tau[k] ? 1u : 0u) << e;
            }
        }
#pragma unroll
        for (int k = 0; k < 3; ++k) { above[k] &= valid; equal[k] &= valid; }
        uint32_t in[3] = {above[0], above[1], above[2]};
        {
            uint32_t t0 = wave_sum(__popc(equal[0])), t1 = wave_sum(__popc(equal[1])), t2 = wave_sum(__popc(equal[2]));
            uint32_t e0 = wave_sum(__popc(in[0] | (in[2] & ~in[1])));  // output count if the unit has no ties
            if (lane == 0) { s_wtie[0][wave] = t0; s_wtie[1][wave] = t1; s_wtie[2][wave] = t2; s_wemit[wave] = e0; }
        }
        __syncthreads();
        uint32_t ut[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) ut[k] = wave_sum(lane < (uint32_t)CW ? s_wtie[k][lane] : 0u);
        const bool any_tie = (ut[0] | ut[1] | ut[2]) != 0;  // uniform over the workgroup
        unsigned long long* drow = a.desc + (size_t)row * (size_t)a.units_per_row * 4;
        if (wave < 3) {
            uint32_t ex = lookback(drow, (int)wave, unit, ut[wave], a.dev_status);
            if (lane == 0) s_pre[wave] = ex;
        } else if (wave == 3 && !any_tie) {
            uint32_t agg = wave_sum(lane < (uint32_t)CW ? s_wemit[lane] : 0u);
            uint32_t ex = lookback(drow, 3, unit, agg, a.dev_status);
            if (lane == 0) s_pre[3] = ex;
        }
        __syncthreads();
        if (any_tie) {
            // rank the entries equal to a threshold key in index order; the first q_k of the row are inside
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                if (ut[k] == 0) continue;
                uint64_t r0 = s_pre[k];
                for (uint32_t w2 = 0; w2 < wave; ++w2) r0 += s_wtie[k][w2];
                const uint64_t q = th.q[k];
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    uint32_t tot;
                    uint32_t ex = wave_excl_small(__popc((equal[k] >> (it * 4)) & 0xFu), tot);
                    uint64_t r = r0 + ex;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int e = it * 4 + c;
                        if ((equal[k] >> e) & 1u) {
                            if (r < q) in[k] |= 1u << e;
                            ++r;
                        }
                    }
                    r0 += tot;
                }
            }
            uint32_t e1 = wave_sum(__popc(in[0] | (in[2] & ~in[1])));
            __syncthreads();  // every wave has read the tentative s_wemit users (wave 3 did not use it)
            if (lane == 0) s_wemit[wave] = e1;
            __syncthreads();
            if (wave == 3) {
                uint32_t agg = wave_sum(lane < (uint32_t)CW ? s_wemit[lane] : 0u);
                uint32_t ex = lookback(drow, 3, unit, agg, a.dev_status);
                if (lane == 0) s_pre[3] = ex;
            }
            __syncthreads();
        }
        const uint32_t emit = in[0] | (in[2] & ~in[1]);
        uint32_t wave_pre = s_pre[3];  // entries of this row before this wave's elements
        for (uint32_t w2 = 0; w2 < wave; ++w2) wave_pre += s_wemit[w2];
        if ((wave & 3u) == 0 && lane == 0) {
            const int64_t tile = unit * (UNIT / TILE) + (wave >> 2);
            if (tile < nt) a.tile_off[(size_t)row * (nt + 1) + tile] = wave_pre;
        }
        if (unit == a.units_per_row - 1 && wave == CW - 1 && lane == 0) {
            const uint32_t total = wave_pre + s_wemit[wave];
            a.tile_off[(size_t)row * (nt + 1) + nt] = total;
            if ((int64_t)total != s_rowoff[row + 1] - s_rowoff[row]) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
        }
        int64_t pos0 = s_rowoff[row] + wave_pre;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            uint32_t tot;
            uint32_t ex = wave_excl_small(__popc((emit >> (it * 4)) & 0xFu), tot);
            int64_t pos = pos0 + ex;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int e = it * 4 + c;
                if ((emit >> e) & 1u) {
                    if (pos < a.capacity) {
                        float v = __uint_as_float(bits[e]);
                        a.idx[pos] = (uint32_t)(wbase + it * 256 + lane * 4 + c);
                        a.val[pos] = ((in[0] >> e) & 1u) ? v : __fmul_rn(v, w);
                    }
                    ++pos;
                }
            }
            pos0 += tot;
        }
        __syncthreads();  // LDS reuse by the next unit
    }
}

// ---------------------------------------------------------------------------------------------------
// host-side launchers
template <int DT, bool VEC>
static mlmc_status launch_select(const mlmc_plan_t* pl, const TopkArgs& a, bool sums, hipStream_t st) {
    dim3 grid(pl->chunks_per_row, pl->M);
    MLMC_LAUNCH(K_HIST1, st, k_hist1<DT, VEC><<<grid, 512, 0, st>>>(a));
    MLMC_LAUNCH(K_SCAN1, st, k_scan1<<<pl->M, 1024, 0, st>>>(a));
    if (sums) MLMC_LAUNCH(K_PASS2, st, k_pass2<DT, VEC, true><<<grid, P2_THREADS, 0, st>>>(a));
    else MLMC_LAUNCH(K_PASS2, st, k_pass2<DT, VEC, false><<<grid, P2_THREADS, 0, st>>>(a));
    dim3 fgrid(pl->L + 1, pl->M);
    if (sums) MLMC_LAUNCH(K_FINISH, st, k_finish<true><<<fgrid, FN_THREADS, 0, st>>>(a));
    else MLMC_LAUNCH(K_FINISH, st, k_finish<false><<<fgrid, FN_THREADS, 0, st>>>(a));
    if (sums) MLMC_LAUNCH(K_NORMS, st, k_norms<<<pl->M, 256, 0, st>>>(a));
    return MLMC_OK;
}

template <int DT, bool VEC>
static mlmc_status launch_compact(const mlmc_plan_t* pl, const TopkArgs& a, hipStream_t st) {
    const int64_t units = pl->units_per_row * pl->M;
    if (pl->cwaves == 8) {
        int grid = (int)(units < 1024 ? units : 1024);
        MLMC_LAUNCH(K_COMPACT, st, k_compact<DT, VEC, 8><<<grid, 512, 0, st>>>(a));
    } else {
        int grid = (int)(units < 512 ? units : 512);
        MLMC_LAUNCH(K_COMPACT, st, k_compact<DT, VEC, 16><<<grid, 1024, 0, st>>>(a));
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

mlmc_status topk_draw(const DrawArgs& da, hipStream_t st) {
    MLMC_LAUNCH(K_DRAW, st, k_draw<<<1, 1024, 0, st>>>(da));
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
