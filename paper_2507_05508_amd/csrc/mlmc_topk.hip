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
//   k_norms    big-integer accumulation of the group sums -> correctly rounded fp64 S_l -> Delta_l (Lemma 3.4)
//   k_draw     p_l, integer CDF, Philox draw, weight, row offsets (Alg. 2 / Alg. 3 "Sample l")
//   k_count / k_tilescan / k_write   index-ordered compaction of base band + drawn band (Eq. (6))
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
// Per row: locate thresholds at bucket resolution, assign candidate slots and sum groups, write the table.
__global__ __launch_bounds__(1024) void k_scan1(TopkArgs a) {
    __shared__ uint32_t s_h[NB1];
    __shared__ uint32_t s_scan[17];
    __shared__ uint32_t s_bmask[NB1 / 32];
    __shared__ int32_t s_active[TMAX];
    __shared__ uint32_t s_tb[TMAX];      // bucket of threshold t; 0xFFFFFFFF none, 0xFFFFFFFE all
    __shared__ uint32_t s_tr[TMAX];
    __shared__ int32_t s_ng[256];
    __shared__ int32_t s_gbase[256];
    __shared__ int32_t s_nslots;
    __shared__ uint32_t s_slotb[SMAX];

    const int row = blockIdx.x, tid = threadIdx.x;
    RowInfo* ri = a.rinfo + row;
    const uint32_t* gh = a.hist1 + (size_t)row * NB1;
    const int L = a.L;
    const int lev = ri->level;  // valid when !all_thresholds (draw ran first)

    for (int b = tid; b < NB1; b += 1024) s_h[b] = gh[b];
    for (int w = tid; w < NB1 / 32; w += 1024) s_bmask[w] = 0;
    if (tid <= L) {
        bool act = a.all_thresholds || tid == 0 || tid == lev - 1 || tid == lev;
        s_active[tid] = act;
        int64_t kt = a.k[tid];
        s_tb[tid] = kt <= 0 ? 0xFFFFFFFFu : 0xFFFFFFFEu;  // overwritten below when 0 < k_t < d
        s_tr[tid] = 0;
    }
    __syncthreads();

    // descending buckets: rb = tid*16 + i  <->  b = NB1 - 1 - rb
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += s_h[NB1 - 1 - (tid * 16 + i)];
    uint32_t total;
    uint32_t running = block_excl_scan<1024>(sum, s_scan, total);
    if (tid == 0 && (int64_t)total != a.d) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    if (sum) {
        for (int i = 0; i < 16; ++i) {
            int b = NB1 - 1 - (tid * 16 + i);
            uint32_t hv = s_h[b];
            if (hv) {
                for (int t = 0; t <= L; ++t) {
                    int64_t kt = a.k[t];
                    if (s_active[t] && kt > 0 && kt < a.d && (int64_t)running < kt && kt <= (int64_t)running + hv) {
                        s_tb[t] = (uint32_t)b;
                        s_tr[t] = (uint32_t)(kt - running);
                    }
                }
                running += hv;
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

    // band of a bucket that is wholly inside one band: number of thresholds whose bucket lies above it
    auto band_of = [&](int b) -> int {
        int n = 0;
        for (int t = 0; t <= L; ++t) {
            uint32_t tb = s_tb[t];
            bool above = tb == 0xFFFFFFFFu ? true : (tb == 0xFFFFFFFEu ? false : (int)tb > b);
            n += above ? 1 : 0;
        }
        return n;  // L + 1 = below the last threshold (k_L < d): in no band
    };

    if (a.all_thresholds) {
        if (tid < 256) {
            int ng = 0, prev = -1;
            for (int i = 63; i >= 0; --i) {
                int b = tid * 64 + i;
                if (s_h[b] && !((s_bmask[b >> 5] >> (b & 31)) & 1u)) {
                    int band = band_of(b);
                    if (band != prev) { ++ng; prev = band; }
                }
            }
            s_ng[tid] = ng;
        }
        __syncthreads();
        if (tid == 0) {
            int run = 0;
            for (int e = 255; e >= 0; --e) { s_gbase[e] = run; run += s_ng[e]; }
            ri->n_groups = run;
            int rs = run <= 32 ? 6 : run <= 64 ? 5 : run <= 128 ? 4 : run <= 256 ? 3 : 2;
            ri->rep_shift = rs;
        }
        __syncthreads();
    }
    if (tid < 256) {
        uint16_t* tab = a.table + (size_t)row * NB1;
        int gid = a.all_thresholds ? s_gbase[tid] - 1 : 0, prev = -1;
        const int ns = s_nslots;
        for (int i = 63; i >= 0; --i) {
            int b = tid * 64 + i;
            uint16_t code = CODE_IGNORE;
            if ((s_bmask[b >> 5] >> (b & 31)) & 1u) {
                int s = 0;
                for (int u = 0; u < ns; ++u) if (s_slotb[u] == (uint32_t)b) s = u;
                code = (uint16_t)(CODE_CAND | s);
            } else if (a.all_thresholds && s_h[b]) {
                int band = band_of(b);
                if (band != prev) {
                    ++gid;
                    prev = band;
                    if (gid < GMAX) {
                        ri->g_exp[gid] = (uint16_t)(tid ? tid : 1);
                        ri->g_band[gid] = (uint16_t)band;
                    }
                }
                code = gid < GMAX ? (uint16_t)gid : CODE_IGNORE;
            }
            tab[b] = code;
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
template <bool SUMS>
__global__ __launch_bounds__(256) void k_finish(TopkArgs a) {
    __shared__ uint32_t hA[512];
    __shared__ uint32_t hB[TMAX][256];
    __shared__ unsigned long long pacc[SUMS ? TMAX + 1 : 1][64][2];
    __shared__ int32_t s_n;
    __shared__ int32_t s_t[TMAX];
    __shared__ uint32_t s_res[TMAX], s_sb[TMAX], s_tau[TMAX], s_q[TMAX], s_eq[TMAX];
    __shared__ int32_t s_sub[TMAX];
    __shared__ uint8_t s_sub_of_sb[512];

    const int s = blockIdx.x, row = blockIdx.y, tid = threadIdx.x;
    RowInfo* ri = a.rinfo + row;
    RowAcc* ra = a.racc + row;
    if (s >= ri->n_slots) return;
    const uint32_t n = ri->slot_cnt[s];
    const uint32_t bucket = ri->slot_bucket[s];
    const uint32_t* list = a.cand + (size_t)row * (size_t)a.d + ri->slot_off[s];
    const int L = a.L;

    for (int i = tid; i < 512; i += 256) { hA[i] = 0; s_sub_of_sb[i] = 0xFF; }
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
    for (uint32_t i = tid; i < n; i += 256) atomicAdd(&hA[(list[i] >> 8) & 511u], 1u);
    __syncthreads();
    if (tid < nthr) {
        uint32_t r = s_res[tid], cum = 0;
        int sb = 511;
        for (; sb > 0; --sb) {
            uint32_t hv = hA[sb];
            if (cum + hv >= r) break;
            cum += hv;
        }
        s_sb[tid] = (uint32_t)sb;
        s_res[tid] = r - cum;
    }
    __syncthreads();
    if (tid == 0) {
        int nsub = 0;
        for (int u = 0; u < nthr; ++u) {
            if (u == 0 || s_sb[u] != s_sb[u - 1]) { s_sub_of_sb[s_sb[u]] = (uint8_t)nsub; ++nsub; }
            s_sub[u] = nsub - 1;
        }
    }
    for (int i = tid; i < TMAX * 256; i += 256) (&hB[0][0])[i] = 0;
    __syncthreads();

    // B: bits 7..0 of the keys in the thresholds' sub-bins
    for (uint32_t i = tid; i < n; i += 256) {
        uint32_t key = list[i];
        uint32_t u = s_sub_of_sb[(key >> 8) & 511u];
        if (u != 0xFF) atomicAdd(&hB[u][key & 255u], 1u);
    }
    __syncthreads();
    if (tid < nthr) {
        const uint32_t* hb = hB[s_sub[tid]];
        uint32_t r = s_res[tid], cum = 0;
        int lb = 255;
        for (; lb > 0; --lb) {
            uint32_t hv = hb[lb];
            if (cum + hv >= r) break;
            cum += hv;
        }
        uint32_t tau = (bucket << B1_SHIFT) | (s_sb[tid] << 8) | (uint32_t)lb;
        s_tau[tid] = tau;
        s_q[tid] = r - cum;
        s_eq[tid] = hb[lb];
        ri->thr_tau[s_t[tid]] = tau;
        ri->thr_q[s_t[tid]] = r - cum;
        if (r - cum > hb[lb] || r - cum == 0) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    }
    if (!SUMS) return;

    // C: exact sums of the parts the thresholds cut the bucket into (piece j: keys strictly between
    // threshold j-1 and threshold j; entries equal to a threshold key are added arithmetically)
    for (int i = tid; i < (TMAX + 1) * 64 * 2; i += 256) (&pacc[0][0][0])[i] = 0ull;
    __syncthreads();
    const uint32_t lane = lane_id();
    for (uint32_t i = tid; i < n; i += 256) {
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
// Delta_l (Lemma 3.4) from the exact group and piece sums.  One thread per (row, band).
struct BigAcc {
    uint32_t w[20];
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
        int P = top * 32 + 31 - __clz(w[top]);  // index of the most significant set bit
        auto bit = [&](int i) -> uint32_t { return i < 0 ? 0u : (w[i >> 5] >> (i & 31)) & 1u; };
        uint64_t mant = 0;
        for (int i = 0; i < 53; ++i) mant = (mant << 1) | bit(P - i);
        if (P >= 53) {
            uint32_t guard = bit(P - 53);
            bool sticky = false;
            for (int i = P - 54; i >= 0 && !sticky; --i) sticky = bit(i) != 0;
            if (guard && (sticky || (mant & 1ull))) ++mant;
            return ldexp((double)mant, P - 52 - 298);
        }
        return ldexp((double)(mant >> (52 - P)), -298);
    }
};

__global__ __launch_bounds__(64) void k_norms(TopkArgs a) {
    const int row = blockIdx.x, l = threadIdx.x;
    if (l > a.L) return;
    const RowInfo* ri = a.rinfo + row;
    const RowAcc* ra = a.racc + row;
    BigAcc acc;
    acc.clear();
    const int G = ri->n_groups;
    for (int g = 0; g < G; ++g) {
        if (ri->g_band[g] == l) {
            int sh = 2 * ((int)ri->g_exp[g] - 1);
            acc.add(ra->gsum[g][0], sh);
            acc.add(ra->gsum[g][1], sh + 32);
        }
    }
    for (int p = 0; p < PMAX; ++p) {
        const Piece& pc = ra->pieces[p];
        if (pc.band_plus1 == l + 1) {
            int sh = 2 * (pc.exp - 1);
            acc.add(pc.lo, sh);
            acc.add(pc.hi, sh + 32);
        }
    }
    if (l >= 1) {
        double S = acc.to_double();
        double nrm = __dsqrt_rn(S);
        a.norms[(size_t)row * a.L + (l - 1)] = nrm;
        if (a.norms_user) a.norms_user[(size_t)row * a.L + (l - 1)] = nrm;
    }
}

// ---------------------------------------------------------------------------------------------------
// Level draw for all rows (one workgroup).
__global__ __launch_bounds__(1024) void k_draw(DrawArgs a) {
    __shared__ int64_t s_nnz[MLMC_MAX_WORKERS];
    const int r = threadIdx.x;
    if (r < a.M) {
        double p[LMAX];
        const int L = a.L;
        if (a.mode == 0) {
            for (int l = 0; l < L; ++l) p[l] = a.p_fixed[l];
        } else if (a.mode == 1) {
            for (int l = 0; l < L; ++l) p[l] = a.p_dev[(size_t)r * L + l];
        } else {
            double tot = 0.0;
            for (int l = 0; l < L; ++l) tot = __dadd_rn(tot, a.p_dev[(size_t)r * L + l]);
            for (int l = 0; l < L; ++l)
                p[l] = tot == 0.0 ? __ddiv_rn(1.0, (double)L) : __ddiv_rn(a.p_dev[(size_t)r * L + l], tot);
        }
        uint32_t x = philox_word0(a.seed, a.step, (uint32_t)r);
        int level = draw_from_p(p, L, x);
        double pl = p[level - 1];
        float w = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
        RowInfo* ri = a.rinfo + r;
        ri->level = level;
        ri->weight = w;
        ri->draw_x = x;
        a.level[r] = level;
        s_nnz[r] = a.is_topk ? a.k[0] + a.k[level] - a.k[level - 1] : 0;
    }
    __syncthreads();
    if (r == 0 && a.is_topk) {
        int64_t run = 0;
        for (int i = 0; i < a.M; ++i) { a.row_off[i] = run; run += s_nnz[i]; }
        a.row_off[a.M] = run;
        if (run > a.capacity) atomicOr(a.dev_status, MLMC_DEV_CAPACITY);
    }
}

// ---------------------------------------------------------------------------------------------------
// Compaction, pass 1: per tile, how many keys are above / equal to each of the three thresholds.
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

template <int DT, bool VEC>
__global__ __launch_bounds__(256) void k_count(TopkArgs a) {
    __shared__ uint32_t s_red[4][6];
    const int row = blockIdx.y, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = tid >> 6;
    const Thr3 th = load_thr3(a.rinfo + row);
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    const int64_t c0 = (int64_t)blockIdx.x * a.chunk;
    const int64_t c1 = c0 + a.chunk < a.d ? c0 + a.chunk : a.d;
    uint32_t* tc = a.tilecnt + (size_t)row * 6 * a.ntiles;
    for (int64_t base = c0; base < c1; base += TILE) {
        uint32_t cnt[6] = {0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int64_t j = base + it * 1024 + tid * 4;
            uint32_t b[4];
            int nv = ld.load4(j, b);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (c < nv) {
                    uint32_t key = key_of_bits(b[c]);
#pragma unroll
                    for (int k = 0; k < 3; ++k) {
                        cnt[2 * k] += key > th.tau[k] ? 1u : 0u;
                        cnt[2 * k + 1] += key == th.tau[k] ? 1u : 0u;
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 6; ++k) cnt[k] = wave_sum(cnt[k]);
        __syncthreads();
        if (lane == 0)
            for (int k = 0; k < 6; ++k) s_red[wave][k] = cnt[k];
        __syncthreads();
        if (tid < 6) tc[(size_t)tid * a.ntiles + base / TILE] = s_red[0][tid] + s_red[1][tid] + s_red[2][tid] + s_red[3][tid];
    }
}

// Compaction, pass 2: per row, tie prefixes and output offsets of every tile.
__global__ __launch_bounds__(1024) void k_tilescan(TopkArgs a) {
    __shared__ uint32_t s_scan[17];
    const int row = blockIdx.x, tid = threadIdx.x;
    const RowInfo* ri = a.rinfo + row;
    const Thr3 th = load_thr3(ri);
    const int64_t nt = a.ntiles;
    const int64_t per = (nt + 1023) / 1024;
    const int64_t t0 = (int64_t)tid * per, t1 = t0 + per < nt ? t0 + per : nt;
    const uint32_t* tc = a.tilecnt + (size_t)row * 6 * nt;
    uint32_t* tp = a.tiepre + (size_t)row * 3 * nt;
    uint32_t* to = a.tile_off + (size_t)row * (nt + 1);
    for (int k = 0; k < 3; ++k) {
        uint32_t sum = 0;
        for (int64_t t = t0; t < t1; ++t) sum += tc[(size_t)(2 * k + 1) * nt + t];
        uint32_t total;
        uint32_t run = block_excl_scan<1024>(sum, s_scan, total);
        for (int64_t t = t0; t < t1; ++t) {
            tp[(size_t)k * nt + t] = run;
            run += tc[(size_t)(2 * k + 1) * nt + t];
        }
    }
    __syncthreads();
    auto emitted = [&](int64_t t) -> uint32_t {
        uint32_t in[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            uint64_t pre = tp[(size_t)k * nt + t], ce = tc[(size_t)(2 * k + 1) * nt + t];
            uint64_t q = th.q[k];
            uint64_t take = q > pre ? q - pre : 0;
            if (take > ce) take = ce;
            in[k] = tc[(size_t)(2 * k) * nt + t] + (uint32_t)take;
        }
        return in[0] + (in[2] - in[1]);
    };
    uint32_t sum = 0;
    for (int64_t t = t0; t < t1; ++t) sum += emitted(t);
    uint32_t total;
    uint32_t run = block_excl_scan<1024>(sum, s_scan, total);
    for (int64_t t = t0; t < t1; ++t) {
        to[t] = run;
        run += emitted(t);
    }
    if (tid == 0) {
        to[nt] = total;
        const int lev = ri->level;
        int64_t nnz = a.k[0] + a.k[lev] - a.k[lev - 1];
        if ((int64_t)total != nnz) atomicOr(a.dev_status, MLMC_DEV_INTERNAL);
    }
}

// Compaction, pass 3: write (index, value) of base band and drawn band in index order.
template <int DT, bool VEC>
__global__ __launch_bounds__(256) void k_write(TopkArgs a) {
    __shared__ uint32_t s_tie[3][4];
    __shared__ uint32_t s_emit[4];
    const int row = blockIdx.y, tid = threadIdx.x;
    const uint32_t lane = lane_id(), wave = tid >> 6;
    const RowInfo* ri = a.rinfo + row;
    const Thr3 th = load_thr3(ri);
    const float w = ri->weight;
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    const int64_t nt = a.ntiles;
    const uint32_t* tc = a.tilecnt + (size_t)row * 6 * nt;
    const uint32_t* tp = a.tiepre + (size_t)row * 3 * nt;
    const uint32_t* to = a.tile_off + (size_t)row * (nt + 1);
    const int64_t out_row = a.row_off[row];
    const int64_t c0 = (int64_t)blockIdx.x * a.chunk;
    const int64_t c1 = c0 + a.chunk < a.d ? c0 + a.chunk : a.d;

    for (int64_t base = c0; base < c1; base += TILE) {
        const int64_t tile = base / TILE;
        if (to[tile + 1] == to[tile]) continue;  // nothing to emit here (uniform)
        // this wave owns elements [base + wave*1024, +1024): 4 iterations of 64 lanes x 4
        uint32_t bits[16];
        uint32_t valid = 0;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int64_t j = base + wave * 1024 + it * 256 + lane * 4;
            uint32_t b[4];
            int nv = ld.load4(j, b);
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
        uint32_t in[3];
        bool any_tie = false;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            above[k] &= valid;
            equal[k] &= valid;
            in[k] = above[k];
            any_tie |= tc[(size_t)(2 * k + 1) * nt + tile] != 0;
        }
        if (any_tie) {  // uniform over the workgroup
            uint32_t pre[3][4];
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                uint32_t run = 0;
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    uint32_t tot;
                    uint32_t ex = wave_excl_small(__popc((equal[k] >> (it * 4)) & 0xFu), tot);
                    pre[k][it] = run + ex;
                    run += tot;
                }
                if (lane == 0) s_tie[k][wave] = run;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                uint64_t wbase = tp[(size_t)k * nt + tile];
                for (uint32_t w2 = 0; w2 < wave; ++w2) wbase += s_tie[k][w2];
                const uint64_t q = th.q[k];
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    uint64_t r = wbase + pre[k][it];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int e = it * 4 + c;
                        if ((equal[k] >> e) & 1u) {
                            if (r < q) in[k] |= 1u << e;
                            ++r;
                        }
                    }
                }
            }
        }
        const uint32_t emit = in[0] | (in[2] & ~in[1]);
        uint32_t epre[4];
        uint32_t run = 0;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            uint32_t tot;
            uint32_t ex = wave_excl_small(__popc((emit >> (it * 4)) & 0xFu), tot);
            epre[it] = run + ex;
            run += tot;
        }
        __syncthreads();  // s_emit (and s_tie) free for reuse
        if (lane == 0) s_emit[wave] = run;
        __syncthreads();
        int64_t pos0 = out_row + to[tile];
        for (uint32_t w2 = 0; w2 < wave; ++w2) pos0 += s_emit[w2];
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            int64_t pos = pos0 + epre[it];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int e = it * 4 + c;
                if ((emit >> e) & 1u) {
                    if (pos < a.capacity) {
                        float v = __uint_as_float(bits[e]);
                        a.idx[pos] = (uint32_t)(base + wave * 1024 + it * 256 + lane * 4 + c);
                        a.val[pos] = ((in[0] >> e) & 1u) ? v : __fmul_rn(v, w);
                    }
                    ++pos;
                }
            }
        }
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
    if (sums) MLMC_LAUNCH(K_FINISH, st, k_finish<true><<<fgrid, 256, 0, st>>>(a));
    else MLMC_LAUNCH(K_FINISH, st, k_finish<false><<<fgrid, 256, 0, st>>>(a));
    if (sums) MLMC_LAUNCH(K_NORMS, st, k_norms<<<pl->M, 64, 0, st>>>(a));
    return MLMC_OK;
}

template <int DT, bool VEC>
static mlmc_status launch_compact(const mlmc_plan_t* pl, const TopkArgs& a, hipStream_t st) {
    dim3 grid(pl->chunks_per_row, pl->M);
    MLMC_LAUNCH(K_COUNT, st, k_count<DT, VEC><<<grid, 256, 0, st>>>(a));
    MLMC_LAUNCH(K_TILESCAN, st, k_tilescan<<<pl->M, 1024, 0, st>>>(a));
    MLMC_LAUNCH(K_WRITE, st, k_write<DT, VEC><<<grid, 256, 0, st>>>(a));
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
