// Bit-wise MLMC (Sec. 3.1 fixed point, App. B floating point) and the server aggregate (Alg. 2 / Alg. 3) on gfx950.
//
//   k_bits_prep     level draw of every row (floating-point ladder; the other ladders draw in k_bits_smax)
//   k_bits_smax     largest |g| key of a sample of every row -> predicted power-of-two scale; level draw             [mlmc_extract.h]
//   k_bits_extract  the one full read: digits floor(|g_j| / s * 2^F), sign plane + field planes packed by wave      [mlmc_extract.h]
//                   ballot, and the true row maximum; a row whose true maximum has a larger exponent than the
//                   sampled one is extracted again by a second launch (which returns at once for every other row)
//   k_agg_bits      out = alpha * sum_i decode_i, rows added in worker order (all plane messages, Round-to-Nearest included)
//   k_tileoff       (fallback) per-tile offsets of index-sorted sparse rows by binary search
//   k_agg_sparse    atomic-free segmented scatter-add: one workgroup owns one dense tile
//   k_message_bits  bits on the wire of every row's message
// The ladder of |g| / max|g| and the Round-to-Nearest ladder are launched from mlmc_vrtn.hip.
#include "mlmc_extract.h"

namespace mlmc {

// ---------------------------------------------------------------------------------------------------
// Level draw of every row (Alg. 2 "Sample l ~ p"), and the per-row state of the call set to its start values.
__global__ __launch_bounds__(1024) void k_bits_prep(BitsArgs a) {
    __shared__ double s_p[LMAX];
    const int r = threadIdx.x;
    if (r < a.L) s_p[r] = a.p_fixed[r];
    if (r == 0) *a.dev_status = 0;
    __syncthreads();
    for (int row = r; row < a.M; row += 1024) {
        const uint32_t x = philox_word0(a.seed, a.step, (uint32_t)row);
        const int level = draw_from_p(s_p, a.L, x);
        const double pl = s_p[level - 1];
        RowInfo* ri = a.rinfo + row;
        ri->level = level;
        ri->weight = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
        ri->draw_x = x;
        a.level[row] = level;
        a.racc[row].rowmax_key = 0u;
        a.racc[row].smpmax_key = 0u;
    }
}

// What a kernel of the aggregate does with the finished sum of entry j: g~_j = alpha * acc (Alg. 2 "Server
// aggregates"), written out and / or applied to the model, x_j <- x_j - eta * g~_j (Alg. 2 "Server updates": one
// multiply, one subtract).
__device__ __forceinline__ void finish_entry(float alpha, float acc, float* out, float eta, float* x, int64_t j) {
    const float gt = __fmul_rn(alpha, acc);
    if (out) __builtin_nontemporal_store(gt, &out[j]);   // written once, read by the caller later
    if (x) x[j] = __fsub_rn(x[j], __fmul_rn(eta, gt));
}

struct AggBitsArgs {
    BitsArgs b;
    const int32_t* level;
    const int32_t* scale_exp;
    float alpha, eta;
};

// out[j] = alpha * sum over rows (worker order) of sign * (f0 * c0 + f * cl): Alg. 2 "Server aggregates".
// A wave owns eight consecutive words of every plane, i.e. 512 consecutive elements; lane = element within a word.
// The eight words of a (row, plane) are one 64-byte scalar load: a plane word is wave-uniform data, and as a
// scalar register pair it is at once the lane mask "this element's bit is set".  A row whose level field is a
// single bit (the most likely levels) costs two selects and one add per element.
struct Words8 {
    uint64_t w[8];
};
__device__ __forceinline__ Words8 load_words8(const uint64_t* __restrict__ p, int nvalid) {
    Words8 r;
    if (nvalid >= 8) {   // uniform
        r = *(const Words8*)p;
    } else {             // the last words of a plane: nothing is read past the plane's end
#pragma unroll
        for (int k = 0; k < 8; ++k) r.w[k] = k < nvalid ? p[k] : 0ull;
    }
    return r;
}

__global__ __launch_bounds__(256) void k_agg_bits(AggBitsArgs a, const uint64_t* __restrict__ planes, float* __restrict__ out,
                                                  float* __restrict__ x) {
    __shared__ float s_c0[MLMC_MAX_WORKERS], s_cl[MLMC_MAX_WORKERS];
    __shared__ uint8_t s_w[MLMC_MAX_WORKERS], s_fl[MLMC_MAX_WORKERS];
    const BitsArgs& b = a.b;
    const int F0 = b.F[0];
    for (int r = threadIdx.x; r < b.M; r += 256) {
        int lev = a.level[r];
        lev = lev < 1 ? 1 : (lev > b.L ? b.L : lev);
        double pl = b.p_fixed[lev - 1];
        if (b.rtn) {   // Round-to-Nearest: c_0 = fp32(2c / D_0); the coefficient comes with the message
            const double c = key_to_double((uint32_t)a.scale_exp[2 * r] & 0x7FFFFFFFu);
            s_c0[r] = F0 > 0 ? (float)__ddiv_rn(__dmul_rn(2.0, c), (double)((1 << F0) - 1)) : 0.0f;
            s_cl[r] = __uint_as_float((uint32_t)a.scale_exp[2 * r + 1]);
            s_w[r] = (uint8_t)b.F[lev];                          // width of the drawn level's code
            s_fl[r] = (uint8_t)(lev > 1 ? b.F[lev - 1] : 0);     // width of the previous level's code when it is sent
            continue;
        }
        if (b.flt) {   // the level's weight fp32(1 / p_l)
            s_c0[r] = 0.0f;
            s_cl[r] = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
        } else if (b.vmx) {   // the scale field carries the largest entry v: c_0 = fp32(v 2^-F_0), c_l = fp32(v 2^-F_l / p_l)
            const uint32_t vkey = (uint32_t)a.scale_exp[r] & 0x7FFFFFFFu, vE = vkey >> 23;
            const double vd = ldexp((double)(vE ? (vkey & 0x7FFFFFu) | 0x800000u : vkey), (int)(vE ? vE : 1u) - 150);
            s_c0[r] = (float)ldexp(vd, -F0);
            s_cl[r] = pl == 0.0 ? 0.0f : (float)__ddiv_rn(ldexp(vd, -b.F[lev]), pl);
        } else {
            int e = a.scale_exp[r];
            s_c0[r] = (float)ldexp(1.0, e - F0);
            s_cl[r] = pl == 0.0 ? 0.0f : (float)__ddiv_rn(ldexp(1.0, e - b.F[lev]), pl);
        }
        s_w[r] = (uint8_t)(b.F[lev] - b.F[lev - 1]);
        s_fl[r] = (uint8_t)b.F[lev];
    }
    __syncthreads();
    const uint32_t lane = lane_id();
    const int64_t nw = b.nwords;
    const int64_t nblk = (nw + 7) / 8;
    const int64_t wave_global = __builtin_amdgcn_readfirstlane((int)(((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6));
    const int64_t nwaves = ((int64_t)gridDim.x * 256) >> 6;
    for (int64_t blk = wave_global; blk < nblk; blk += nwaves) {
        const int64_t w0 = blk * 8;
        const int nvalid = nw - w0 < 8 ? (int)(nw - w0) : 8;
        float acc[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
        for (int r = 0; r < b.M; ++r) {   // rows in worker order
            const int wd = __builtin_amdgcn_readfirstlane((int)s_w[r]);
            const float cl = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(s_cl[r])));
            const uint64_t* rp = planes + (size_t)r * b.nplanes * nw + w0;
            const Words8 sg = load_words8(rp, nvalid);
            if (b.rtn) {
                // codes n_{b_0} (if any), n_{b_{l-1}} (if sent) and n_{b_l} from their planes, sign-extended; the residual
                // integer k = n_cur D' - n_prev D; value = fp32(n_0) c_0 + fp32(k) coefficient
                const int bp = __builtin_amdgcn_readfirstlane((int)s_fl[r]);
                const float c0 = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(s_c0[r])));
                const int bprev = bp > 0 ? bp : F0;               // level 1: the previous code is the base code
                const int D = (1 << wd) - 1, Dp = bprev > 0 ? (1 << bprev) - 1 : 1;
                uint32_t u0[8], u1[8], u2[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) { u0[k] = 0; u1[k] = 0; u2[k] = 0; }
                for (int q = 0; q < F0; ++q) {
                    const Words8 pw = q == 0 ? sg : load_words8(rp + (size_t)q * nw, nvalid);
                    const uint32_t bit = 1u << q;
#pragma unroll
                    for (int k = 0; k < 8; ++k) u0[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
                for (int q = 0; q < bp; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(F0 + q) * nw, nvalid);
                    const uint32_t bit = 1u << q;
#pragma unroll
                    for (int k = 0; k < 8; ++k) u1[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
                for (int q = 0; q < wd; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(F0 + bp + q) * nw, nvalid);
                    const uint32_t bit = 1u << q;
#pragma unroll
                    for (int k = 0; k < 8; ++k) u2[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int32_t n0 = F0 > 0 ? (int32_t)(u0[k] << (32 - F0)) >> (32 - F0) : 0;
                    const int32_t np_ = bp > 0 ? (int32_t)(u1[k] << (32 - bp)) >> (32 - bp) : n0;
                    const int32_t nc = (int32_t)(u2[k] << (32 - wd)) >> (32 - wd);
                    float v = __fmul_rn((float)(nc * Dp - np_ * D), cl);
                    if (F0 > 0) v = __fadd_rn(__fmul_rn((float)n0, c0), v);
                    acc[k] = __fadd_rn(acc[k], v);
                }
            } else if (b.flt) {
                // App. B: sign, exponent field and base digits give C^{F_0}; the level digits, placed under the same
                // sign and exponent, minus the bare power of two give the residual (exact); weight, then one add
                const int Fl = __builtin_amdgcn_readfirstlane((int)s_fl[r]);
                uint32_t ev[8], f[8], f0[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) { ev[k] = 0; f[k] = 0; f0[k] = 0; }
                for (int q = 0; q < 8; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(1 + q) * nw, nvalid);
                    const uint32_t bit = 1u << (23 + q);
#pragma unroll
                    for (int k = 0; k < 8; ++k) ev[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
                for (int q = 0; q < F0; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(9 + q) * nw, nvalid);
                    const uint32_t bit = 1u << (23 - F0 + q);
#pragma unroll
                    for (int k = 0; k < 8; ++k) f0[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
                for (int q = 0; q < wd; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(9 + F0 + q) * nw, nvalid);
                    const uint32_t bit = 1u << (23 - Fl + q);
#pragma unroll
                    for (int k = 0; k < 8; ++k) f[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t se = ev[k] | (__builtin_amdgcn_inverse_ballot_w64(sg.w[k]) ? 0x80000000u : 0u);
                    const float res = __fsub_rn(__uint_as_float(se | f[k]), __uint_as_float(se));
                    const float v = __fadd_rn(__uint_as_float(se | f0[k]), __fmul_rn(res, cl));
                    acc[k] = __fadd_rn(acc[k], v);
                }
            } else if (F0 == 0 && wd == 1) {
                // f is 0 or 1: the entry is +-cl or absent (adding +0 leaves the sum as it is)
                const Words8 fw = load_words8(rp + nw, nvalid);
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    float v = __builtin_amdgcn_inverse_ballot_w64(fw.w[k] & ~sg.w[k]) ? cl : 0.0f;
                    v = __builtin_amdgcn_inverse_ballot_w64(fw.w[k] & sg.w[k]) ? -cl : v;
                    acc[k] = __fadd_rn(acc[k], v);
                }
            } else {
                const float c0 = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(s_c0[r])));
                uint32_t f[8], f0[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) { f[k] = 0; f0[k] = 0; }
                for (int q = 0; q < F0; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(1 + q) * nw, nvalid);
                    const uint32_t bit = 1u << q;
#pragma unroll
                    for (int k = 0; k < 8; ++k) f0[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
                for (int q = 0; q < wd; ++q) {
                    const Words8 pw = load_words8(rp + (size_t)(1 + F0 + q) * nw, nvalid);
                    const uint32_t bit = 1u << q;
#pragma unroll
                    for (int k = 0; k < 8; ++k) f[k] |= __builtin_amdgcn_inverse_ballot_w64(pw.w[k]) ? bit : 0u;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    float v = __fmul_rn((float)f[k], cl);
                    if (F0 > 0) v = __fadd_rn(__fmul_rn((float)f0[k], c0), v);
                    acc[k] = __fadd_rn(acc[k], __builtin_amdgcn_inverse_ballot_w64(sg.w[k]) ? -v : v);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int64_t j = (w0 + k) * 64 + lane;
            if (j < b.d) finish_entry(a.alpha, acc[k], out, a.eta, x, j);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
struct AggSparseArgs {
    int32_t M;
    int64_t d, ntiles;
    const int64_t* row_off;
    const uint32_t* idx;
    const float* val;
    int64_t capacity;          // entries idx / val hold
    const uint32_t* tile_off;  // [M][ntiles + 1]
    uint32_t* tile_off_out;    // k_tileoff target
    float alpha;
    float* out;                // the dense update g~ (may be null when only x is wanted)
    float eta;
    float* x;                  // server update x <- x - eta * g~ (null: no update)
};

__global__ __launch_bounds__(256) void k_tileoff(AggSparseArgs a) {
    const int64_t n = (int64_t)a.M * (a.ntiles + 1);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int r = (int)(i / (a.ntiles + 1));
        const int64_t t = i % (a.ntiles + 1);
        int64_t s = a.row_off[r], e = a.row_off[r + 1];   // entries past the capacity were never written
        if (s > a.capacity) s = a.capacity;
        if (e > a.capacity) e = a.capacity;
        if (e < s) e = s;
        const uint64_t target = (uint64_t)t * TILE;
        int64_t lo = s, hi = e;  // first position with idx >= target
        while (lo < hi) {
            int64_t mid = lo + ((hi - lo) >> 1);
            if ((uint64_t)a.idx[mid] < target) lo = mid + 1; else hi = mid;
        }
        a.tile_off_out[i] = (uint32_t)(lo - s);
    }
}

// One workgroup per dense tile: LDS accumulators, rows added one after the other (indices within a row are
// distinct, so plain read-modify-write is race free), then one coalesced write of alpha * acc.
__global__ __launch_bounds__(256) void k_agg_sparse(AggSparseArgs a) {
    // dynamic LDS, sized by the number of rows (M * 12 bytes), so that a CU holds as many workgroups as its wave
    // slots allow: the tile's accumulators, then every row's start and length inside the tile
    extern __shared__ __align__(16) unsigned char s_dyn_agg[];
    float* s_acc = (float*)s_dyn_agg;
    int64_t* s_beg = (int64_t*)(s_dyn_agg + TILE * sizeof(float));
    uint32_t* s_len = (uint32_t*)(s_dyn_agg + TILE * sizeof(float) + (size_t)a.M * sizeof(int64_t));
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * TILE;
    for (int i = threadIdx.x; i < TILE; i += 256) s_acc[i] = 0.0f;
    for (int r = threadIdx.x; r < a.M; r += 256) {
        const uint32_t* to = a.tile_off + (size_t)r * (a.ntiles + 1);
        // a tile holds at most TILE entries of a row and they lie inside the row's message: an offset table that
        // says otherwise (a failed compress call, a caller's own table) must not steer reads out of bounds
        const int64_t beg = a.row_off[r] + to[tile];
        uint32_t len = to[tile + 1] - to[tile];
        if (to[tile + 1] < to[tile] || len > (uint32_t)TILE || beg < a.row_off[r] || beg + len > a.row_off[r + 1] ||
            beg + len > a.capacity) len = 0;
        s_beg[r] = beg;
        s_len[r] = len;
    }
    __syncthreads();
    // rows in groups of eight: the first 256 entries of every row of the group are fetched back to back (a thread's
    // entry, or the row's last one when it has fewer), then added in worker order
    constexpr int RG = 8;
    for (int r0 = 0; r0 < a.M; r0 += RG) {
        uint32_t pidx[RG];
        float pval[RG];
#pragma unroll
        for (int k = 0; k < RG; ++k) {
            const int r = r0 + k;
            const uint32_t len = r < a.M ? s_len[r] : 0u;
            pidx[k] = 0xFFFFFFFFu;
            pval[k] = 0.0f;
            if (len) {  // uniform
                const uint32_t e = threadIdx.x < len ? threadIdx.x : len - 1u;
                pidx[k] = a.idx[s_beg[r] + e];
                pval[k] = a.val[s_beg[r] + e];
            }
        }
#pragma unroll
        for (int k = 0; k < RG; ++k) {
            const int r = r0 + k;
            const uint32_t len = r < a.M ? s_len[r] : 0u;
            if (len) {  // uniform
                const int64_t beg = s_beg[r];
                if (threadIdx.x < len) {
                    const uint32_t off = pidx[k] - (uint32_t)base;
                    if (off < (uint32_t)TILE) s_acc[off] = __fadd_rn(s_acc[off], pval[k]);
                }
                // the rest of a long row: four loads per thread in flight (past the end: the last entry, discarded)
                for (uint32_t i0 = threadIdx.x + 256; i0 < len; i0 += 1024) {
                    uint32_t qi[4];
                    float qv[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const uint32_t i = i0 + (uint32_t)u * 256u;
                        const uint32_t e = i < len ? i : len - 1u;
                        qi[u] = a.idx[beg + e];
                        qv[u] = a.val[beg + e];
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const uint32_t off = qi[u] - (uint32_t)base;
                        if (i0 + (uint32_t)u * 256u < len && off < (uint32_t)TILE) s_acc[off] = __fadd_rn(s_acc[off], qv[u]);
                    }
                }
                __syncthreads();
            }
        }
    }
    for (int i = threadIdx.x; i < TILE; i += 256) {
        int64_t j = base + i;
        if (j < a.d) finish_entry(a.alpha, s_acc[i], a.out, a.eta, a.x, j);
    }
}

// Bits that name one of n alternatives.
__device__ __forceinline__ int ceil_log2_dev(int64_t n) { return n <= 1 ? 0 : 64 - __clzll((unsigned long long)(n - 1)); }

// Bits every worker's message takes on the wire.  Rank bands (Sec. 3, Sec. 3.2): every entry as a 32-bit value and an
// index into d, plus the level.  Fixed-point ladder (Sec. 3.1): per entry the sign, the base bits and the bits of
// the level field, plus the 32-bit scale exponent and the level.
struct MsgBitsArgs {
    int32_t kind, M, L;
    int64_t d, s;
    int64_t ladder[TMAX];
    const int32_t* level;
    unsigned long long* bits;
};
__global__ __launch_bounds__(256) void k_message_bits(MsgBitsArgs a) {
    __shared__ int64_t s_lad[TMAX];
    if (a.kind != MLMC_STOPK && (int)threadIdx.x <= a.L) s_lad[threadIdx.x] = a.ladder[threadIdx.x];
    __syncthreads();
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= a.M) return;
    int lev = a.level[r];
    lev = lev < 1 ? 1 : (lev > a.L ? a.L : lev);
    unsigned long long n;
    if (a.kind == MLMC_STOPK) {   // the drawn segment: s entries, the last one what is left
        const int64_t lo = (int64_t)(lev - 1) * a.s;
        const int64_t cnt = lo + a.s < a.d ? a.s : a.d - lo;
        a.bits[r] = (unsigned long long)cnt * (unsigned long long)(32 + ceil_log2_dev(a.d)) + (unsigned long long)ceil_log2_dev(a.L);
        return;
    }
    const int64_t width = s_lad[lev] - s_lad[lev - 1];
    if (a.kind == MLMC_TOPK) n = (unsigned long long)(s_lad[0] + width) * (unsigned long long)(32 + ceil_log2_dev(a.d));
    else if (a.kind == MLMC_FBITS) n = (unsigned long long)a.d * (unsigned long long)(9 + s_lad[0] + width);
    else if (a.kind == MLMC_RTN) n = (unsigned long long)a.d * (unsigned long long)(s_lad[0] + (lev > 1 ? s_lad[lev - 1] : 0) + s_lad[lev]) + 64ull;
    else n = (unsigned long long)a.d * (unsigned long long)(1 + s_lad[0] + width) + 32ull;
    a.bits[r] = n + (unsigned long long)ceil_log2_dev(a.L);
}

mlmc_status message_bits(const mlmc_plan_t* pl, const int32_t* level, unsigned long long* bits, hipStream_t st) {
    MsgBitsArgs a;
    a.kind = pl->kind;
    a.M = pl->M;
    a.L = pl->L;
    a.d = pl->d;
    a.s = pl->s;
    if (pl->kind != MLMC_STOPK)
        for (int t = 0; t <= pl->L; ++t) a.ladder[t] = pl->ladder[t];
    a.level = level;
    a.bits = bits;
    MLMC_LAUNCH(K_MSGBITS, st, k_message_bits<<<(pl->M + 255) / 256, 256, 0, st>>>(a));
    return MLMC_OK;
}

// ---------------------------------------------------------------------------------------------------
mlmc_status vbits_extract(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, dim3 egrid, hipStream_t st);   // mlmc_vrtn.hip

mlmc_status bits_compress(const mlmc_plan_t* pl, const BitsArgs& a0, bool vec, hipStream_t st) {
    BitsArgs a = a0;
    if (a.flt) MLMC_LAUNCH(K_DRAW, st, k_bits_prep<<<1, 1024, 0, st>>>(a));
    // a wave takes about four tiles (its loads run ahead across tiles); at least some 2048 waves in all
    int64_t ntiles = pl->ntiles;
    int gx = (int)((ntiles + 15) / 16);
    if ((int64_t)gx * pl->M < 512) gx = (int)((ntiles + 3) / 4);
    int cap = 4096 / pl->M > 0 ? 4096 / pl->M : 1;
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    dim3 egrid(gx, pl->M);
#define MLMC_EXTRACT_V(ID, DT, VEC, REDO, KIND, SMALL, BIG)                                                              \
    do {                                                                                                                \
        if (small) MLMC_LAUNCH(ID, st, k_bits_extract<DT, VEC, REDO, SMALL, KIND><<<egrid, 256, 0, st>>>(a));            \
        else MLMC_LAUNCH(ID, st, k_bits_extract<DT, VEC, REDO, BIG, KIND><<<egrid, 256, 0, st>>>(a));                    \
    } while (0)
#define MLMC_EXTRACT(ID, REDO, KIND, SMALL, BIG)                                                                         \
    do {                                                                                                                \
        if (pl->dtype == MLMC_F32) {                                                                                    \
            if (vec) MLMC_EXTRACT_V(ID, MLMC_F32, true, REDO, KIND, SMALL, BIG);                                         \
            else MLMC_EXTRACT_V(ID, MLMC_F32, false, REDO, KIND, SMALL, BIG);                                            \
        } else {                                                                                                        \
            if (vec) MLMC_EXTRACT_V(ID, MLMC_BF16, true, REDO, KIND, SMALL, BIG);                                        \
            else MLMC_EXTRACT_V(ID, MLMC_BF16, false, REDO, KIND, SMALL, BIG);                                           \
        }                                                                                                               \
    } while (0)
    if (a.flt) {
        // floating-point ladder (App. B): no scale, so nothing to find before the one read
        const bool small = pl->nplanes <= 11;
        MLMC_EXTRACT(K_BITS_EXTRACT, false, 1, 11, MAX_FPLANES);
        return MLMC_OK;
    }
    // sampled (or, for short rows, exact) row maxima
    const int64_t nblk = (pl->d + 1023) / 1024;
    const int64_t ns = (nblk >> a.sample_shift) > 0 ? (nblk >> a.sample_shift) : 1;
    int64_t sw = (ns + 7) / 8;   // a block per wave, up to four workgroups of eight waves on every CU
    const int64_t scap = 1024 / pl->M > 0 ? 1024 / pl->M : 1;
    if (sw > scap) sw = scap;
    if (sw < 1) sw = 1;
    const dim3 sgrid((unsigned)sw, pl->M);
    // the first launch of the call: its workgroups leave one maximum each (nothing to clear beforehand) and draw the levels
    static_assert(1024 <= SMAX_PARTS_MAX, "sw is at most 1024");
    a.smax_parts = (int32_t)sw;
    if (pl->dtype == MLMC_F32) {
        if (vec) MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_F32, true, true><<<sgrid, SMAX_THREADS, 0, st>>>(a));
        else MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_F32, false, true><<<sgrid, SMAX_THREADS, 0, st>>>(a));
    } else {
        if (vec) MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_BF16, true, true><<<sgrid, SMAX_THREADS, 0, st>>>(a));
        else MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_BF16, false, true><<<sgrid, SMAX_THREADS, 0, st>>>(a));
    }
    const bool small = pl->nplanes <= 9;
    if (a.vmx) return vbits_extract(pl, a, vec, egrid, st);   // the maxima above are exact (every block was read): one extraction
    MLMC_EXTRACT(K_BITS_EXTRACT, false, 0, 9, MAX_PLANES);
    if (a.sample_shift > 0) MLMC_EXTRACT(K_BITS_REDO, true, 0, 9, MAX_PLANES);   // rows whose sampled maximum fell short (returns at once for the others)
#undef MLMC_EXTRACT_V
#undef MLMC_EXTRACT
    return MLMC_OK;
}

mlmc_status agg_bits(const mlmc_plan_t* pl, const BitsArgs& b, const int32_t* level, const int32_t* scale_exp,
                     const uint64_t* planes, float alpha, float* out, float eta, float* x, hipStream_t st) {
    AggBitsArgs a;
    a.b = b;
    a.level = level;
    a.scale_exp = scale_exp;
    a.alpha = alpha;
    a.eta = eta;
    int64_t waves = (b.nwords + 7) / 8;   // a wave takes eight words at a time
    int blocks = (int)((waves + 3) / 4);
    if (blocks > 8192) blocks = 8192;
    if (blocks < 1) blocks = 1;
    MLMC_LAUNCH(K_AGG_BITS, st, k_agg_bits<<<blocks, 256, 0, st>>>(a, planes, out, x));
    return MLMC_OK;
}

mlmc_status agg_sparse(const mlmc_plan_t* pl, const int64_t* row_off, const uint32_t* idx, const float* val, int64_t capacity,
                       const uint32_t* tile_off, uint32_t* tile_off_ws, float alpha, float* out, float eta, float* x,
                       hipStream_t st) {
    AggSparseArgs a;
    a.M = pl->M;
    a.d = pl->d;
    a.ntiles = pl->ntiles;
    a.row_off = row_off;
    a.idx = idx;
    a.val = val;
    a.capacity = capacity;
    a.tile_off = tile_off;
    a.tile_off_out = tile_off_ws;
    a.alpha = alpha;
    a.out = out;
    a.eta = eta;
    a.x = x;
    if (!tile_off) {
        int64_t n = (int64_t)pl->M * (pl->ntiles + 1);
        int blocks = (int)((n + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        MLMC_LAUNCH(K_TILEOFF, st, k_tileoff<<<blocks, 256, 0, st>>>(a));
        a.tile_off = tile_off_ws;
    }
    const size_t lds = TILE * sizeof(float) + (size_t)pl->M * (sizeof(int64_t) + sizeof(uint32_t));
    MLMC_LAUNCH(K_AGG_SPARSE, st, k_agg_sparse<<<(unsigned)pl->ntiles, 256, lds, st>>>(a));
    return MLMC_OK;
}

}  // namespace mlmc
