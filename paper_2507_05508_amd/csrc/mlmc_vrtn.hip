// Fixed-point ladder of |g| / max|g| (Sec. 3.1 as written) and Round-to-Nearest MLMC (Sec. 3.3, App. G.2) on gfx950:
// the launches that need the exact largest entry of a row before the extraction.
#include "mlmc_extract.h"

namespace mlmc {

// The extraction of the largest-entry ladder: the maxima are exact (every block was read), one launch.
mlmc_status vbits_extract(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, dim3 egrid, hipStream_t st) {
    const bool small = pl->nplanes <= 9;
#define MLMC_VEXTRACT(DT, VEC)                                                                                           \
    do {                                                                                                                \
        if (small) MLMC_LAUNCH(K_BITS_EXTRACT, st, k_bits_extract<DT, VEC, false, 9, 2><<<egrid, 256, 0, st>>>(a));       \
        else MLMC_LAUNCH(K_BITS_EXTRACT, st, k_bits_extract<DT, VEC, false, MAX_PLANES, 2><<<egrid, 256, 0, st>>>(a));   \
    } while (0)
    if (pl->dtype == MLMC_F32) {
        if (vec) MLMC_VEXTRACT(MLMC_F32, true);
        else MLMC_VEXTRACT(MLMC_F32, false);
    } else {
        if (vec) MLMC_VEXTRACT(MLMC_BF16, true);
        else MLMC_VEXTRACT(MLMC_BF16, false);
    }
#undef MLMC_VEXTRACT
    return MLMC_OK;
}

// ---------------------------------------------------------------------------------------------------
// Round-to-Nearest MLMC.  k_rtn_prep clears the per-row state; k_bits_smax (every block) finds c; k_rtn_norms sums
// the squared residual integers of every level; k_rtn_draw turns them into norms, probabilities, the draw and the
// coefficient; k_rtn_extract writes the planes of the drawn message's codes.
__global__ __launch_bounds__(256) void k_rtn_prep(BitsArgs a) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t == 0) *a.dev_status = 0;
    if (t < a.M) {
        a.racc[t].rowmax_key = 0u;
        a.racc[t].smpmax_key = 0u;
    }
    if (t < a.M * a.L * 2) a.rtn_sums[t] = 0ull;
}

template <int DT, bool VEC>
__global__ __launch_bounds__(256) void k_rtn_norms(BitsArgs a) {
    const int row = blockIdx.y;
    const uint32_t ckey = a.racc[row].smpmax_key;
    if (ckey == 0u) return;   // a zero row: every residual is zero
    const double c = key_to_double(ckey), den = 2.0 * c, inv_den = __ddiv_rn(1.0, den);
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    const int L = a.L;
    // Everything below is fp64 arithmetic on integers that fp64 holds exactly: |g| D has 40 bits, a code 16, a residual
    // integer k fewer than 18, k^2 fewer than 36, and a thread adds far fewer than 2^17 of them per level.
    RtnCode code[RTN_LMAX + 1];
    double Dcur[RTN_LMAX + 1], Dprev[RTN_LMAX + 1];   // D of level t; D' of level t (1 when the previous width is 0)
#pragma unroll
    for (int t = 0; t <= RTN_LMAX; ++t) {
        code[t] = rtn_code_of(t <= L ? a.F[t] : 0);
        Dcur[t] = code[t].D;
        Dprev[t] = t >= 1 && t <= L && a.F[t - 1] > 0 ? (double)((1 << a.F[t - 1]) - 1) : 1.0;
    }
    double acc[RTN_LMAX];
#pragma unroll
    for (int l = 0; l < RTN_LMAX; ++l) acc[l] = 0.0;
    auto code_of = [&](double av, int t) -> double { return rtn_code_f64(av, code[t], c, den, inv_den); };
    auto one = [&](uint32_t bits) {
        const double av = key_to_double(key_of_bits(bits));
        double nprev = code[0].b > 0 ? code_of(av, 0) : 0.0;
#pragma unroll
        for (int l = 1; l <= RTN_LMAX; ++l) {
            if (l <= L) {   // uniform
                const double ncur = code_of(av, l);
                const double k = __fma_rn(ncur, Dprev[l], -__dmul_rn(nprev, Dcur[l]));
                acc[l - 1] = __fma_rn(k, k, acc[l - 1]);
                nprev = ncur;
            }
        }
    };
    // groups of four elements, four loads of a thread in flight
    const int64_t nq = (a.d + 3) / 4, qstride = (int64_t)gridDim.x * 256;
    int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; q + 3 * qstride < nq - 1; q += 4 * qstride) {   // none of the four is the row's last (possibly partial) group
        uint32_t b[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) ld.load4_full((q + u * qstride) * 4, b[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 4; ++e) one(b[u][e]);
    }
    for (; q < nq; q += qstride) {
        uint32_t b[4];
        const int nv = ld.load4(q * 4, b);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (u < nv) one(b[u]);
    }
    // One pair of global atomics per workgroup and level (atomics of many waves on one address take turns): the waves'
    // sums meet in LDS first.
    __shared__ unsigned long long s_part[4][RTN_LMAX];
    const uint32_t wave = threadIdx.x >> 6;
#pragma unroll
    for (int l = 0; l < RTN_LMAX; ++l) {
        if (l < L) {
            unsigned long long v = (unsigned long long)acc[l];
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
            if (lane_id() == 0) s_part[wave][l] = v;
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < L) {
        const int l = threadIdx.x;
        const unsigned long long v = s_part[0][l] + s_part[1][l] + s_part[2][l] + s_part[3][l];   // < 2^53 + 2: no overflow
        if (v) {
            atomicAdd(&a.rtn_sums[((size_t)row * L + l) * 2], v & 0xFFFFFFFFull);
            atomicAdd(&a.rtn_sums[((size_t)row * L + l) * 2 + 1], v >> 32);
        }
    }
}

// Per row (one thread each): Delta_l = (2c / (D D')) sqrt(S_l), S_l the integer sum converted to fp64 once;
// probabilities (Lemma 3.4, or the plan's), the draw (Alg. 2 / Alg. 3), level, c and the coefficient.
__global__ __launch_bounds__(64) void k_rtn_draw(BitsArgs a, int norms_only) {
    __shared__ double s_p[64][RTN_LMAX];
    __shared__ uint32_t s_big[64][20];
    const int row = blockIdx.x * 64 + threadIdx.x;
    if (row >= a.M) return;
    const int L = a.L;
    const uint32_t ckey = a.racc[row].smpmax_key;
    if (ckey >= 0x7F800000u) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
    const double c = key_to_double(ckey);
    double* p = s_p[threadIdx.x];
    double factor[RTN_LMAX];
#pragma unroll
    for (int l = 0; l < RTN_LMAX; ++l) factor[l] = 0.0;
    for (int l = 1; l <= L; ++l) {
        const unsigned long long lo = a.rtn_sums[((size_t)row * L + (l - 1)) * 2], hi = a.rtn_sums[((size_t)row * L + (l - 1)) * 2 + 1];
        // S = hi 2^32 + lo as 32-bit words
        uint32_t* w = s_big[threadIdx.x];
        for (int i = 0; i < 20; ++i) w[i] = 0u;
        const unsigned long long w1 = (lo >> 32) + (hi & 0xFFFFFFFFull);
        w[0] = (uint32_t)lo;
        w[1] = (uint32_t)w1;
        const unsigned long long w2 = (w1 >> 32) + (hi >> 32);
        w[2] = (uint32_t)w2;
        w[3] = (uint32_t)(w2 >> 32);
        BigAcc big;
        big.w = w;
        const double Sd = ldexp(big.to_double(), 298);
        const double D = (double)((1 << a.F[l]) - 1), Dp = a.F[l - 1] > 0 ? (double)((1 << a.F[l - 1]) - 1) : 1.0;
        const double f = __ddiv_rn(__dmul_rn(2.0, c), __dmul_rn(D, Dp));
        const double nrm = __dmul_rn(f, __dsqrt_rn(Sd));
#pragma unroll
        for (int q = 0; q < RTN_LMAX; ++q) if (q == l - 1) factor[q] = f;
        p[l - 1] = nrm;
        a.norms[(size_t)row * L + (l - 1)] = nrm;
        if (a.norms_user) a.norms_user[(size_t)row * L + (l - 1)] = nrm;
    }
    if (norms_only) return;
    if (a.adaptive) {
        double tot = 0.0;
        for (int l = 0; l < L; ++l) tot = __dadd_rn(tot, p[l]);
        for (int l = 0; l < L; ++l) p[l] = tot == 0.0 ? __ddiv_rn(1.0, (double)L) : __ddiv_rn(p[l], tot);
    } else {
        for (int l = 0; l < L; ++l) p[l] = a.p_fixed[l];
    }
    const uint32_t x = philox_word0(a.seed, a.step, (uint32_t)row);
    const int level = draw_from_p(p, L, x);
    const double pl = p[level - 1];
    double f = 0.0;
#pragma unroll
    for (int q = 0; q < RTN_LMAX; ++q) if (q == level - 1) f = factor[q];
    a.rinfo[row].level = level;
    a.rinfo[row].draw_x = x;
    a.level[row] = level;
    a.scale_exp[2 * row] = (int32_t)ckey;
    a.scale_exp[2 * row + 1] = (int32_t)__float_as_uint(pl == 0.0 ? 0.0f : (float)__ddiv_rn(f, pl));
}

template <int DT, bool VEC>
__global__ __launch_bounds__(256) void k_rtn_extract(BitsArgs a) {
    __shared__ __align__(16) uint32_t s_tr[4][1024];
    uint32_t* slds = s_tr[threadIdx.x >> 6];
    const int row = blockIdx.y;
    const int level = a.rinfo[row].level;
    RtnRow rr;
    rr.c = key_to_double(a.racc[row].smpmax_key);
    rr.den = 2.0 * rr.c;
    rr.inv_den = rr.c > 0.0 ? __ddiv_rn(1.0, rr.den) : 0.0;
    rr.code[0] = rtn_code_of(a.F[0]);
    rr.code[1] = rtn_code_of(level > 1 ? a.F[level - 1] : 0);
    rr.code[2] = rtn_code_of(a.F[level]);
    const int np = rr.code[0].b + rr.code[1].b + rr.code[2].b;
    uint32_t maxkey = 0;
    if (np <= 8) bits_extract_tiles<DT, VEC, 8, 5>(a, row, 1, level, np, maxkey, slds, 0.0, 0.0, &rr);
    else if (np <= 16) bits_extract_tiles<DT, VEC, 16, 5>(a, row, 1, level, np, maxkey, slds, 0.0, 0.0, &rr);
    else bits_extract_tiles<DT, VEC, MAX_FPLANES, 5>(a, row, 1, level, np, maxkey, slds, 0.0, 0.0, &rr);
}

// Round-to-Nearest MLMC: largest entry, residual sums, draw, codes.  message == false: norms only.
mlmc_status rtn_compress(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, bool message, hipStream_t st) {
    const int M = pl->M;
    int pb = (M * pl->L * 2 + 255) / 256;
    if (pb < (M + 255) / 256) pb = (M + 255) / 256;
    MLMC_LAUNCH(K_DRAW, st, k_rtn_prep<<<pb, 256, 0, st>>>(a));
    const int64_t nblk = (pl->d + 1023) / 1024;
    int64_t sw = (nblk + 7) / 8;
    const int64_t scap = 1024 / M > 0 ? 1024 / M : 1;
    if (sw > scap) sw = scap;
    if (sw < 1) sw = 1;
    const dim3 sgrid((unsigned)sw, M);
    int64_t nw = (pl->d + 4 * 256 * 8 - 1) / (4 * 256 * 8);   // a thread takes at least about eight groups of four elements
    const int64_t ncap = 2048 / M > 0 ? 2048 / M : 1;          // eight workgroups per CU in all: few atomics per sum
    if (nw > ncap) nw = ncap;
    const int64_t nmin = (pl->d + ((int64_t)1 << 24) - 1) >> 24;   // a thread adds at most 2^16 squares below 2^36: exact in fp64
    if (nw < nmin) nw = nmin;
    if (nw < 1) nw = 1;
    const dim3 ngrid((unsigned)nw, M);
    int64_t ntiles = pl->ntiles;
    int gx = (int)((ntiles + 15) / 16);
    if ((int64_t)gx * M < 512) gx = (int)((ntiles + 3) / 4);
    const int cap = 4096 / M > 0 ? 4096 / M : 1;
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    const dim3 egrid(gx, M);
    // with the plan's own probabilities the draw needs no norms: that read of the input is made only when they are asked for
    const bool need_norms = pl->adaptive || !message || a.norms_user != nullptr;
#define MLMC_RTN_STEPS(DT, VEC)                                                                                          \
    do {                                                                                                                \
        MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<DT, VEC, false><<<sgrid, SMAX_THREADS, 0, st>>>(a));                            \
        if (need_norms) MLMC_LAUNCH(K_RTN_NORMS, st, k_rtn_norms<DT, VEC><<<ngrid, 256, 0, st>>>(a));                     \
        MLMC_LAUNCH(K_RTN_DRAW, st, k_rtn_draw<<<(M + 63) / 64, 64, 0, st>>>(a, message ? 0 : 1));                        \
        if (message) MLMC_LAUNCH(K_BITS_EXTRACT, st, k_rtn_extract<DT, VEC><<<egrid, 256, 0, st>>>(a));                  \
    } while (0)
    if (pl->dtype == MLMC_F32) {
        if (vec) MLMC_RTN_STEPS(MLMC_F32, true);
        else MLMC_RTN_STEPS(MLMC_F32, false);
    } else {
        if (vec) MLMC_RTN_STEPS(MLMC_BF16, true);
        else MLMC_RTN_STEPS(MLMC_BF16, false);
    }
#undef MLMC_RTN_STEPS
    return MLMC_OK;
}

}  // namespace mlmc
