// Extraction of bit-plane messages on gfx950, shared by the translation units that launch it: the row maximum
// (k_bits_smax), the tile packer (bits_extract_tiles) and the extraction kernel of the bit-wise ladders
// (k_bits_extract).  Sec. 3.1 (fixed point), App. B (floating point), Sec. 3.3 / App. G.2 (Round-to-Nearest codes).
#pragma once
#include "mlmc_device.h"

namespace mlmc {

// Largest |g| key of the sampled blocks of every row (block b of 1024 elements is sampled when b % S == S / 2,
// S = 2^sample_shift; S = 1 reads the whole row and the result is the row maximum itself).
// PARTS: nothing is cleared beforehand, so no launch precedes this one: every workgroup stores its own maximum (the
// readers take the largest of a row's, row_smpmax), and the first workgroup of a row draws the row's level (Alg. 2
// "Sample l ~ p") and sets the state that the extraction accumulates into to its start values.
constexpr int SMAX_THREADS = 512;
template <int DT, bool VEC, bool PARTS>
__global__ __launch_bounds__(SMAX_THREADS) void k_bits_smax(BitsArgs a) {
    const int row = blockIdx.y;
    if (PARTS && blockIdx.x == 0) {   // uniform over the workgroup
        __shared__ double s_p[LMAX];
        if ((int)threadIdx.x < a.L) s_p[threadIdx.x] = a.p_fixed[threadIdx.x];
        __syncthreads();
        if (threadIdx.x == 0) {
            if (row == 0) *a.dev_status = 0;   // no workgroup of this launch reports through it
            const uint32_t x = philox_word0(a.seed, a.step, (uint32_t)row);
            const int level = draw_from_p(s_p, a.L, x);
            const double pl = s_p[level - 1];
            RowInfo* ri = a.rinfo + row;
            ri->level = level;
            ri->weight = pl == 0.0 ? 0.0f : (float)__ddiv_rn(1.0, pl);
            ri->draw_x = x;
            a.level[row] = level;
            a.racc[row].rowmax_key = 0u;
        }
    }
    const int64_t S = (int64_t)1 << a.sample_shift, first = S >> 1;
    const int64_t nblk = (a.d + 1023) / 1024;
    const int64_t ns = nblk > first ? (nblk - first + S - 1) / S : 0;
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t maxkey = 0;
    // a wave's blocks, the loads of the next one in flight while the current one is reduced
    const int64_t i0 = (int64_t)blockIdx.x * (SMAX_THREADS / 64) + wave, istride = (int64_t)gridDim.x * (SMAX_THREADS / 64);
    auto fetch = [&](int64_t i, uint32_t (&b)[4][4]) {
        const int64_t blk = first + i * S;
        const int64_t base = blk * 1024 + lane * 4;
        if ((blk + 1) * 1024 <= a.d) {   // a whole block: four loads in flight
#pragma unroll
            for (int q = 0; q < 4; ++q) ld.load4_stream(base + q * 256, b[q]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) ld.load4(base + q * 256, b[q]);   // past the end: +0
        }
    };
    auto reduce = [&](const uint32_t (&b)[4][4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = key_of_bits(b[q][c]);
                maxkey = key > maxkey ? key : maxkey;
            }
    };
    uint32_t b0[4][4], b1[4][4];
    int64_t i = i0;
    if (i < ns) fetch(i, b0);
    for (; i < ns; i += 2 * istride) {
        const bool more1 = i + istride < ns, more2 = i + 2 * istride < ns;   // uniform
        if (more1) fetch(i + istride, b1);
        reduce(b0);
        if (more2) fetch(i + 2 * istride, b0);
        if (more1) reduce(b1);
    }
    // the waves' maxima meet in LDS: atomics of many waves on one address take turns
    maxkey = wave_max(maxkey);
    __shared__ uint32_t s_wmax[SMAX_THREADS / 64];
    if (lane == 0) s_wmax[wave] = maxkey;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = 0;
#pragma unroll
        for (int w = 0; w < SMAX_THREADS / 64; ++w) m = s_wmax[w] > m ? s_wmax[w] : m;
        if (PARTS) {
            ((uint32_t*)a.racc[row].gsum)[blockIdx.x] = m;   // a non-finite entry is reported by the extraction, which sees every entry
        } else if (m) {
            atomicMax(&a.racc[row].smpmax_key, m);
            if (m >= 0x7F800000u) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
        }
    }
}

// The largest key k_bits_smax found in a row (every lane of the calling wave gets it).
__device__ __forceinline__ uint32_t row_smpmax(const BitsArgs& a, int row) {
    const RowAcc* ra = a.racc + row;
    if (a.smax_parts == 0) return ra->smpmax_key;
    const uint32_t* part = (const uint32_t*)ra->gsum;
    uint32_t m = 0;
    for (int i = (int)lane_id(); i < a.smax_parts; i += 64) {
        const uint32_t v = part[i];
        m = v > m ? v : m;
    }
    return wave_max(m);
}

// v_writelane_b32 through its compiler intrinsic (this compiler has no builtin of that name): the result is `old`
// with lane `lane` (uniform) replaced by the uniform value `sval`.  As an intrinsic, not inline assembly, so that
// the compiler keeps the wait states the instruction needs after the compare that produced sval.
extern "C" __device__ int mlmc_writelane_i32(int sval, int lane, int old) __asm("llvm.amdgcn.writelane.i32");
__device__ __forceinline__ void put_lane(uint32_t& dst, uint32_t sval, int lane) {
    dst = (uint32_t)mlmc_writelane_i32((int)sval, lane, (int)dst);
}

// ---------------------------------------------------------------------------------------------------
// Round-to-Nearest ladder (Sec. 3.3, App. G.2).  Code of magnitude a at width b: n = rne(a D / (2c)), D = 2^b - 1, cut
// at N = 2^(b-1) - 1.  a D is an exact double (40 bits); n0 = rint(a D * (1 / 2c)) is off by at most one, and the
// remainder a D - n0 2c, exact in one fused multiply-add, decides: beyond +-c the neighbour, exactly +-c the even one.
struct RtnCode {
    double D;     // 2^b - 1 (0: no such code)
    int32_t N;    // 2^(b-1) - 1
    int32_t b;    // width in bits
};
__device__ __forceinline__ int32_t rtn_code_abs(double a, const RtnCode& k, double c, double den, double inv_den) {
    const double num = __dmul_rn(a, k.D);
    double n = rint(__dmul_rn(num, inv_den));
    const double rem = __fma_rn(-n, den, num);
    n += rem > c ? 1.0 : 0.0;
    n -= rem < -c ? 1.0 : 0.0;
    int32_t ni = (int32_t)n;
    if ((rem == c || rem == -c) && (ni & 1)) ni += rem > 0.0 ? 1 : -1;
    return ni < k.N ? ni : k.N;
}
// The same code as a double, the short way.  n = rint(a D / 2c) computed with the rounded reciprocal is the exact
// round-to-nearest-even unless the exact quotient lies within 2^-37 of a half-integer; the remainder a D - n 2c, exact
// in one fused multiply-add, tells: below c in magnitude, n is right (and, a being below c then, inside the code's
// range); otherwise (a tie, a near tie, the largest entry itself, a non-finite c) the code is computed the long way.
__device__ __forceinline__ double rtn_code_f64(double a, const RtnCode& k, double c, double den, double inv_den) {
    const double num = __dmul_rn(a, k.D);
    double n = rint(__dmul_rn(num, inv_den));
    const double rem = __fma_rn(-n, den, num);
    if (__builtin_expect(!(fabs(rem) < c), 0)) n = (double)rtn_code_abs(a, k, c, den, inv_den);
    return n;
}
__device__ __forceinline__ RtnCode rtn_code_of(int b) {
    RtnCode k;
    k.b = b;
    k.D = b > 0 ? (double)((1 << b) - 1) : 0.0;
    k.N = b > 0 ? (1 << (b - 1)) - 1 : 0;
    return k;
}
// |g| as an exact double from its key
__device__ __forceinline__ double key_to_double(uint32_t key) {
    const uint32_t E = key >> 23;
    return ldexp((double)(E ? (key & 0x7FFFFFu) | 0x800000u : key), (int)(E ? E : 1u) - 150);
}
struct RtnRow {          // what the extraction of a row needs: c and the (up to three) codes of its message, in plane order
    double c, den, inv_den;
    RtnCode code[3];
};

// One wave packs one tile of 4096 elements: iteration i covers elements [64 i, 64 i + 64) of the tile, so a
// ballot is the plane word of those 64 elements; it is kept in lane i and the 64 words of a plane go out in one
// store.  Emax is the exponent the scale is taken from.  NPC: compile-time bound on the planes of the row (np <= NPC);
// BASE: the ladder has a base field (F_0 > 0).  Returns the largest key met, through maxkey.
//
// Digits (Sec. 3.1): |g| = sig * 2^(E' - 150), scale s = 2^(Emax - 126), so floor(|g| / s * 2^F) = sig >> (24 - F + Emax - E').
// Bit b of (sig >> (24 - F_l + Emax - E')) for b < F_l - F_{l-1} is bit b of the level field.
// MODE 0 / 1: fixed-point ladder without / with a base field (F_0 > 0); MODE 2: floating-point ladder (App. B);
// MODE 3 / 4: fixed-point ladder of |g| / v, v the largest entry of the row (vd, as a double; vr = 1 / vd), without /
// with a base field; MODE 5: Round-to-Nearest ladder: the planes are the bits of the row's codes (no sign plane:
// plane p is bit p of the value `digits` returns).  MODE 3 / 4 digits: m = min(floor(|g| 2^Q / v), 2^Q - 1), Q = F_L.  |g| 2^Q and v are exact doubles;
// n = trunc(|g| 2^Q * vr) is off by at most one, and the remainder |g| 2^Q - n v, exact in one fused multiply-add
// (n v has at most 48 bits), says which way.
template <int DT, bool VEC, int NPC, int MODE>
__device__ __forceinline__ void bits_extract_tiles(const BitsArgs& a, int row, int Emax, int level, int np, uint32_t& maxkey,
                                                   uint32_t* slds, double vd = 0.0, double vr = 0.0, const RtnRow* rr = nullptr) {
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    RowLoader<DT, false> ld(a.g, a.ld, a.d, row);
    RowLoader<DT, VEC> ld4(a.g, a.ld, a.d, row);
    const int64_t ntiles = (a.d + TILE - 1) / TILE;
    const int64_t nwhole = a.d / TILE;   // tiles with all 4096 elements
    const int F0 = a.F[0];
    constexpr bool BASE = MODE == 1 || MODE == 4;
    const int Q = a.F[a.L];
    const uint32_t vcap = vd > 0.0 ? (Q >= 32 ? 0xFFFFFFFFu : (1u << Q) - 1u) : 0u;   // a zero row has only zero digits
    const uint32_t vsl = (uint32_t)(Q - a.F[level]), vs0 = (uint32_t)(Q - F0);
    const uint32_t Cl = (uint32_t)(24 - a.F[level] + Emax), C0 = (uint32_t)(24 - F0 + Emax);
    const uint32_t mask0 = BASE ? (1u << F0) - 1u : 0u;
    const uint32_t fsl = (uint32_t)(23 - a.F[level]), fs0 = (uint32_t)(23 - F0);   // floating-point ladder: digit positions
    uint32_t wlo[NPC], whi[NPC];   // lane i: word i of the tile's planes
#pragma unroll
    for (int p = 0; p < NPC; ++p) { wlo[p] = 0; whi[p] = 0; }
    // plane p >= 1 <-> bit p - 1 of the value returned here (base field first, then the level field; for the
    // floating-point ladder the eight exponent bits come first)
    auto digits = [&](uint32_t bits) -> uint32_t {
        const uint32_t key = key_of_bits(bits);
        maxkey = key > maxkey ? key : maxkey;
        const uint32_t E = key >> 23;
        if (MODE == 5) {
            // the codes of the message, two's complement cut to their widths, one after the other from bit 0
            const double av = key_to_double(key);
            uint32_t x = 0, at = 0;
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const RtnCode kq = rr->code[q];
                if (kq.b > 0) {   // uniform
                    int32_t n = rr->c > 0.0 ? (int32_t)rtn_code_f64(av, kq, rr->c, rr->den, rr->inv_den) : 0;
                    n = (int32_t)bits < 0 ? -n : n;
                    x |= ((uint32_t)n & ((1u << kq.b) - 1u)) << at;
                    at += (uint32_t)kq.b;
                }
            }
            return x;
        }
        if (MODE == 2) {
            // App. B: the digits m_1..m_F of the mantissa are the top F bits of the 23-bit fraction field
            const uint32_t frac = key & 0x7FFFFFu;
            const uint32_t base = F0 ? frac >> fs0 : 0u;
            return E | ((base | ((frac >> fsl) << F0)) << 8);
        }
        const uint32_t hid = (key & 0x7FFFFFu) | 0x800000u;
        const uint32_t sig = key < hid ? key : hid;       // exponent field 0: no hidden bit
        const uint32_t Ec = E > 1u ? E : 1u;
        if (MODE >= 3) {
            const double xg = ldexp((double)sig, (int)Ec - 150 + Q);   // |g| 2^Q
            uint32_t n = (uint32_t)__dmul_rn(xg, vr);
            const double rem = __fma_rn(-(double)n, vd, xg);
            n += rem >= vd ? 1u : 0u;
            n -= rem < 0.0 ? 1u : 0u;
            n = n < vcap ? n : vcap;
            const uint32_t xv = n >> vsl;
            if (!BASE) return xv;
            return ((n >> vs0) & mask0) | (xv << F0);
        }
        const uint32_t sl = Cl - Ec;                      // >= 32 (also "negative"): every digit is zero
        const uint32_t x = sig >> (sl < 31u ? sl : 31u);
        if (!BASE) return x;
        const uint32_t s0 = C0 - Ec;
        const uint32_t x0 = sig >> (s0 < 31u ? s0 : 31u);
        return (x0 & mask0) | (x << F0);
    };
    // the ballots of iteration i (elements 64 i .. 64 i + 63 of the tile, one per lane) go to lane i of the tile's words
    auto pack16 = [&](int g4, const uint32_t (&v)[16]) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int i = g4 * 16 + u;
            const uint32_t bits = v[u];
            const uint32_t x = digits(bits);
            {
                const uint64_t w = __ballot(MODE == 5 ? (x & 1u) != 0u : (int32_t)bits < 0);
                put_lane(wlo[0], (uint32_t)w, i);
                put_lane(whi[0], (uint32_t)(w >> 32), i);
            }
#pragma unroll
            for (int p = 1; p < NPC; ++p) {
                if (p < np) {   // uniform
                    const uint64_t w = __ballot((x & (1u << (MODE == 5 ? p : p - 1))) != 0u);
                    put_lane(wlo[p], (uint32_t)w, i);
                    put_lane(whi[p], (uint32_t)(w >> 32), i);
                }
            }
        }
    };
    auto store_words = [&](int64_t tile) {
        const int64_t w0 = tile * 64 + lane;
        if (w0 < a.nwords) {
            uint64_t* dst = a.planes + (size_t)row * a.nplanes * a.nwords + w0;
#pragma unroll
            for (int p = 0; p < NPC; ++p)
                if (p < np) dst[(size_t)p * a.nwords] = ((uint64_t)whi[p] << 32) | wlo[p];
        }
    };
    const int64_t first = (int64_t)blockIdx.x * 4 + wave, stride = (int64_t)gridDim.x * 4;
    int64_t tile = first;
    if (VEC) {
        // Whole tiles of an aligned row: sixteen 16-byte loads per lane and tile (a load covers 256 consecutive
        // elements, four per lane), eight in flight, also across the wave's tiles.  Four loads at a time pass
        // through the wave's LDS buffer, written as loaded and read back one element per lane, so that a ballot
        // is a plane word.
        uint32_t bufA[4][4], bufB[4][4];
        auto fetch4 = [&](int64_t t, int l0, uint32_t (&buf)[4][4]) {
#pragma unroll
            for (int q = 0; q < 4; ++q) ld4.load4_stream(t * TILE + (int64_t)((l0 + q) * 256) + (int64_t)lane * 4, buf[q]);
        };
        auto transpose16 = [&](const uint32_t (&buf)[4][4], uint32_t (&v)[16]) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *(uint4*)(slds + q * 256 + lane * 4) = make_uint4(buf[q][0], buf[q][1], buf[q][2], buf[q][3]);
            wave_lds_sync();
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = slds[u * 64 + lane];
            wave_lds_sync();   // the next writes come after these reads
        };
        if (tile < nwhole) {
            fetch4(tile, 0, bufA);
            fetch4(tile, 4, bufB);
        }
        for (; tile < nwhole; tile += stride) {
            const bool more = tile + stride < nwhole;   // uniform
            uint32_t v[16];
            transpose16(bufA, v);
            fetch4(tile, 8, bufA);
            pack16(0, v);
            transpose16(bufB, v);
            fetch4(tile, 12, bufB);
            pack16(1, v);
            transpose16(bufA, v);
            if (more) fetch4(tile + stride, 0, bufA);
            pack16(2, v);
            transpose16(bufB, v);
            if (more) fetch4(tile + stride, 4, bufB);
            pack16(3, v);
            store_words(tile);
        }
    } else {
        // a row that is not aligned for 16-byte loads: one element per lane and load, sixteen loads in flight
        for (; tile < nwhole; tile += stride) {
            for (int g4 = 0; g4 < 4; ++g4) {
                uint32_t v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = ld.load1_stream(tile * TILE + (g4 * 16 + u) * 64 + lane);
                pack16(g4, v);
            }
            store_words(tile);
        }
    }
    if (tile < ntiles) {   // the ragged last tile of the row (one wave of the row gets here)
        const int64_t base = tile * TILE;
#pragma unroll
        for (int p = 0; p < NPC; ++p) { wlo[p] = 0; whi[p] = 0; }
        for (int i = 0; i < 64; ++i) {
            const int64_t j = base + i * 64 + lane;
            const uint32_t bits = j < a.d ? ld.load1(j) : 0u;
            const uint32_t x = digits(bits);
            const bool me = (int)lane == i;
            {
                const uint64_t w = __ballot(MODE == 5 ? (x & 1u) != 0u : (int32_t)bits < 0);
                wlo[0] = me ? (uint32_t)w : wlo[0];
                whi[0] = me ? (uint32_t)(w >> 32) : whi[0];
            }
#pragma unroll
            for (int p = 1; p < NPC; ++p) {
                if (p < np) {   // uniform
                    const uint64_t w = __ballot((x & (1u << (MODE == 5 ? p : p - 1))) != 0u);
                    wlo[p] = me ? (uint32_t)w : wlo[p];
                    whi[p] = me ? (uint32_t)(w >> 32) : whi[p];
                }
            }
        }
        store_words(tile);
    }
}

// The row's message under the scale taken from the sampled maximum; the true maximum of the row is tracked on the
// way.  REDO (second launch, only when the maximum was sampled): rows whose true maximum has a larger exponent than
// the sampled one are extracted again with the true one; every other row is already final and is skipped.
// NPCMAX: bound on the planes of any row of the plan (the kernel holds only the variants it can need, so that a
// plan with few planes is not charged the registers of the widest one).  FLT: floating-point ladder (no scale).
// KIND 2: fixed-point ladder of |g| / v: the row maximum was read exactly beforehand (sample of every block).
template <int DT, bool VEC, bool REDO, int NPCMAX, int KIND>
__global__ __launch_bounds__(256) void k_bits_extract(BitsArgs a) {
    constexpr bool FLT = KIND == 1;
    __shared__ __align__(16) uint32_t s_tr[4][1024];   // per wave: four loads of 256 elements on their way from "four per lane" to "one per lane"
    uint32_t* slds = s_tr[threadIdx.x >> 6];
    const int row = blockIdx.y;
    RowAcc* ra = a.racc + row;
    const uint32_t smpmax = row_smpmax(a, row);
    const uint32_t Es = smpmax >> 23;
    uint32_t Ex = Es;
    if (REDO) {
        Ex = ra->rowmax_key >> 23;
        if (Ex == Es) return;
    }
    const int Emax = Ex ? (int)Ex : 1;
    const int level = a.rinfo[row].level;
    const int F0 = a.F[0];
    const int np = (FLT ? 9 : 1) + F0 + (a.F[level] - a.F[level - 1]);   // planes written for this row
    if (KIND == 0 && blockIdx.x == 0 && threadIdx.x == 0) a.scale_exp[row] = Emax - 126;
    uint32_t maxkey = 0;
    if constexpr (KIND == 2) {
        const uint32_t vkey = smpmax;   // the largest |g| of the row
        if (blockIdx.x == 0 && threadIdx.x == 0) a.scale_exp[row] = (int32_t)vkey;
        const uint32_t vE = vkey >> 23;
        const double vd = ldexp((double)(vE ? (vkey & 0x7FFFFFu) | 0x800000u : vkey), (int)(vE ? vE : 1u) - 150);
        const double vr = vd > 0.0 ? __ddiv_rn(1.0, vd) : 0.0;
        if (F0 == 0) {
            if (np <= 9) bits_extract_tiles<DT, VEC, 9, 3>(a, row, Emax, level, np, maxkey, slds, vd, vr);
            else if constexpr (NPCMAX > 9) bits_extract_tiles<DT, VEC, MAX_PLANES, 3>(a, row, Emax, level, np, maxkey, slds, vd, vr);
        } else {
            if (np <= 9) bits_extract_tiles<DT, VEC, 9, 4>(a, row, Emax, level, np, maxkey, slds, vd, vr);
            else if constexpr (NPCMAX > 9) bits_extract_tiles<DT, VEC, MAX_PLANES, 4>(a, row, Emax, level, np, maxkey, slds, vd, vr);
        }
    } else if constexpr (FLT) {
        if (np <= 11) bits_extract_tiles<DT, VEC, 11, 2>(a, row, Emax, level, np, maxkey, slds);
        else if constexpr (NPCMAX > 11) {
            if (np <= 17) bits_extract_tiles<DT, VEC, 17, 2>(a, row, Emax, level, np, maxkey, slds);
            else if (np <= 25) bits_extract_tiles<DT, VEC, 25, 2>(a, row, Emax, level, np, maxkey, slds);
            else bits_extract_tiles<DT, VEC, MAX_FPLANES, 2>(a, row, Emax, level, np, maxkey, slds);
        }
    } else if (F0 == 0) {
        if (np <= 3) bits_extract_tiles<DT, VEC, 3, 0>(a, row, Emax, level, np, maxkey, slds);
        else if (np <= 5) bits_extract_tiles<DT, VEC, 5, 0>(a, row, Emax, level, np, maxkey, slds);
        else if (np <= 9) bits_extract_tiles<DT, VEC, 9, 0>(a, row, Emax, level, np, maxkey, slds);
        else if constexpr (NPCMAX > 9) {
            if (np <= 17) bits_extract_tiles<DT, VEC, 17, 0>(a, row, Emax, level, np, maxkey, slds);
            else bits_extract_tiles<DT, VEC, MAX_PLANES, 0>(a, row, Emax, level, np, maxkey, slds);
        }
    } else {
        if (np <= 5) bits_extract_tiles<DT, VEC, 5, 1>(a, row, Emax, level, np, maxkey, slds);
        else if (np <= 9) bits_extract_tiles<DT, VEC, 9, 1>(a, row, Emax, level, np, maxkey, slds);
        else if constexpr (NPCMAX > 9) {
            if (np <= 17) bits_extract_tiles<DT, VEC, 17, 1>(a, row, Emax, level, np, maxkey, slds);
            else bits_extract_tiles<DT, VEC, MAX_PLANES, 1>(a, row, Emax, level, np, maxkey, slds);
        }
    }
    if (!REDO) {
        // one atomic per workgroup (the workgroups of a launch end together, and atomics on one address take turns)
        maxkey = wave_max(maxkey);
        __syncthreads();   // every wave is done with its transposing buffer
        if (lane_id() == 0) s_tr[0][threadIdx.x >> 6] = maxkey;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t m = s_tr[0][0];
#pragma unroll
            for (int w = 1; w < 4; ++w) m = s_tr[0][w] > m ? s_tr[0][w] : m;
            if (m) {
                atomicMax(&ra->rowmax_key, m);
                if (m >= 0x7F800000u) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
            }
        }
    }
}

}  // namespace mlmc
