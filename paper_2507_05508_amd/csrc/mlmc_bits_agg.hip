// Fixed-point bit-wise MLMC (Sec. 3.1) and the server aggregate (Alg. 2 / Alg. 3) on gfx950.
//
//   k_bits_prep     level draw of every row
//   k_bits_smax     largest |g| key of a sample of every row (integer atomic max) -> predicted power-of-two scale
//   k_bits_extract  the one full read: digits floor(|g_j| / s * 2^F), sign plane + field planes packed by wave
//                   ballot, and the true row maximum; a row whose true maximum has a larger exponent than the
//                   sampled one is extracted again by a second launch (which returns at once for every other row)
//   k_agg_bits      out = alpha * sum_i decode_i, rows added in worker order
//   k_tileoff       (fallback) per-tile offsets of index-sorted sparse rows by binary search
//   k_agg_sparse    atomic-free segmented scatter-add: one workgroup owns one dense tile
#include "mlmc_device.h"

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

// Largest |g| key of the sampled blocks of every row (block b of 1024 elements is sampled when b % S == S / 2,
// S = 2^sample_shift; S = 1 reads the whole row and the result is the row maximum itself).
constexpr int SMAX_THREADS = 512;
template <int DT, bool VEC>
__global__ __launch_bounds__(SMAX_THREADS) void k_bits_smax(BitsArgs a) {
    const int row = blockIdx.y;
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
    maxkey = wave_max(maxkey);
    if (lane == 0 && maxkey) {
        atomicMax(&a.racc[row].smpmax_key, maxkey);
        if (maxkey >= 0x7F800000u) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
    }
}

// v_writelane_b32 through its compiler intrinsic (this compiler has no builtin of that name): the result is `old`
// with lane `lane` (uniform) replaced by the uniform value `sval`.  As an intrinsic, not inline assembly, so that
// the compiler keeps the wait states the instruction needs after the compare that produced sval.
extern "C" __device__ int mlmc_writelane_i32(int sval, int lane, int old) __asm("llvm.amdgcn.writelane.i32");
__device__ __forceinline__ void put_lane(uint32_t& dst, uint32_t sval, int lane) {
    dst = (uint32_t)mlmc_writelane_i32((int)sval, lane, (int)dst);
}

// One wave packs one tile of 4096 elements: iteration i covers elements [64 i, 64 i + 64) of the tile, so a
// ballot is the plane word of those 64 elements; it is kept in lane i and the 64 words of a plane go out in one
// store.  Emax is the exponent the scale is taken from.  NPC: compile-time bound on the planes of the row (np <= NPC);
// BASE: the ladder has a base field (F_0 > 0).  Returns the largest key met, through maxkey.
//
// Digits (Sec. 3.1): |g| = sig * 2^(E' - 150), scale s = 2^(Emax - 126), so floor(|g| / s * 2^F) = sig >> (24 - F + Emax - E').
// Bit b of (sig >> (24 - F_l + Emax - E')) for b < F_l - F_{l-1} is bit b of the level field.
// MODE 0 / 1: fixed-point ladder without / with a base field (F_0 > 0); MODE 2: floating-point ladder (App. B);
// MODE 3 / 4: fixed-point ladder of |g| / v, v the largest entry of the row (vd, as a double; vr = 1 / vd), without /
// with a base field.  Its digits: m = min(floor(|g| 2^Q / v), 2^Q - 1), Q = F_L.  |g| 2^Q and v are exact doubles;
// n = trunc(|g| 2^Q * vr) is off by at most one, and the remainder |g| 2^Q - n v, exact in one fused multiply-add
// (n v has at most 48 bits), says which way.
template <int DT, bool VEC, int NPC, int MODE>
__device__ __forceinline__ void bits_extract_tiles(const BitsArgs& a, int row, int Emax, int level, int np, uint32_t& maxkey,
                                                   uint32_t* slds, double vd = 0.0, double vr = 0.0) {
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
                const uint64_t w = __ballot((int32_t)bits < 0);
                put_lane(wlo[0], (uint32_t)w, i);
                put_lane(whi[0], (uint32_t)(w >> 32), i);
            }
#pragma unroll
            for (int p = 1; p < NPC; ++p) {
                if (p < np) {   // uniform
                    const uint64_t w = __ballot((x & (1u << (p - 1))) != 0u);
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
                const uint64_t w = __ballot((int32_t)bits < 0);
                wlo[0] = me ? (uint32_t)w : wlo[0];
                whi[0] = me ? (uint32_t)(w >> 32) : whi[0];
            }
#pragma unroll
            for (int p = 1; p < NPC; ++p) {
                if (p < np) {   // uniform
                    const uint64_t w = __ballot((x & (1u << (p - 1))) != 0u);
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
    const uint32_t Es = ra->smpmax_key >> 23;
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
        const uint32_t vkey = ra->smpmax_key;   // the largest |g| of the row
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
        maxkey = wave_max(maxkey);
        if (lane_id() == 0 && maxkey) {
            atomicMax(&ra->rowmax_key, maxkey);
            if (maxkey >= 0x7F800000u) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
        }
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
        double pl = b.p_fixed[lev - 1];
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
            if (b.flt) {
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
mlmc_status bits_compress(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, hipStream_t st) {
    MLMC_LAUNCH(K_DRAW, st, k_bits_prep<<<1, 1024, 0, st>>>(a));
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
    if (pl->dtype == MLMC_F32) {
        if (vec) MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_F32, true><<<sgrid, SMAX_THREADS, 0, st>>>(a));
        else MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_F32, false><<<sgrid, SMAX_THREADS, 0, st>>>(a));
    } else {
        if (vec) MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_BF16, true><<<sgrid, SMAX_THREADS, 0, st>>>(a));
        else MLMC_LAUNCH(K_BITS_MAX, st, k_bits_smax<MLMC_BF16, false><<<sgrid, SMAX_THREADS, 0, st>>>(a));
    }
    const bool small = pl->nplanes <= 9;
    if (a.vmx) {   // the maxima above are exact (every block was read): one extraction
        MLMC_EXTRACT(K_BITS_EXTRACT, false, 2, 9, MAX_PLANES);
        return MLMC_OK;
    }
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
