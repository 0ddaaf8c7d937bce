// Device-side helpers: wave64 primitives, row loaders, key arithmetic, Philox4x32-10.
#pragma once
#include "mlmc_internal.h"

namespace mlmc {

__device__ __forceinline__ uint32_t lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// number of set bits of m below this lane
__device__ __forceinline__ uint32_t mbcnt(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Orders LDS traffic between the lanes of one wave (no instruction beyond the waits the fences need).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        uint32_t u = __shfl_xor(v, o, 64);
        v = u > v ? u : v;
    }
    return v;
}

// Exclusive prefix over the lanes of a small count c (0..7), and the wave total.
__device__ __forceinline__ uint32_t wave_excl_small(uint32_t c, uint32_t& total) {
    uint64_t b0 = __ballot(c & 1u), b1 = __ballot(c & 2u), b2 = __ballot(c & 4u);
    total = __popcll(b0) + 2u * __popcll(b1) + 4u * __popcll(b2);
    return mbcnt(b0) + 2u * mbcnt(b1) + 4u * mbcnt(b2);
}

// Exclusive scan over a workgroup of NT threads (NT multiple of 64, <= 1024). `lds` holds NT/64 + 1 words.
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* lds, uint32_t& total) {
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        uint32_t u = __shfl_up(inc, o, 64);
        if (lane >= (uint32_t)o) inc += u;
    }
    __syncthreads();
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int w = 0; w < NT / 64; ++w) {
            uint32_t t = lds[w];
            lds[w] = run;
            run += t;
        }
        lds[NT / 64] = run;
    }
    __syncthreads();
    total = lds[NT / 64];
    return lds[wave] + inc - v;
}

// Strided loop over [i0, i1) for a group of NT threads (this thread starts at i0 + t): U loads are issued back to
// back before the first is consumed.  A loop whose every load sits behind its own bounds check is compiled to one
// load, one wait per iteration; here whole batches take a branch-free path and the ragged rest is one more batch
// whose out-of-range loads are redirected to the last element and discarded.
template <int U, int NT, class Load, class Proc>
__device__ __forceinline__ void batched_loop(uint32_t i0, uint32_t i1, uint32_t t, Load load, Proc proc) {
    if (i1 <= i0) return;
    uint32_t i = i0 + t;
    if (i1 >= (uint32_t)((U - 1) * NT)) {
        const uint32_t lim = i1 - (uint32_t)((U - 1) * NT);   // i + (U-1)*NT < i1  <=>  i < lim
        for (; i < lim; i += (uint32_t)(U * NT)) {
            decltype(load(0u)) v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load(i + (uint32_t)(u * NT));
#pragma unroll
            for (int u = 0; u < U; ++u) proc(i + (uint32_t)(u * NT), v[u]);
        }
    }
    if (i < i1) {   // fewer than U strides are left for this thread
        decltype(load(0u)) v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t k = i + (uint32_t)(u * NT);
            v[u] = load(k < i1 ? k : i1 - 1u);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t k = i + (uint32_t)(u * NT);
            if (k < i1) proc(k, v[u]);
        }
    }
}

// ---- keys ----------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t key_of_bits(uint32_t fp32_bits) { return fp32_bits & 0x7FFFFFFFu; }

// square of the 24-bit significand (no hidden bit when the exponent field is 0): < 2^48
__device__ __forceinline__ uint64_t sig_square(uint32_t key) {
    uint32_t frac = key & 0x7FFFFFu;
    uint32_t sig = (key >> 23) ? (frac | 0x800000u) : frac;
    return (uint64_t)sig * (uint64_t)sig;
}

// ---- row loaders: four consecutive elements starting at j (j % 4 == 0), as fp32 bit patterns -------
// DT = MLMC_F32 / MLMC_BF16.  VEC: the row start and ld allow one aligned 16-byte (8-byte for bf16) load.
template <int DT, bool VEC>
struct RowLoader {
    const void* row;
    int64_t d;
    __device__ __forceinline__ RowLoader(const void* g, int64_t ld, int64_t d_, int r) : d(d_) {
        if (DT == MLMC_F32)
            row = (const void*)((const float*)g + (int64_t)r * ld);
        else
            row = (const void*)((const uint16_t*)g + (int64_t)r * ld);
    }
    // returns the number of valid elements (0..4); invalid ones read as +0
    __device__ __forceinline__ int load4(int64_t j, uint32_t (&b)[4]) const {
        int64_t left = d - j;
        int nv = left >= 4 ? 4 : (left > 0 ? (int)left : 0);
        if (DT == MLMC_F32) {
            const uint32_t* p = (const uint32_t*)row + j;
            if (VEC && nv == 4) {
                uint4 v = *(const uint4*)p;
                b[0] = v.x; b[1] = v.y; b[2] = v.z; b[3] = v.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) b[c] = c < nv ? p[c] : 0u;
            }
        } else {
            const uint16_t* p = (const uint16_t*)row + j;
            if (VEC && nv == 4) {
                uint2 v = *(const uint2*)p;
                b[0] = v.x << 16; b[1] = v.x & 0xFFFF0000u; b[2] = v.y << 16; b[3] = v.y & 0xFFFF0000u;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) b[c] = c < nv ? ((uint32_t)p[c] << 16) : 0u;
            }
        }
        return nv;
    }
    // four consecutive elements that are all inside the row (j + 4 <= d): no branch, so that several of these
    // loads can be in flight before the first result is needed
    __device__ __forceinline__ void load4_full(int64_t j, uint32_t (&b)[4]) const {
        if (DT == MLMC_F32) {
            const uint32_t* p = (const uint32_t*)row + j;
            if (VEC) {
                uint4 v = *(const uint4*)p;
                b[0] = v.x; b[1] = v.y; b[2] = v.z; b[3] = v.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) b[c] = p[c];
            }
        } else {
            const uint16_t* p = (const uint16_t*)row + j;
            if (VEC) {
                uint2 v = *(const uint2*)p;
                b[0] = v.x << 16; b[1] = v.x & 0xFFFF0000u; b[2] = v.y << 16; b[3] = v.y & 0xFFFF0000u;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) b[c] = (uint32_t)p[c] << 16;
            }
        }
    }
    // load4_full for a row that is streamed through once: a non-temporal load, so that the row does not push
    // what the kernel writes and reads back soon after (its staged lists) out of the L2
    __device__ __forceinline__ void load4_stream(int64_t j, uint32_t (&b)[4]) const {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        if (DT == MLMC_F32 && VEC) {
            const u32x4 v = __builtin_nontemporal_load((const u32x4*)((const uint32_t*)row + j));
            b[0] = v.x; b[1] = v.y; b[2] = v.z; b[3] = v.w;
        } else if (DT != MLMC_F32 && VEC) {
            const u32x2 v = __builtin_nontemporal_load((const u32x2*)((const uint16_t*)row + j));
            b[0] = v.x << 16; b[1] = v.x & 0xFFFF0000u; b[2] = v.y << 16; b[3] = v.y & 0xFFFF0000u;
        } else {
            load4_full(j, b);
        }
    }
    __device__ __forceinline__ uint32_t load1_stream(int64_t j) const {
        if (DT == MLMC_F32) return __builtin_nontemporal_load((const uint32_t*)row + j);
        return (uint32_t)__builtin_nontemporal_load((const uint16_t*)row + j) << 16;
    }
    __device__ __forceinline__ uint32_t load1(int64_t j) const {
        if (DT == MLMC_F32) return ((const uint32_t*)row)[j];
        return (uint32_t)((const uint16_t*)row)[j] << 16;
    }
};

// ---- Philox4x32-10 (Salmon et al., SC'11), from the published round function ----------------------
__device__ __forceinline__ uint32_t philox_word0(uint64_t seed, uint64_t step, uint32_t worker) {
    uint32_t c0 = (uint32_t)step, c1 = (uint32_t)(step >> 32), c2 = worker, c3 = 0u;
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        uint64_t pa = (uint64_t)0xD2511F53u * c0;
        uint64_t pb = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)pb;
        c3 = (uint32_t)pa;
        c0 = n0;
        c2 = n2;
    }
    return c0;
}

// Level draw shared by the Top-k and bit-wise paths: integer inverse CDF of one 32-bit uniform.
// p: L probabilities (local array).  Returns the level in 1..L.
__device__ __forceinline__ int draw_from_p(const double* p, int L, uint32_t x) {
    double c = 0.0;
    int level = L;
    bool found = false;
    for (int l = 0; l < L; ++l) {
        c = __dadd_rn(c, p[l]);
        double t = floor(__dmul_rn(c, 4294967296.0));
        uint64_t T;
        if (!(t > 0.0)) T = 0;
        else if (t >= 4294967296.0) T = 4294967296ull;
        else T = (uint64_t)t;
        if (l == L - 1) T = 4294967296ull;
        if (!found && (uint64_t)x < T) {
            level = l + 1;
            found = true;
        }
    }
    return level;
}

// ---- exact sums of squares: a 640-bit integer count of 2^-298 units -> correctly rounded fp64 ----------
struct BigAcc {
    uint32_t* w;  // 20 words, least significant first
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

}  // namespace mlmc
