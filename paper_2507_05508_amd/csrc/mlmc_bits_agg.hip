// Fixed-point bit-wise MLMC (Sec. 3.1) and the server aggregate (Alg. 2 / Alg. 3) on gfx950.
//
//   k_bits_max      row maximum of the |g| keys (integer atomic max) -> power-of-two scale
//   k_bits_extract  digits m_j = floor(|g_j| / s * 2^Q), sign plane + field planes packed by wave ballot
//   k_agg_bits      out = alpha * sum_i decode_i, rows added in worker order
//   k_tileoff       (fallback) per-tile offsets of index-sorted sparse rows by binary search
//   k_agg_sparse    atomic-free segmented scatter-add: one workgroup owns one dense tile
#include "mlmc_device.h"

namespace mlmc {

// ---------------------------------------------------------------------------------------------------
constexpr int BITS_MAX_CHUNKS = 4;
template <int DT, bool VEC>
__global__ __launch_bounds__(512) void k_bits_max(BitsArgs a) {
    const int row = blockIdx.y;
    const int64_t span = (int64_t)a.chunk * BITS_MAX_CHUNKS;   // several chunks per workgroup: long unchecked runs
    const int64_t c0 = (int64_t)blockIdx.x * span;
    const int64_t c1 = c0 + span < a.d ? c0 + span : a.d;
    RowLoader<DT, VEC> ld(a.g, a.ld, a.d, row);
    uint32_t maxkey = 0;
    constexpr int64_t STEP = 512 * 4;
    int64_t j = c0 + (int64_t)threadIdx.x * 4;
    for (; j + 3 * STEP + 4 <= c1; j += 4 * STEP) {   // four loads in flight, no bounds checks inside
        uint32_t b[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) ld.load4_full(j + u * STEP, b[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = key_of_bits(b[u][c]);
                maxkey = key > maxkey ? key : maxkey;
            }
    }
    for (; j < c1; j += STEP) {
        uint32_t b[4];
        int nv = ld.load4(j, b);
        if (j + nv > c1) nv = (int)(c1 - j);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t key = c < nv ? key_of_bits(b[c]) : 0u;
            maxkey = key > maxkey ? key : maxkey;
        }
    }
    maxkey = wave_max(maxkey);
    if (lane_id() == 0) {
        atomicMax(&a.racc[row].rowmax_key, maxkey);
        if (maxkey >= 0x7F800000u) atomicOr(a.dev_status, MLMC_DEV_NONFINITE);
    }
}

// Per-row constants of the extraction / decode.
struct BitsRow {
    int level, Emax, Q, F0, Fl, width;
};
__device__ __forceinline__ BitsRow bits_row(const BitsArgs& a, int row) {
    BitsRow r;
    r.level = a.rinfo[row].level;
    uint32_t E = a.racc[row].rowmax_key >> 23;
    r.Emax = E ? (int)E : 1;
    r.Q = a.F[a.L];
    r.F0 = a.F[0];
    r.Fl = a.F[r.level];
    r.width = a.F[r.level] - a.F[r.level - 1];
    return r;
}

// One wave packs one tile of 4096 elements: iteration i covers elements [64 i, 64 i + 64) of the tile, so a
// ballot is the plane word of those 64 elements; lane i keeps word i and the 64 words go out in one store.
// NPC: compile-time bound on the planes of the row (its actual count np <= NPC), so that the per-slot loop over
// planes is as long as needed and no longer.
template <int DT, int NPC>
__device__ __forceinline__ void bits_extract_row(const BitsArgs& a, int row, const BitsRow& br, int np) {
    const uint32_t lane = lane_id(), wave = (uint32_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    RowLoader<DT, false> ld(a.g, a.ld, a.d, row);
    const int64_t ntiles = (a.d + TILE - 1) / TILE;
    // tiles (and rows) are taken from the end: what the scale pass read last is the part of the input that the
    // memory-side cache most likely still holds
    for (int64_t rt = (int64_t)blockIdx.x * 4 + wave; rt < ntiles; rt += (int64_t)gridDim.x * 4) {
        const int64_t tile = ntiles - 1 - rt;
        const int64_t base = tile * TILE;
        uint64_t words[NPC];
#pragma unroll
        for (int p = 0; p < NPC; ++p) words[p] = 0;
        auto digits = [&](uint32_t bits) -> uint32_t {
            uint32_t key = key_of_bits(bits);
            uint32_t E = key >> 23;
            uint32_t sig = E ? ((key & 0x7FFFFFu) | 0x800000u) : (key & 0x7FFFFFu);
            int shift = (24 - br.Q) + (br.Emax - (int)(E ? E : 1u));
            uint32_t m = shift < 32 ? (sig >> shift) : 0u;   // floor(|g| / 2^e * 2^Q), e = Emax - 126
            uint32_t f0 = br.F0 ? (m >> (br.Q - br.F0)) : 0u;
            uint32_t f = (m >> (br.Q - br.Fl)) & ((1u << br.width) - 1u);
            return (bits >> 31) | (f0 << 1) | (f << (1 + br.F0));  // plane p <-> bit p
        };
        auto pack = [&](int i, uint32_t packed) {
#pragma unroll
            for (int p = 0; p < NPC; ++p) {
                if (p < np) {
                    uint64_t w = __ballot((packed >> p) & 1u);
                    if (lane == (uint32_t)i) words[p] = w;
                }
            }
        };
        if (base + TILE <= a.d) {   // a whole tile: sixteen loads in flight, no bounds checks inside
            for (int i0 = 0; i0 < 64; i0 += 16) {
                uint32_t v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = ld.load1_stream(base + (i0 + u) * 64 + lane);
#pragma unroll
                for (int u = 0; u < 16; ++u) pack(i0 + u, digits(v[u]));
            }
        } else {
            for (int i = 0; i < 64; ++i) {
                const int64_t j = base + i * 64 + lane;
                const uint32_t bits = j < a.d ? ld.load1(j) : 0u;
                pack(i, digits(bits));
            }
        }
        const int64_t w0 = tile * 64 + lane;
        if (w0 < a.nwords) {
            uint64_t* dst = a.planes + (size_t)row * a.nplanes * a.nwords + w0;
#pragma unroll
            for (int p = 0; p < NPC; ++p)
                if (p < np) dst[(size_t)p * a.nwords] = words[p];
        }
    }
}

// One wave packs one tile of 4096 elements: iteration i covers elements [64 i, 64 i + 64) of the tile, so a
// ballot is the plane word of those 64 elements; lane i keeps word i and the 64 words go out in one store.
template <int DT>
__global__ __launch_bounds__(256) void k_bits_extract(BitsArgs a) {
    const int row = a.M - 1 - (int)blockIdx.y;
    const BitsRow br = bits_row(a, row);
    const int np = 1 + br.F0 + br.width;  // planes written for this row
    if (blockIdx.x == 0 && threadIdx.x == 0) a.scale_exp[row] = br.Emax - 126;
    if (np <= 3) bits_extract_row<DT, 3>(a, row, br, np);
    else if (np <= 5) bits_extract_row<DT, 5>(a, row, br, np);
    else if (np <= 9) bits_extract_row<DT, 9>(a, row, br, np);
    else if (np <= 17) bits_extract_row<DT, 17>(a, row, br, np);
    else bits_extract_row<DT, MAX_PLANES>(a, row, br, np);
}

struct AggBitsArgs {
    BitsArgs b;
    const int32_t* level;
    const int32_t* scale_exp;
    const uint64_t* planes;
    float alpha;
    float* out;
};

// out[j] = alpha * sum over rows (worker order) of sign * (f0 * c0 + f * cl): Alg. 2 "Server aggregates".
// A wave owns word w of every plane, i.e. elements 64 w .. 64 w + 63 (lane = element).  The words it needs (one
// per row and plane) are fetched by different lanes in one load per group of rows; a word is then read from its
// lane as a wave-wide mask whose bit `lane` is the element's bit.  NPC bounds the planes of any row.
template <int NPC>
__global__ __launch_bounds__(256) void k_agg_bits(AggBitsArgs a) {
    __shared__ float s_c0[MLMC_MAX_WORKERS], s_cl[MLMC_MAX_WORKERS];
    __shared__ uint8_t s_w[MLMC_MAX_WORKERS];
    const BitsArgs& b = a.b;
    const int F0 = b.F[0];
    for (int r = threadIdx.x; r < b.M; r += 256) {
        int lev = a.level[r];
        int e = a.scale_exp[r];
        double pl = b.p_fixed[lev - 1];
        s_c0[r] = (float)ldexp(1.0, e - F0);
        s_cl[r] = pl == 0.0 ? 0.0f : (float)__ddiv_rn(ldexp(1.0, e - b.F[lev]), pl);
        s_w[r] = (uint8_t)(b.F[lev] - b.F[lev - 1]);
    }
    __syncthreads();
    constexpr int RPG = 64 / NPC;   // rows whose words fit one register across the wave
    const uint32_t lane = lane_id();
    const int rr_l = (int)lane / NPC, pp_l = (int)lane % NPC;
    const int64_t nw = b.nwords;
    const int64_t wave_global = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * 256) >> 6;
    for (int64_t w = wave_global; w < nw; w += nwaves) {
        float acc = 0.0f;
        for (int r0 = 0; r0 < b.M; r0 += RPG) {
            uint64_t mine = 0;
            {
                const int r = r0 + rr_l;
                if (rr_l < RPG && r < b.M && pp_l < 1 + F0 + (int)s_w[r])
                    mine = a.planes[((size_t)r * b.nplanes + pp_l) * nw + w];
            }
#pragma unroll
            for (int rr = 0; rr < RPG; ++rr) {
                const int r = r0 + rr;
                if (r < b.M) {   // uniform
                const int np = 1 + F0 + (int)s_w[r];
                uint32_t f0 = 0, f = 0;
#pragma unroll
                for (int p = 1; p < NPC; ++p) {
                    if (p < np) {   // uniform
                        const uint64_t word = ((uint64_t)__builtin_amdgcn_readlane((uint32_t)(mine >> 32), rr * NPC + p) << 32) |
                                              (uint32_t)__builtin_amdgcn_readlane((uint32_t)mine, rr * NPC + p);
                        const bool bit = __builtin_amdgcn_inverse_ballot_w64(word);
                        if (p <= F0) f0 |= bit ? 1u << (p - 1) : 0u;
                        else f |= bit ? 1u << (p - 1 - F0) : 0u;
                    }
                }
                const uint64_t sw = ((uint64_t)__builtin_amdgcn_readlane((uint32_t)(mine >> 32), rr * NPC) << 32) |
                                    (uint32_t)__builtin_amdgcn_readlane((uint32_t)mine, rr * NPC);
                const bool sign = __builtin_amdgcn_inverse_ballot_w64(sw);
                float v = __fmul_rn((float)f, s_cl[r]);
                if (F0 > 0) v = __fadd_rn(__fmul_rn((float)f0, s_c0[r]), v);
                acc = __fadd_rn(acc, sign ? -v : v);
                }
            }
        }
        const int64_t j = w * 64 + lane;
        if (j < b.d) __builtin_nontemporal_store(__fmul_rn(a.alpha, acc), &a.out[j]);
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
    float* out;
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
    __shared__ float s_acc[TILE];
    __shared__ int64_t s_beg[MLMC_MAX_WORKERS];
    __shared__ uint32_t s_len[MLMC_MAX_WORKERS];
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
        if (j < a.d) __builtin_nontemporal_store(__fmul_rn(a.alpha, s_acc[i]), &a.out[j]);   // written once, read by the caller later
    }
}

// ---------------------------------------------------------------------------------------------------
mlmc_status bits_compress(const mlmc_plan_t* pl, const BitsArgs& a, bool vec, hipStream_t st) {
    dim3 grid((pl->chunks_per_row + BITS_MAX_CHUNKS - 1) / BITS_MAX_CHUNKS, pl->M);
    if (pl->dtype == MLMC_F32) {
        if (vec) MLMC_LAUNCH(K_BITS_MAX, st, k_bits_max<MLMC_F32, true><<<grid, 512, 0, st>>>(a));
        else MLMC_LAUNCH(K_BITS_MAX, st, k_bits_max<MLMC_F32, false><<<grid, 512, 0, st>>>(a));
    } else {
        if (vec) MLMC_LAUNCH(K_BITS_MAX, st, k_bits_max<MLMC_BF16, true><<<grid, 512, 0, st>>>(a));
        else MLMC_LAUNCH(K_BITS_MAX, st, k_bits_max<MLMC_BF16, false><<<grid, 512, 0, st>>>(a));
    }
    int64_t ntiles = pl->ntiles;
    int gx = (int)((ntiles + 3) / 4);
    int cap = 4096 / pl->M > 0 ? 4096 / pl->M : 1;
    if (gx > cap) gx = cap;
    if (gx < 1) gx = 1;
    dim3 egrid(gx, pl->M);
    if (pl->dtype == MLMC_F32) MLMC_LAUNCH(K_BITS_EXTRACT, st, k_bits_extract<MLMC_F32><<<egrid, 256, 0, st>>>(a));
    else MLMC_LAUNCH(K_BITS_EXTRACT, st, k_bits_extract<MLMC_BF16><<<egrid, 256, 0, st>>>(a));
    return MLMC_OK;
}

mlmc_status agg_bits(const mlmc_plan_t* pl, const BitsArgs& b, const int32_t* level, const int32_t* scale_exp,
                     const uint64_t* planes, float alpha, float* out, hipStream_t st) {
    AggBitsArgs a;
    a.b = b;
    a.level = level;
    a.scale_exp = scale_exp;
    a.planes = planes;
    a.alpha = alpha;
    a.out = out;
    int64_t waves = b.nwords;
    int blocks = (int)((waves + 3) / 4);
    if (blocks > 8192) blocks = 8192;
    if (blocks < 1) blocks = 1;
    const int np = b.nplanes;   // 1 + F_0 + widest level field: bounds the planes of any row
    if (np <= 3) MLMC_LAUNCH(K_AGG_BITS, st, k_agg_bits<3><<<blocks, 256, 0, st>>>(a));
    else if (np <= 5) MLMC_LAUNCH(K_AGG_BITS, st, k_agg_bits<5><<<blocks, 256, 0, st>>>(a));
    else if (np <= 9) MLMC_LAUNCH(K_AGG_BITS, st, k_agg_bits<9><<<blocks, 256, 0, st>>>(a));
    else if (np <= 17) MLMC_LAUNCH(K_AGG_BITS, st, k_agg_bits<17><<<blocks, 256, 0, st>>>(a));
    else MLMC_LAUNCH(K_AGG_BITS, st, k_agg_bits<MAX_PLANES><<<blocks, 256, 0, st>>>(a));
    return MLMC_OK;
}

mlmc_status agg_sparse(const mlmc_plan_t* pl, const int64_t* row_off, const uint32_t* idx, const float* val, int64_t capacity,
                       const uint32_t* tile_off, uint32_t* tile_off_ws, float alpha, float* out, hipStream_t st) {
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
    if (!tile_off) {
        int64_t n = (int64_t)pl->M * (pl->ntiles + 1);
        int blocks = (int)((n + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        MLMC_LAUNCH(K_TILEOFF, st, k_tileoff<<<blocks, 256, 0, st>>>(a));
        a.tile_off = tile_off_ws;
    }
    MLMC_LAUNCH(K_AGG_SPARSE, st, k_agg_sparse<<<(unsigned)pl->ntiles, 256, 0, st>>>(a));
    return MLMC_OK;
}

}  // namespace mlmc
