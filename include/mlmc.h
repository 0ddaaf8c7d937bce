/*
 * mlmc.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of Multilevel Monte
 * Carlo (MLMC) gradient compression.
 *
 * Setting (paper, Sec. 2.1 "Problem Statement", Alg. 2, Alg. 3): M workers each hold a d-dimensional
 * stochastic gradient.  Per step every worker draws a level l ~ p, sends the MLMC estimate
 *     g~ = g^0 + (g^l - g^{l-1}) / p^l,   g^l = C^l(g)                          (Eq. (5), Eq. (6))
 * and the server forms (1/M) sum_i g~_i.  Here the M workers are the M rows of one device matrix.
 *
 * Conventions that hold for every entry point
 *   - "dev" pointers are device (HIP) memory owned by the caller; "host" pointers are host memory.  The
 *     library never allocates, frees or retains device memory; the plan is a host object.
 *   - All device work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     the call returns without synchronising.  The return value covers what the host can detect
 *     (MLMC_EINVAL for bad arguments, MLMC_EHIP for a failed launch).  Conditions only the device can see
 *     are OR-ed into *dev_status (MLMC_DEV_* bits), which the library clears at the start of the call.
 *   - `ws` is a dev scratch buffer of at least the `workspace_bytes` reported by mlmc_plan, 256-byte aligned.
 *     Calls that share a workspace must be ordered on one stream.
 *   - Row i of g is worker i: element j of row i is g[i * ld + j], ld >= d, dtype as planned.
 *   - Results are a pure function of (g, plan, p, seed, step): no atomics on floating point, no
 *     dependence on scheduling.
 *
 * Orders and roundings (fixed so that an independent implementation can reproduce every bit)
 *   - Magnitude order: key_j = bit pattern of |g_j| as fp32 (bf16 inputs are widened exactly);
 *     rank(j) = #{i : key_i > key_j} + #{i < j : key_i == key_j}.  Top-k keeps rank < k.
 *   - Band l (l = 1..L) = {j : k_{l-1} <= rank(j) < k_l}; base band = {j : rank(j) < k_0}.
 *   - Delta_l = sqrt(S_l), S_l = exact sum of g_j^2 over band l rounded once to fp64 (Lemma 3.4).
 *   - Adaptive p_l = Delta_l / (Delta_1 + ... + Delta_L) (fp64, sum in level order); all-zero -> 1/L.
 *   - Draw: T_l = floor((p_1 + ... + p_l) * 2^32) (running fp64 sum), T_L = 2^32;
 *     x = word 0 of Philox4x32-10 with key = (seed_lo, seed_hi), counter = (step_lo, step_hi, i, 0);
 *     level = min{l : x < T_l}.
 *   - Weight w = (float)(1.0 / p_level) (0 if p_level == 0); band values are the fp32 product g_j * w.
 */
#ifndef MLMC_H
#define MLMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mlmc_plan_s mlmc_plan_t; /* opaque, host side, owned by the library */

typedef enum {
    MLMC_OK = 0,
    MLMC_EINVAL = 1,   /* bad argument (ladder, probabilities, sizes, null pointers, alignment) */
    MLMC_ENOMEM = 2,   /* host allocation failed */
    MLMC_EHIP = 3,     /* a HIP call or kernel launch failed */
    MLMC_ELIMIT = 4    /* mlmc_compress_bits_static: the plan needs more scratch than MLMC_STATIC_SCRATCH_BYTES */
} mlmc_status;

/* bits OR-ed into *dev_status by the kernels */
#define MLMC_DEV_CAPACITY 1  /* row_off[M] > capacity: entries past capacity were not written */
#define MLMC_DEV_NONFINITE 2 /* an Inf or NaN input was seen (it is ordered by its bit pattern) */
#define MLMC_DEV_INTERNAL 4  /* an internal consistency check failed (counts do not add up) */
#define MLMC_DEV_REDONE 8    /* not an error: a row's sampled threshold search was refuted and the row was redone exactly */

typedef enum { MLMC_F32 = 0, MLMC_BF16 = 1 } mlmc_dtype;
typedef enum { MLMC_TOPK = 0, MLMC_BITS = 1, MLMC_FBITS = 2, MLMC_STOPK = 3, MLMC_VBITS = 4, MLMC_RTN = 5 } mlmc_kind;

#define MLMC_MAX_LEVELS 32   /* L <= 32 */
#define MLMC_MAX_WORKERS 1024 /* M <= 1024 */
#define MLMC_MAX_SLEVELS 65536 /* MLMC_STOPK: L = ceil(d / s) <= 65536 */
#define MLMC_MAX_RTN_LEVELS 8  /* MLMC_RTN: L <= 8 */
#define MLMC_TILE 4096       /* elements per tile of the per-row offset table */

/*
 * Plan: the inputs of Alg. 2 / Alg. 3 other than the gradients (multilevel compressor C^l, level
 * probabilities) for M workers of dimension d (Sec. 2.1).
 *   kind == MLMC_TOPK: ladder = ranks k_0..k_L, 0 <= k_0 < k_1 < ... < k_L <= d        (Sec. 3.2)
 *   kind == MLMC_BITS: ladder = kept fraction bits F_0..F_L, 0 <= F_0 < ... < F_L <= 24 (Sec. 3.1)
 *   kind == MLMC_VBITS: the same ladder of fraction bits, with the entries divided by the largest entry of the row itself
 *            as Sec. 3.1 writes it (MLMC_BITS divides by the power of two above it): digits m_j = min(floor(|g_j| /
 *            max|g| * 2^F_L), 2^F_L - 1) - the cap is for the entries of the largest magnitude, whose quotient 1 has no
 *            binary expansion below 1; C^F keeps the first F of them.  The row maximum is read exactly before the
 *            extraction (two reads of the input); mlmc_plan_set_sampling does not apply.
 *   kind == MLMC_FBITS: ladder = kept mantissa digits F_0..F_L, 0 <= F_0 < ... < F_L <= 23 (App. B: the
 *            floating-point compressor C^F keeps sign, exponent and the first F mantissa digits of every entry;
 *            the paper's ladder is F = 0, 1, ..., 52 for fp64, here 0..23 for fp32 inputs)
 *   kind == MLMC_RTN: Round-to-Nearest ladder (Sec. 3.3, App. G.2): ladder = bit widths b_0..b_L, 0 <= b_0 < ... < b_L <= 16,
 *            L <= MLMC_MAX_RTN_LEVELS.  C^b(v)_j = n_j * 2c / (2^b - 1) with c = max_j |v_j| (sent with the message) and
 *            the code n_j = the exact quotient v_j (2^b - 1) / (2c) rounded to the nearest integer, ties to even,
 *            kept within |n_j| <= 2^(b-1) - 1 (a symmetric b-bit code); b = 0 is the zero vector.  A message holds the
 *            codes of the levels involved: b_0 + b_{l-1} + b_l planes at most 32.  p_fixed may be NULL: Lemma 3.4's
 *            probabilities from every row's residual norms (Alg. 3).
 *   kind == MLMC_STOPK: s-segmented Top-k (Sec. 2.2, Sec. 3.2): ladder = {s} (one entry, the segment length, s >= 1);
 *            the row sorted by magnitude is cut into segments of s entries, C^l keeps the first l of them, so
 *            k_l = min(s l, d), g^0 = 0, and L must be ceil(d / s) <= MLMC_MAX_SLEVELS.  p_fixed must be NULL: the
 *            probabilities are Lemma 3.4's, over all L levels, from every row itself (Alg. 3).  The message of a
 *            row is its drawn segment (s entries; the last segment may be shorter).
 *   p_fixed: host, L entries for levels 1..L, each > 0, summing to 1 within 1e-9; NULL selects the
 *            adaptive probabilities of Lemma 3.4 (MLMC_TOPK only).  Lemma 3.3 / Lemma B.1: 2^-l / (1 - 2^-L).
 *   1 <= M <= MLMC_MAX_WORKERS, 1 <= d < 2^31, 1 <= L <= MLMC_MAX_LEVELS.
 * Outputs (host): *plan; *workspace_bytes; *sparse_capacity_worst = M * (k_0 + widest band) entries
 * (0 for the bit-wise kinds; M * s for MLMC_STOPK).  Returns MLMC_EINVAL and leaves *plan NULL on a bad argument.
 */
mlmc_status mlmc_plan(mlmc_plan_t **plan, int kind, int M, int64_t d, int in_dtype, int L,
                      const int64_t *ladder, const double *p_fixed, size_t *workspace_bytes,
                      int64_t *sparse_capacity_worst);
void mlmc_plan_destroy(mlmc_plan_t *plan);

/*
 * Tuning hook.  MLMC_TOPK plans: the rank thresholds of Top-k (Sec. 2.2, Sec. 3.2) are first located from a
 * histogram of one 1024-element block out of 2^shift of every row, then proven or refuted by exact counts
 * taken during the full read; a refuted row is redone from an exact histogram.  MLMC_BITS plans: the row scale
 * (Sec. 3.1) is first taken from the largest entry of the same sample of blocks, the full read extracts the
 * message under that scale and finds the true maximum; a row whose true maximum needs a larger scale is
 * extracted again.  So `shift` changes run time only, never a result.  mlmc_plan picks the shift from d
 * (0 for short rows = exact at once).  0 <= shift <= 12; MLMC_EINVAL otherwise.
 */
mlmc_status mlmc_plan_set_sampling(mlmc_plan_t *plan, int shift);

/*
 * Tuning hook (MLMC_TOPK plans).  With staging on (the default) the read that selects the thresholds also sets
 * aside the members of the band the message will hold (Eq. (6)): the level is known before the read when p is
 * given, and predicted from the sampled histogram when p is adaptive (Alg. 3); the message is then assembled
 * from what was set aside and the rows are read once.  A wrong prediction, a drawn band wider than an eighth of
 * the row (cheaper to collect by reading again), or staging switched off, makes the library read the row a
 * second time.  Run time only, never a result.
 */
mlmc_status mlmc_plan_set_staging(mlmc_plan_t *plan, int enable);

/*
 * Tuning hook (MLMC_TOPK plans).  The message of Eq. (6) is written by two kernels that serve disjoint rows: one
 * assembles it from what the selection read set aside, the other reads a row again.  With overlap on (the default for
 * plans of 8 rows or more and 2^28 elements or more; the fork and the join cost more than they gain on smaller ones) the
 * second runs on a stream the plan owns (default priority, created at the first call, destroyed with the plan), forked
 * from and joined to `hip_stream` with events, so the caller's stream stays in order.
 * Off: both run on `hip_stream`.  Run time only, never a result.
 */
mlmc_status mlmc_plan_set_overlap(mlmc_plan_t *plan, int enable);

/* MLMC_TOPK plans: elements of a row that one workgroup of the selection read takes (a multiple of MLMC_TILE, at most
 * 2^18); 0 for other plans.  For tests and tuning: results never depend on it. */
int64_t mlmc_plan_chunk(const mlmc_plan_t *plan);
/* Tiles per row of the offset table: ceil(d / MLMC_TILE). */
int64_t mlmc_plan_num_tiles(const mlmc_plan_t *plan);
/* Planes per row of the packed message: MLMC_BITS and MLMC_VBITS 1 + F_0 + max_l (F_l - F_{l-1}); MLMC_FBITS 9 + F_0 + max_l (F_l - F_{l-1});
 * MLMC_RTN b_0 + max_l ((l > 1 ? b_{l-1} : 0) + b_l); else 0. */
int mlmc_plan_num_planes(const mlmc_plan_t *plan);

/* Lemma 3.3 form: p[l-1] = 2^-l / (1 - 2^-L), l = 1..L (host array of L doubles). */
mlmc_status mlmc_geometric_p(int L, double *p);

const char *mlmc_status_string(int status);

/*
 * Per-level residual norms Delta_l = ||C_l(g) - C_{l-1}(g)||_2, l = 1..L, of every row (Lemma 3.4; for
 * rank bands Delta_l^2 is the sum of squares over band l, App. D).  MLMC_TOPK and MLMC_STOPK plans.
 *   g: dev [M][ld];  norms: dev [M][L] fp64 (out);  dev_status: dev [1] int32 (out).
 */
mlmc_status mlmc_level_norms(const mlmc_plan_t *plan, const void *g, int64_t ld, double *norms,
                             int32_t *dev_status, void *ws, void *hip_stream);

/*
 * Worker side of Alg. 2 (fixed p) / Alg. 3 (adaptive p) for the Top-k ladder: draw the level, emit
 * C_0(g) + (C_l(g) - C_{l-1}(g)) / p_l as an index-sorted sparse band.
 *   p: NULL -> the plan's p_fixed, or (adaptive plan) Lemma 3.4 probabilities computed here from g;
 *      else dev [M][L] fp64: probabilities (p_is_norms == 0) or norms to be normalised (p_is_norms != 0).
 *   seed, step: the draw of worker i depends on (seed, step, i) only.
 *   level:   dev [M] int32 (out), drawn level in 1..L.
 *   row_off: dev [M+1] int64 (out), exclusive prefix of nnz_i = k_0 + k_l - k_{l-1}.
 *   idx/val: dev [capacity] uint32 / float (out); row i occupies [row_off[i], row_off[i+1]), ascending idx.
 *            Base-band entries carry g_j, drawn-band entries carry fp32(g_j * w_i).
 *   tile_off: dev [M][num_tiles + 1] uint32 (out) or NULL; tile_off[i][t] = number of entries of row i
 *            with idx < t * MLMC_TILE (so tile_off[i][num_tiles] = nnz_i).  Lets mlmc_aggregate skip a search.
 *   norms_out: dev [M][L] fp64 (out) or NULL; written only when p == NULL on an adaptive plan.
 * MLMC_STOPK plans: p must be NULL and p_is_norms 0; every other argument as above (level in 1..ceil(d / s)).
 */
mlmc_status mlmc_compress_topk(const mlmc_plan_t *plan, const void *g, int64_t ld, const double *p,
                               int p_is_norms, uint64_t seed, uint64_t step, int32_t *level,
                               int64_t *row_off, uint32_t *idx, float *val, int64_t capacity,
                               uint32_t *tile_off, double *norms_out, int32_t *dev_status, void *ws,
                               void *hip_stream);

/*
 * Worker side of Alg. 2 for the fixed-point bit-wise ladder (Sec. 3.1).  Per row: scale s = 2^e with
 * e = max(E_max, 1) - 126 (E_max = largest fp32 exponent field in the row, so |g_j| / s < 1),
 * m_j = floor(|g_j| / s * 2^{F_L}); drawn level l; message = sign plane, F_0 base-field planes
 * (bits of m_j >> (F_L - F_0), LSB first), F_l - F_{l-1} level-field planes (bits of
 * (m_j >> (F_L - F_l)) mod 2^{F_l - F_{l-1}}, LSB first).
 *   level: dev [M] int32 (out);  scale_exp: dev [M] int32 (out), the exponent e.
 *   planes: dev [M][num_planes][ceil(d/64)] uint64 (out); word w bit b <-> element 64 w + b, pad bits 0;
 *           planes beyond 1 + F_0 + (F_l - F_{l-1}) of a row are left untouched.
 *
 * MLMC_VBITS plans: the same message with the digits of |g_j| / max|g| (see mlmc_plan); scale_exp[i] receives the bit
 * pattern of the fp32 number max_j |g_ij| (the largest entry, "transmitted" with the message, Sec. 3.1) instead of an
 * exponent.  Decoded value: sign_j * [ fp32(f0_j) * fp32(v 2^-F_0) + fp32(f_j) * fp32(v 2^-F_l / p_l) ], v that number.
 *
 * MLMC_FBITS plans (App. B, floating-point ladder): no scale; C^{F_0}(g) + (C^{F_l}(g) - C^{F_{l-1}}(g)) / p_l with
 * C^F = mantissa truncated to F digits.  Message per row: sign plane, 8 planes of the exponent field (LSB first),
 * F_0 planes of the first F_0 mantissa digits read as a number (LSB first), F_l - F_{l-1} planes of the digits
 * F_{l-1}+1 .. F_l read as a number (LSB first).  scale_exp may be NULL (it is not written).  bf16 inputs are widened.
 */
mlmc_status mlmc_compress_bits(const mlmc_plan_t *plan, const void *g, int64_t ld, uint64_t seed,
                               uint64_t step, int32_t *level, int32_t *scale_exp, uint64_t *planes,
                               int32_t *dev_status, void *ws, void *hip_stream);

/*
 * Worker side of Alg. 2 / Alg. 3 for the Round-to-Nearest ladder (MLMC_RTN plans; Sec. 3.3, App. G.2).  The residual of
 * level l is C^{b_l}(v) - C^{b_{l-1}}(v) = (2c / (D D')) k with the integers k_j = n_{b_l} D' - n_{b_{l-1}} D,
 * D = 2^{b_l} - 1, D' = 2^{b_{l-1}} - 1 (D' = 1, n = 0 for b_{l-1} = 0); Delta_l = (2c / (D D')) sqrt(sum_j k_j^2) with
 * the integer sum exact and rounded once to fp64 (Lemma 3.4).  Three reads of the input: largest entry, norms, codes
 * (two when the plan has its own probabilities and norms_out is NULL: the norms are then not computed).
 *   level: dev [M] int32 (out);  scale: dev [M][2] int32 (out): the bit patterns of c and of the coefficient
 *   fp32((2c / (D D')) / p_l) that the server multiplies k with;  planes: dev [M][num_planes][ceil(d/64)] uint64 (out):
 *   per row the planes of the codes n_{b_0} (b_0 of them, if b_0 > 0), n_{b_{l-1}} (if l > 1) and n_{b_l}, each code
 *   in two's complement cut to its width, least significant plane first; word w bit k <-> element 64 w + k; pad bits
 *   zero; planes past those are not written.  norms_out: dev [M][L] fp64 or NULL.
 *   Decoded value (mlmc_aggregate): fp32(n_{b_0}) * fp32(2c / D_0) + fp32(k_j) * coefficient, single fp32 operations.
 */
mlmc_status mlmc_compress_rtn(const mlmc_plan_t *plan, const void *g, int64_t ld, uint64_t seed, uint64_t step,
                              int32_t *level, int32_t *scale, uint64_t *planes, double *norms_out,
                              int32_t *dev_status, void *ws, void *hip_stream);

/*
 * mlmc_compress_bits for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * mlmc_compress_bits, without `ws`: the scratch (per-row maxima and draw records) lives in a device array of
 * MLMC_STATIC_SCRATCH_BYTES bytes inside the library, one copy per GPU, held until the process ends.  The call
 * allocates nothing and frees nothing.  Its first call on a device looks the array's address up
 * (hipGetSymbolAddress); make that call outside a graph capture.
 *   Limit: the plan's workspace_bytes must not exceed MLMC_STATIC_SCRATCH_BYTES (M up to about 80 workers),
 *   else MLMC_ELIMIT and nothing is enqueued.
 *   All calls on one GPU share the array, on any stream and for any plan: calls that overlap on a GPU race.
 *   Order them on one stream, or with events.  The array keeps the previous call's contents; the part that must
 *   start at zero is cleared on the stream at the start of every call.
 */
#define MLMC_STATIC_SCRATCH_BYTES (1 << 20)
mlmc_status mlmc_compress_bits_static(const mlmc_plan_t *plan, const void *g, int64_t ld, uint64_t seed,
                                      uint64_t step, int32_t *level, int32_t *scale_exp, uint64_t *planes,
                                      int32_t *dev_status, void *hip_stream);

/*
 * Server side (Alg. 2 / Alg. 3 "Server aggregates"): out[j] = fp32(alpha * acc_j), acc_j the fp32 sum over
 * workers in worker order (alpha = 1/M gives the paper's mean).
 *   MLMC_TOPK / MLMC_STOPK plan: row_off, idx, val as written by mlmc_compress_topk (level unused, may be NULL);
 *     capacity = entries that idx / val hold (as passed to mlmc_compress_topk): entries at positions >= capacity
 *     are never read, so a message that did not fit (MLMC_DEV_CAPACITY) cannot steer reads out of bounds;
 *     tile_off as written there, or NULL (then it is rebuilt by binary search into ws).  A worker without an
 *     entry at j is skipped.
 *   MLMC_BITS plan: level, scale_exp, planes as written by mlmc_compress_bits; the decoded value of
 *     worker i at j is sign * [ fp32(f0) * fp32(2^(e - F_0)) + fp32(f) * fp32(2^(e - F_l) / p_l) ].
 *   MLMC_RTN plan: level, scale_exp = the [M][2] `scale` of mlmc_compress_rtn, planes; decoded as stated there.
 *   MLMC_FBITS plan: level, planes (scale_exp unused, may be NULL); with sign s, exponent field E, base digits f0 and
 *     level digits f of worker i at j: base = float(s, E, f0 << (23 - F_0)), residual = float(s, E, f << (23 - F_l)) -
 *     float(s, E, 0) (exact), decoded value = fp32(base + fp32(residual * fp32(1 / p_l))).
 *   out: dev [d] fp32, fully overwritten.
 */
mlmc_status mlmc_aggregate(const mlmc_plan_t *plan, const int32_t *level, const int64_t *row_off,
                           const uint32_t *idx, const float *val, int64_t capacity, const uint32_t *tile_off,
                           const int32_t *scale_exp, const uint64_t *planes, float alpha, float *out,
                           void *ws, void *hip_stream);

/*
 * Server side with the model update fused in (Alg. 2 / Alg. 3 "Server aggregates" and "Server updates"):
 * g~_j = fp32(alpha * acc_j) as in mlmc_aggregate, then x_j <- fp32(x_j - fp32(eta * g~_j)) (one multiply, one subtract),
 * inside the same pass over the dense tiles, so that the update is not written and read again.
 *   x:   dev [d] fp32, in and out (the model x_t -> x_{t+1}).
 *   out: dev [d] fp32 (out) or NULL when g~ itself is not wanted; must not alias x.
 *   Every other argument as in mlmc_aggregate.
 */
mlmc_status mlmc_aggregate_update(const mlmc_plan_t *plan, const int32_t *level, const int64_t *row_off,
                                  const uint32_t *idx, const float *val, int64_t capacity,
                                  const uint32_t *tile_off, const int32_t *scale_exp, const uint64_t *planes,
                                  float alpha, float eta, float *x, float *out, void *ws, void *hip_stream);

/*
 * Bits every worker's message of this step takes on the wire (the "communicated bits" of Sec. 5), from the drawn levels:
 *   MLMC_TOPK, MLMC_STOPK: nnz_i * (32 + ceil(log2 d)) + ceil(log2 L): every entry of the base band and of the drawn band as a
 *     32-bit value and an index into d, plus the level (Sec. 3: the residual of Top-k is one rank band).
 *   MLMC_BITS: d * (1 + F_0 + F_l - F_{l-1}) + 32 + ceil(log2 L): per entry the sign, the base bits and the level
 *     field, plus the scale exponent and the level (Sec. 3.1; with F = 0..63 and a 64-bit scale: 2 d + 64 + 6).
 *   MLMC_FBITS: d * (9 + F_0 + F_l - F_{l-1}) + ceil(log2 L): per entry sign, 8 exponent bits, base and level digits
 *     (App. B; for fp64 with one digit per level: 13 d + log2 52).
 *   level: dev [M] int32 as written by a compress call;  bits: dev [M] uint64 (out).
 */
mlmc_status mlmc_message_bits(const mlmc_plan_t *plan, const int32_t *level, uint64_t *bits, void *hip_stream);

/*
 * Per-kernel timing for benchmarks (measurement aid, not part of the method).  While enabled, every kernel
 * the library launches is bracketed by a pair of HIP events on the launch stream; mlmc_profile_get waits
 * for the recorded events and returns the accumulated device time and launch count of kernel `id`
 * (0 <= id < mlmc_profile_num_kernels()).  Host side, process wide, not thread safe; off by default.
 */
void mlmc_profile_enable(int on);
void mlmc_profile_reset(void);
int mlmc_profile_num_kernels(void);
const char *mlmc_profile_kernel_name(int id);
mlmc_status mlmc_profile_get(int id, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* MLMC_H */
