"""Plain CPU definition of MLMC gradient compression (Top-k ladder, fixed-point bit-wise ladder) and
of the server aggregate.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py): slow, written for checking by eye against the paper,
never tuned, never used by the product path.

What is computed, with the passages it follows:

* Top-k compressor C_l = Top-k_l (Sec. 2.2 "Top-k"; Sec. 3.2): keep the k_l entries of largest
  magnitude.  The order that decides "largest" is total: magnitude descending, ties (equal |g|,
  including +0/-0) broken by the lower index.  It is realised by one full stable sort.
* MLMC estimate (Eq. (5), Eq. (6), Alg. 2 worker steps): g~ = g^0 + (g^l - g^{l-1}) / p^l with l ~ p.
  For a rank ladder k_0 < k_1 < ... < k_L the residual g^l - g^{l-1} is the band of entries with rank
  in [k_{l-1}, k_l) (Sec. 3, remark after Alg. 2), and g^0 = C_0(g) is the band [0, k_0) (the paper's own
  choice is k_0 = 0, i.e. g^0 = 0).
* Adaptive probabilities (Lemma 3.4, Alg. 3): p^l = Delta^l / sum_l' Delta^l', Delta^l = ||g^l - g^{l-1}||_2.
* Fixed probabilities of the geometric form of Lemma 3.3: p^l = 2^-l / (1 - 2^-L), l = 1..L.
* Fixed-point bit-wise compressor (Sec. 2.2 "Fixed-point compressors", Sec. 3.1): entries are normalised
  to magnitude < 1, written as sign + binary fraction, and C^F keeps the F most significant fraction bits.
* The same ladder with the entries divided by the largest entry itself, as Sec. 3.1 writes it (`vmax_digits` and the
  `*_vbits*` functions): the digits of |g_j| / max|g|, capped at 2^Q - 1 for the entries of the largest magnitude.
* Round-to-Nearest ladder (Sec. 3.3, App. G.2; the `rtn_*` functions): codes by exact rounding of v (2^b - 1) / (2c),
  residual norms of Lemma 3.4 from exact integer sums, the message as the planes of the codes involved.
* Server aggregate (Alg. 2 / Alg. 3 "Server aggregates"): out = alpha * sum_i g~_i, alpha = 1/M for the mean.

Readings where the paper is silent (each is also what the HIP library documents):

* Norms: S_l = sum_{j in band l} g_j^2 is the exact real-number sum rounded once to fp64
  (round-to-nearest-even); Delta^l = IEEE sqrt(S_l).  Exact sums do not depend on summation order.
* Level draw: integer CDF thresholds T_l = floor(c_l * 2^32), c_l = p_1 + ... + p_l accumulated in fp64 in
  level order, T_L = 2^32; x = one Philox4x32-10 word per (seed, step, worker); l = min{l : x < T_l}.
* Weight: w = fp32(1.0 / p_l) (fp64 divide, then round to fp32); entry value = fp32(g_j * w), one multiply.
  If p_l = 0 (reachable only through CDF rounding; the band is then the zero vector) w = 0.
* All-zero residuals (sum of Delta = 0): uniform p_l = 1/L.
* Bit-wise scale: power of two s = 2^e strictly above the row maximum, e = max(E_max, 1) - 126 with E_max the
  largest biased exponent field in the row, so |g_j| / s < 1 and the fraction bits are exact.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .philox import level_uniform

TWO32 = 4294967296.0


def _ceil_log2(n: int) -> int:
    """Bits that name one of n alternatives: ceil(log2 n), 0 for n <= 1."""
    return max(int(n) - 1, 0).bit_length()


# ----------------------------------------------------------------------------------------------
# inputs
# ----------------------------------------------------------------------------------------------
def as_f32(row: np.ndarray) -> np.ndarray:
    """A row as float32 values.  uint16 rows are bf16 bit patterns (exact upcast)."""
    row = np.asarray(row)
    if row.dtype == np.uint16:
        return (row.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if row.dtype != np.float32:
        raise TypeError("rows are float32 or uint16 (bf16 bits)")
    return row


def magnitude_keys(g32: np.ndarray) -> np.ndarray:
    """|g| as an unsigned integer that orders like the magnitude: the fp32 bit pattern, sign cleared."""
    return np.ascontiguousarray(g32).view(np.uint32) & np.uint32(0x7FFFFFFF)


def magnitude_order(g32: np.ndarray) -> np.ndarray:
    """Indices sorted by magnitude descending, equal magnitudes by index ascending (one stable sort)."""
    inv = np.uint32(0x7FFFFFFF) - magnitude_keys(g32)
    return np.argsort(inv, kind="stable")


# ----------------------------------------------------------------------------------------------
# level probabilities and the draw
# ----------------------------------------------------------------------------------------------
def geometric_p(L: int) -> List[float]:
    """Lemma 3.3 form: p^l = 2^-l / (1 - 2^-L), l = 1..L (fp64)."""
    return [math.ldexp(1.0, -l) / (1.0 - math.ldexp(1.0, -L)) for l in range(1, L + 1)]


def adaptive_p(norms: Sequence[float]) -> List[float]:
    """Lemma 3.4: p^l = Delta^l / sum Delta (sum in level order, fp64); uniform if every Delta is 0."""
    total = 0.0
    for x in norms:
        total = total + float(x)
    L = len(norms)
    if total == 0.0:
        return [1.0 / L] * L
    return [float(x) / total for x in norms]


def cdf_thresholds(p: Sequence[float]) -> List[int]:
    L = len(p)
    out, c = [], 0.0
    for l in range(L):
        c = c + float(p[l])
        t = int(math.floor(c * TWO32))
        out.append(min(max(t, 0), 1 << 32))
    out[L - 1] = 1 << 32
    return out


def draw_level(p: Sequence[float], seed: int, step: int, worker: int) -> int:
    """l in 1..L with probability p^l: inverse CDF of one 32-bit uniform (Alg. 2 "Sample l ~ p^l")."""
    x = level_uniform(seed, step, worker)
    for l, t in enumerate(cdf_thresholds(p), start=1):
        if x < t:
            return l
    raise AssertionError("unreachable: T_L = 2^32")


def level_weight(p_l: float) -> np.float32:
    if p_l == 0.0:
        return np.float32(0.0)
    return np.float32(1.0 / float(p_l))


# ----------------------------------------------------------------------------------------------
# exact sums of squares
# ----------------------------------------------------------------------------------------------
SUMSQ_UNIT_LOG2 = -298  # squares are integer multiples of 2^-298 (smallest fp32 denormal squared)


def exact_sumsq(g32: np.ndarray) -> int:
    """sum_j g_j^2 as an exact integer count of 2^-298 units.

    An fp32 magnitude is sig * 2^(E' - 150) with sig the 24-bit significand (no hidden bit for
    denormals) and E' = max(E, 1), so g^2 = sig^2 * 2^(2(E' - 1)) units.  Entries are grouped by E' and the
    integer squares (< 2^48) are summed in two 32-bit halves so that uint64 sums cannot overflow.
    """
    keys = magnitude_keys(g32)
    if keys.size == 0:
        return 0
    E = (keys >> np.uint32(23)).astype(np.int64)
    frac = (keys & np.uint32(0x7FFFFF)).astype(np.uint64)
    sig = np.where(E > 0, frac | np.uint64(0x800000), frac)
    Ep = np.maximum(E, 1)
    sq = sig * sig
    total = 0
    for e in np.unique(Ep):
        sel = sq[Ep == e]
        lo = int(np.sum(sel & np.uint64(0xFFFFFFFF), dtype=np.uint64))
        hi = int(np.sum(sel >> np.uint64(32), dtype=np.uint64))
        total += ((hi << 32) + lo) << (2 * (int(e) - 1))
    return total


def units_to_f64(n_units: int) -> float:
    """Exact integer count of 2^-298 units -> nearest fp64 (Python's int/int division is correctly rounded)."""
    return n_units / (1 << 298)


def level_norms_row(row: np.ndarray, ladder: Sequence[int]) -> Tuple[List[float], List[int]]:
    """Delta^l = ||C_l(g) - C_{l-1}(g)||_2 for l = 1..L (Lemma 3.4), and the exact band sums S_0..S_L in units."""
    g = as_f32(row)
    order = magnitude_order(g)
    L = len(ladder) - 1
    units = [exact_sumsq(g[order[:ladder[0]]])]
    for l in range(1, L + 1):
        units.append(exact_sumsq(g[order[ladder[l - 1]:ladder[l]]]))
    norms = [math.sqrt(units_to_f64(u)) for u in units[1:]]
    return norms, units


# ----------------------------------------------------------------------------------------------
# Top-k MLMC
# ----------------------------------------------------------------------------------------------
def topk_dense(row: np.ndarray, k: int) -> np.ndarray:
    """C(g) = Top-k(g) as a dense vector (Sec. 2.2)."""
    g = as_f32(row)
    out = np.zeros_like(g)
    keep = magnitude_order(g)[:k]
    out[keep] = g[keep]
    return out


def compress_topk_row(row: np.ndarray, ladder: Sequence[int], p: Optional[Sequence[float]],
                      seed: int, step: int, worker: int, force_level: Optional[int] = None):
    """One worker's MLMC Top-k message (Alg. 2 / Alg. 3 worker steps).

    p = None selects the adaptive probabilities of Lemma 3.4 computed from this row.
    Returns dict(level, weight, idx uint32 ascending, val float32, norms list[L], p list[L]).
    """
    g = as_f32(row)
    d = g.size
    L = len(ladder) - 1
    assert 0 <= ladder[0] and all(ladder[i] < ladder[i + 1] for i in range(L)) and ladder[L] <= d
    order = magnitude_order(g)
    norms = None
    if p is None:
        norms, _ = level_norms_row(row, ladder)
        p = adaptive_p(norms)
    p = [float(x) for x in p]
    level = draw_level(p, seed, step, worker) if force_level is None else int(force_level)
    w = level_weight(p[level - 1])
    base = order[:ladder[0]]
    band = order[ladder[level - 1]:ladder[level]]
    in_band = np.zeros(d, dtype=bool)
    in_band[band] = True
    idx = np.sort(np.concatenate([base, band])).astype(np.uint32)
    val = g[idx].copy()
    sel = in_band[idx]
    val[sel] = val[sel] * w          # one fp32 multiply per band entry
    return dict(level=level, weight=w, idx=idx, val=val.astype(np.float32), norms=norms, p=p)


def stopk_ladder(d: int, s: int) -> List[int]:
    """The ladder of s-segmented Top-k (Sec. 2.2): the vector sorted by magnitude is cut into segments of length s
    (the last one may be shorter); C^l keeps the first l segments, so k_l = min(s l, d), l = 0..ceil(d / s), and the
    residual g^l - g^{l-1} is the l-th segment (Sec. 3.2)."""
    L = -(-d // s)
    return [min(s * l, d) for l in range(L + 1)]


def compress_topk(G: np.ndarray, ladder, p, seed: int, step: int, norms_override=None):
    """All M rows.  Row i is worker i.  p: list[L] shared by all rows, or None (adaptive).
    norms_override[i] (optional) replaces the oracle's own Delta for row i in the adaptive case."""
    msgs = []
    for i in range(G.shape[0]):
        pi = p
        if p is None and norms_override is not None:
            pi = adaptive_p(norms_override[i])
        msgs.append(compress_topk_row(G[i], ladder, pi, seed, step, i))
    return msgs


def sparse_to_dense(idx: np.ndarray, val: np.ndarray, d: int) -> np.ndarray:
    out = np.zeros(d, dtype=np.float32)
    out[idx] = val
    return out


# ----------------------------------------------------------------------------------------------
# fixed-point bit-wise MLMC
# ----------------------------------------------------------------------------------------------
def bits_scale_exponent(g32: np.ndarray) -> int:
    """e with s = 2^e > max|g| and |g|/s < 1: e = max(E_max, 1) - 126 (E_max = largest exponent field)."""
    keys = magnitude_keys(g32)
    Emax = int(keys.max() >> np.uint32(23)) if keys.size else 0
    return max(Emax, 1) - 126


def fixed_point_digits(g32: np.ndarray, e: int, Q: int) -> np.ndarray:
    """m_j = floor(|g_j| / 2^e * 2^Q): the first Q fraction bits of the normalised magnitude (Sec. 3.1)."""
    a = np.abs(g32.astype(np.float64))
    return np.floor(np.ldexp(a, Q - e)).astype(np.uint64)


def bits_truncate_dense(row: np.ndarray, F: int, Q: int) -> np.ndarray:
    """C^F(g): keep the F most significant fraction bits (out of the Q considered), as float64 values."""
    g = as_f32(row)
    e = bits_scale_exponent(g)
    m = fixed_point_digits(g, e, Q)
    kept = (m >> np.uint64(Q - F)).astype(np.float64)
    return np.where(np.signbit(g), -1.0, 1.0) * np.ldexp(kept, e - F)


def pack_plane(bits: np.ndarray) -> np.ndarray:
    """bool[d] -> uint64[ceil(d/64)], word w bit b <-> element 64 w + b, pad bits zero."""
    d = bits.size
    nw = (d + 63) // 64
    padded = np.zeros(nw * 64, dtype=np.uint8)
    padded[:d] = bits
    return np.packbits(padded, bitorder="little").view("<u8").astype(np.uint64)


def unpack_plane(words: np.ndarray, d: int) -> np.ndarray:
    return np.unpackbits(words.astype("<u8").view(np.uint8), bitorder="little")[:d].astype(bool)


def compress_bits_row(row: np.ndarray, F: Sequence[int], p: Sequence[float], seed: int, step: int,
                      worker: int, force_level: Optional[int] = None):
    """One worker's fixed-point MLMC message: level, scale exponent, sign plane, base-field planes
    (F_0 of them, LSB first), level-field planes (F_l - F_{l-1} of them, LSB first)."""
    g = as_f32(row)
    L = len(F) - 1
    Q = F[L]
    assert 0 <= F[0] and all(F[i] < F[i + 1] for i in range(L)) and Q <= 24
    e = bits_scale_exponent(g)
    m = fixed_point_digits(g, e, Q)
    level = draw_level(p, seed, step, worker) if force_level is None else int(force_level)
    width = F[level] - F[level - 1]
    field = (m >> np.uint64(Q - F[level])) & np.uint64((1 << width) - 1)
    base = (m >> np.uint64(Q - F[0])) if F[0] > 0 else np.zeros_like(m)
    planes = [pack_plane(np.signbit(g))]
    for b in range(F[0]):
        planes.append(pack_plane(((base >> np.uint64(b)) & np.uint64(1)).astype(bool)))
    for b in range(width):
        planes.append(pack_plane(((field >> np.uint64(b)) & np.uint64(1)).astype(bool)))
    return dict(level=level, scale_exp=e, planes=np.stack(planes), p_level=float(p[level - 1]))


def decode_bits_row(msg, F: Sequence[int], d: int) -> np.ndarray:
    """The fp32 vector g~ the server adds for this worker:
    g~_j = sign_j * [ fp32(f0_j) * c_0 + fp32(f_j) * c_l ], c_0 = fp32(2^(e - F_0)),
    c_l = fp32(2^(e - F_l) / p_l); products and the sum are single fp32 operations."""
    level, e, planes = msg["level"], msg["scale_exp"], msg["planes"]
    width = F[level] - F[level - 1]
    sign = unpack_plane(planes[0], d)
    f0 = np.zeros(d, dtype=np.uint32)
    for b in range(F[0]):
        f0 |= unpack_plane(planes[1 + b], d).astype(np.uint32) << np.uint32(b)
    f = np.zeros(d, dtype=np.uint32)
    for b in range(width):
        f |= unpack_plane(planes[1 + F[0] + b], d).astype(np.uint32) << np.uint32(b)
    p_l = msg["p_level"]
    c_l = np.float32(math.ldexp(1.0, e - F[level]) / p_l) if p_l != 0.0 else np.float32(0.0)
    v = f.astype(np.float32) * c_l
    if F[0] > 0:
        c_0 = np.float32(math.ldexp(1.0, e - F[0]))
        v = f0.astype(np.float32) * c_0 + v
    return np.where(sign, -v, v).astype(np.float32)


def compress_bits(G: np.ndarray, F, p, seed: int, step: int):
    return [compress_bits_row(G[i], F, p, seed, step, i) for i in range(G.shape[0])]


# ----------------------------------------------------------------------------------------------
# fixed-point bit-wise MLMC, entries divided by the largest entry itself (Sec. 3.1 as written)
# ----------------------------------------------------------------------------------------------
def vmax_digits(g32: np.ndarray, Q: int):
    """Sec. 3.1 divides every entry by the largest entry v = max_j |g_j| and expands |g_j| / v in binary.  The first Q
    digits as an integer: m_j = min(floor(|g_j| / v * 2^Q), 2^Q - 1); the cap is the reading for the entries with
    |g_j| = v, whose quotient 1 has no expansion below 1.  Returns (m, v); a zero row gives m = 0, v = 0.
    The quotient is taken in fp64: |g_j| 2^Q and v are exact there, the division is correctly rounded, and a quotient
    that is not an integer lies at least 2^-24 away from the next one (its denominator divides v's 24-bit
    significand), far more than the rounding error of a number below 2^24: so the floor is that of the exact ratio."""
    a = np.abs(g32.astype(np.float64))
    v = np.float32(np.abs(g32).max()) if g32.size else np.float32(0.0)
    if v == 0.0:
        return np.zeros(g32.shape, dtype=np.uint64), v
    q = np.floor(np.ldexp(a, Q) / np.float64(v))
    return np.minimum(q, float((1 << Q) - 1)).astype(np.uint64), v


def vbits_truncate_dense(row: np.ndarray, F: int, Q: int) -> np.ndarray:
    """C^F(g) of this ladder: sign_j * (m_j >> (Q - F)) * 2^-F * v, as float64 values."""
    g = as_f32(row)
    m, v = vmax_digits(g, Q)
    kept = (m >> np.uint64(Q - F)).astype(np.float64)
    return np.where(np.signbit(g), -1.0, 1.0) * np.ldexp(kept, -F) * np.float64(v)


def compress_vbits_row(row: np.ndarray, F: Sequence[int], p: Sequence[float], seed: int, step: int,
                       worker: int, force_level: Optional[int] = None):
    """One worker's message: level, the largest entry v (an fp32 number, "transmitted" with the message, Sec. 3.1),
    and the same planes as the power-of-two ladder: sign, F_0 base planes, F_l - F_{l-1} level planes, LSB first."""
    g = as_f32(row)
    L = len(F) - 1
    Q = F[L]
    assert 0 <= F[0] and all(F[i] < F[i + 1] for i in range(L)) and Q <= 24
    m, v = vmax_digits(g, Q)
    level = draw_level(p, seed, step, worker) if force_level is None else int(force_level)
    width = F[level] - F[level - 1]
    field = (m >> np.uint64(Q - F[level])) & np.uint64((1 << width) - 1)
    base = (m >> np.uint64(Q - F[0])) if F[0] > 0 else np.zeros_like(m)
    planes = [pack_plane(np.signbit(g))]
    for b in range(F[0]):
        planes.append(pack_plane(((base >> np.uint64(b)) & np.uint64(1)).astype(bool)))
    for b in range(width):
        planes.append(pack_plane(((field >> np.uint64(b)) & np.uint64(1)).astype(bool)))
    return dict(level=level, vmax=np.float32(v), planes=np.stack(planes), p_level=float(p[level - 1]))


def decode_vbits_row(msg, F: Sequence[int], d: int) -> np.ndarray:
    """g~_j = sign_j * [ fp32(f0_j) * c_0 + fp32(f_j) * c_l ], c_0 = fp32(v 2^-F_0), c_l = fp32(v 2^-F_l / p_l)
    (the constants in fp64, rounded once); products and the sum are single fp32 operations."""
    level, planes = msg["level"], msg["planes"]
    v = float(msg["vmax"])
    width = F[level] - F[level - 1]
    sign = unpack_plane(planes[0], d)
    f0 = np.zeros(d, dtype=np.uint32)
    for b in range(F[0]):
        f0 |= unpack_plane(planes[1 + b], d).astype(np.uint32) << np.uint32(b)
    f = np.zeros(d, dtype=np.uint32)
    for b in range(width):
        f |= unpack_plane(planes[1 + F[0] + b], d).astype(np.uint32) << np.uint32(b)
    p_l = msg["p_level"]
    c_l = np.float32(math.ldexp(v, -F[level]) / p_l) if p_l != 0.0 else np.float32(0.0)
    val = f.astype(np.float32) * c_l
    if F[0] > 0:
        c_0 = np.float32(math.ldexp(v, -F[0]))
        val = f0.astype(np.float32) * c_0 + val
    return np.where(sign, -val, val).astype(np.float32)


def compress_vbits(G: np.ndarray, F, p, seed: int, step: int):
    return [compress_vbits_row(G[i], F, p, seed, step, i) for i in range(G.shape[0])]


def aggregate_vbits(msgs, F, d: int, alpha: float) -> np.ndarray:
    acc = np.zeros(d, dtype=np.float32)
    for msg in msgs:
        acc = acc + decode_vbits_row(msg, F, d)
    return (np.float32(alpha) * acc).astype(np.float32)


# ----------------------------------------------------------------------------------------------
# floating-point bit-wise MLMC (App. B)
# ----------------------------------------------------------------------------------------------
MANT_BITS = 23   # fp32 inputs: the mantissa digits m_1..m_23 (the paper writes the fp64 case, 52 digits)


def float_truncate(g32: np.ndarray, F: int) -> np.ndarray:
    """Floating-point compressor C^F (App. B): sign and exponent kept, the mantissa sum truncated to its first F
    digits.  On the fp32 bit pattern this clears the low 23 - F mantissa bits (also right for denormals and zero)."""
    bits = np.ascontiguousarray(g32, dtype=np.float32).view(np.uint32)
    keep = np.uint32((0xFFFFFFFF << (MANT_BITS - F)) & 0xFFFFFFFF)
    return (bits & keep).view(np.float32)


def fbits_estimate_dense(row: np.ndarray, F: Sequence[int], level: int, p_level: float) -> np.ndarray:
    """g~ = C^{F_0}(g) + (C^{F_l}(g) - C^{F_{l-1}}(g)) / p_l (Eq. (5)) for the mantissa ladder F, as the fp32 vector the
    server adds: the residual is exact in fp32 (both terms share sign and exponent), then one fp32 multiply by
    w = fp32(1 / p_l) and one fp32 add."""
    g = as_f32(row)
    r = (float_truncate(g, F[level]) - float_truncate(g, F[level - 1])).astype(np.float32)
    return (float_truncate(g, F[0]) + (r * level_weight(p_level)).astype(np.float32)).astype(np.float32)


def compress_fbits_row(row: np.ndarray, F: Sequence[int], p: Sequence[float], seed: int, step: int, worker: int,
                       force_level: Optional[int] = None):
    """One worker's floating-point MLMC message: level; sign plane; 8 exponent planes (bits of the exponent field,
    LSB first); F_0 base planes (bits of the first F_0 mantissa digits as a number, LSB first); F_l - F_{l-1} level
    planes (bits of the mantissa digits F_{l-1}+1 .. F_l as a number, LSB first).  App. B: the residual keeps the sign
    and the exponent of the entry and adds the level's mantissa digits."""
    g = as_f32(row)
    L = len(F) - 1
    assert 0 <= F[0] and all(F[i] < F[i + 1] for i in range(L)) and F[L] <= MANT_BITS
    bits = np.ascontiguousarray(g).view(np.uint32)
    level = draw_level(p, seed, step, worker) if force_level is None else int(force_level)
    width = F[level] - F[level - 1]
    frac = bits & np.uint32(0x7FFFFF)
    E = (bits >> np.uint32(23)) & np.uint32(0xFF)
    base = frac >> np.uint32(MANT_BITS - F[0]) if F[0] > 0 else np.zeros_like(frac)
    field = (frac >> np.uint32(MANT_BITS - F[level])) & np.uint32((1 << width) - 1)
    planes = [pack_plane((bits >> np.uint32(31)).astype(bool))]
    for b in range(8):
        planes.append(pack_plane(((E >> np.uint32(b)) & np.uint32(1)).astype(bool)))
    for b in range(F[0]):
        planes.append(pack_plane(((base >> np.uint32(b)) & np.uint32(1)).astype(bool)))
    for b in range(width):
        planes.append(pack_plane(((field >> np.uint32(b)) & np.uint32(1)).astype(bool)))
    return dict(level=level, planes=np.stack(planes), p_level=float(p[level - 1]))


def decode_fbits_row(msg, F: Sequence[int], d: int) -> np.ndarray:
    """The fp32 vector the server adds for a floating-point MLMC message: with sign s, exponent field E, base digits
    f0 and level digits f, C^{F_0} = float(s, E, f0 << (23 - F_0)); the residual is float(s, E, f << (23 - F_l)) -
    float(s, E, 0) (exact in fp32); g~ = fp32(C^{F_0} + fp32(residual * w))."""
    level, planes = msg["level"], msg["planes"]
    width = F[level] - F[level - 1]
    sign = unpack_plane(planes[0], d).astype(np.uint32)
    E = np.zeros(d, dtype=np.uint32)
    for b in range(8):
        E |= unpack_plane(planes[1 + b], d).astype(np.uint32) << np.uint32(b)
    f0 = np.zeros(d, dtype=np.uint32)
    for b in range(F[0]):
        f0 |= unpack_plane(planes[9 + b], d).astype(np.uint32) << np.uint32(b)
    f = np.zeros(d, dtype=np.uint32)
    for b in range(width):
        f |= unpack_plane(planes[9 + F[0] + b], d).astype(np.uint32) << np.uint32(b)
    se = (sign << np.uint32(31)) | (E << np.uint32(23))
    base_val = (se | (f0 << np.uint32(MANT_BITS - F[0]))).view(np.float32) if F[0] > 0 else se.view(np.float32)
    r = ((se | (f << np.uint32(MANT_BITS - F[level]))).view(np.float32) - se.view(np.float32)).astype(np.float32)
    return (base_val + (r * level_weight(msg["p_level"])).astype(np.float32)).astype(np.float32)


def compress_fbits(G: np.ndarray, F, p, seed: int, step: int):
    return [compress_fbits_row(G[i], F, p, seed, step, i) for i in range(G.shape[0])]


def aggregate_fbits(msgs, F, d: int, alpha: float) -> np.ndarray:
    acc = np.zeros(d, dtype=np.float32)
    for msg in msgs:
        acc = acc + decode_fbits_row(msg, F, d)
    return (np.float32(alpha) * acc).astype(np.float32)


def message_bits_floating_point(F: Sequence[int], level: int, d: int, exponent_bits: int = 8) -> int:
    """Bits one worker sends for a floating-point MLMC message (App. B): per entry the sign, the exponent, the F_0 base
    digits and the level's digits, plus the level.  For fp64 (11 exponent bits, unit ladder of 52 digits) this is the
    paper's 13 d + log2(52), rounded up."""
    L = len(F) - 1
    return d * (1 + exponent_bits + F[0] + F[level] - F[level - 1]) + _ceil_log2(L)


# ----------------------------------------------------------------------------------------------
# Round-to-Nearest MLMC (Sec. 3.3 "RTN", App. G.2): C^l(v) = delta^l clip(round(v / delta^l), -c, c), delta^l = 2c / (2^l - 1)
# ----------------------------------------------------------------------------------------------
# Readings (the paper gives the formula only): the clipping value c is the largest magnitude of the vector and is sent
# with the message; "round" is round-half-to-even of the exact quotient (what torch.round and numpy.rint do); the clip
# acts on the rounded integer and keeps it in the range of a symmetric l-bit code, |n| <= 2^(l-1) - 1 (so 2^l - 1
# values, the count delta^l is built from); level 0 of a ladder that starts at 0 bits is the zero vector.  The ladder
# holds bit widths b_0 < b_1 < ... < b_L <= 16; the top level is not the identity, the estimate is unbiased for
# C^{b_L}(v), as for the fixed-point ladder.
def rtn_codes(g32: np.ndarray, c: np.float32, b: int) -> np.ndarray:
    """n_j = clamp(rne(v_j (2^b - 1) / (2c)), -(2^(b-1) - 1), 2^(b-1) - 1) as int64; b = 0 or c = 0 gives zeros.
    The quotient is rounded from its fp64 value and then corrected with the exact remainder |v| D - n 2c (both
    products have at most 41 significant bits and the remainder is exact in fp64), so the result is the rounding of
    the exact real quotient, ties to even."""
    if b == 0 or float(c) == 0.0:
        return np.zeros(g32.shape, dtype=np.int64)
    D = float((1 << b) - 1)
    a = np.abs(g32.astype(np.float64))
    num = a * D
    den = 2.0 * float(c)
    n = np.rint(num / den)
    rem = num - n * den                       # exact
    n = n + (rem > float(c)) - (rem < -float(c))
    tie = np.abs(rem) == float(c)             # exactly between two integers: the even one
    odd = np.fmod(n, 2.0) != 0.0
    n = np.where(tie & odd, n + np.sign(rem), n)
    n = np.minimum(n, float((1 << (b - 1)) - 1))
    return np.where(np.signbit(g32), -n, n).astype(np.int64)


def rtn_dense(row: np.ndarray, b: int) -> np.ndarray:
    """C^b(v) as float64 values: n_j * 2c / (2^b - 1)."""
    g = as_f32(row)
    c = np.float32(np.abs(g).max()) if g.size else np.float32(0.0)
    if b == 0 or c == 0:
        return np.zeros(g.shape)
    return rtn_codes(g, c, b).astype(np.float64) * (2.0 * float(c) / float((1 << b) - 1))


def rtn_residual_ints(g32: np.ndarray, c: np.float32, b_prev: int, b_cur: int) -> np.ndarray:
    """C^{b_cur} - C^{b_prev} = (2c / (D D')) k with the integers k_j = n_cur D' - n_prev D, D = 2^b_cur - 1,
    D' = 2^b_prev - 1 (D' = 1 and n_prev = 0 when b_prev = 0)."""
    D = (1 << b_cur) - 1
    Dp = (1 << b_prev) - 1 if b_prev > 0 else 1
    n_prev = rtn_codes(g32, c, b_prev) if b_prev > 0 else 0
    return rtn_codes(g32, c, b_cur) * Dp - n_prev * D


def rtn_level_norms_row(row: np.ndarray, B: Sequence[int]) -> List[float]:
    """Delta_l = ||C^{b_l}(v) - C^{b_{l-1}}(v)||_2 (Lemma 3.4), l = 1..L: (2c / (D D')) sqrt(sum_j k_j^2) with the
    integer sum exact, converted to fp64 once (round to nearest even), then one sqrt, one divide and one multiply."""
    g = as_f32(row)
    c = np.float32(np.abs(g).max()) if g.size else np.float32(0.0)
    out = []
    for l in range(1, len(B)):
        k = rtn_residual_ints(g, c, B[l - 1], B[l])
        kk = k.astype(np.int64)
        assert kk.size * int(np.abs(kk).max(initial=0)) ** 2 < 2 ** 63     # the int64 dot product below is exact
        S = int(np.dot(kk, kk))
        D = (1 << B[l]) - 1
        Dp = (1 << B[l - 1]) - 1 if B[l - 1] > 0 else 1
        out.append((2.0 * float(c) / float(D * Dp)) * math.sqrt(float(S)))
    return out


def _rtn_code_planes(n: np.ndarray, b: int) -> List[np.ndarray]:
    """The b planes of a code in two's complement truncated to b bits, least significant first."""
    u = n.astype(np.int64) & np.int64((1 << b) - 1)
    return [pack_plane(((u >> np.int64(q)) & np.int64(1)).astype(bool)) for q in range(b)]


def compress_rtn_row(row: np.ndarray, B: Sequence[int], p: Optional[Sequence[float]], seed: int, step: int, worker: int,
                     force_level: Optional[int] = None):
    """One worker's RTN MLMC message (Alg. 3 when p is None: probabilities from this row's residual norms): level,
    c, the coefficient fp32((2c / (D D')) / p_l) the server multiplies the residual integers with, and the planes of
    the codes n_{b_0} (if b_0 > 0), n_{b_{l-1}} (if l > 1) and n_{b_l}, in that order."""
    g = as_f32(row)
    L = len(B) - 1
    assert 0 <= B[0] and all(B[i] < B[i + 1] for i in range(L)) and B[L] <= 16
    c = np.float32(np.abs(g).max()) if g.size else np.float32(0.0)
    norms = rtn_level_norms_row(g, B)
    probs = adaptive_p(norms) if p is None else list(p)
    level = draw_level(probs, seed, step, worker) if force_level is None else int(force_level)
    p_l = float(probs[level - 1])
    planes = []
    if B[0] > 0:
        planes += _rtn_code_planes(rtn_codes(g, c, B[0]), B[0])
    if level > 1:
        planes += _rtn_code_planes(rtn_codes(g, c, B[level - 1]), B[level - 1])
    planes += _rtn_code_planes(rtn_codes(g, c, B[level]), B[level])
    D = (1 << B[level]) - 1
    Dp = (1 << B[level - 1]) - 1 if B[level - 1] > 0 else 1
    coef = np.float32((2.0 * float(c) / float(D * Dp)) / p_l) if p_l != 0.0 else np.float32(0.0)
    return dict(level=level, c=c, coef=coef, planes=np.stack(planes), p_level=p_l, norms=norms)


def _rtn_unpack_code(planes: np.ndarray, first: int, b: int, d: int) -> np.ndarray:
    u = np.zeros(d, dtype=np.int64)
    for q in range(b):
        u |= unpack_plane(planes[first + q], d).astype(np.int64) << np.int64(q)
    return np.where(u >= (1 << (b - 1)), u - (1 << b), u) if b > 0 else u


def decode_rtn_row(msg, B: Sequence[int], d: int) -> np.ndarray:
    """g~_j = fp32(n_{b_0}) * fp32(2c / D_0) + fp32(k_j) * coef with k_j = n_cur D' - n_prev D rebuilt from the codes;
    products and the sum are single fp32 operations (the first term only when b_0 > 0)."""
    level, planes = msg["level"], msg["planes"]
    at = 0
    n0 = None
    if B[0] > 0:
        n0 = _rtn_unpack_code(planes, 0, B[0], d)
        at = B[0]
    if level > 1:
        n_prev = _rtn_unpack_code(planes, at, B[level - 1], d)
        at += B[level - 1]
    else:
        n_prev = n0 if n0 is not None else np.zeros(d, dtype=np.int64)
    n_cur = _rtn_unpack_code(planes, at, B[level], d)
    D = (1 << B[level]) - 1
    Dp = (1 << B[level - 1]) - 1 if B[level - 1] > 0 else 1
    k = n_cur * Dp - n_prev * D
    val = k.astype(np.float32) * np.float32(msg["coef"])
    if n0 is not None:
        c0 = np.float32(2.0 * float(msg["c"]) / float((1 << B[0]) - 1))
        val = n0.astype(np.float32) * c0 + val
    return val.astype(np.float32)


def compress_rtn(G: np.ndarray, B, p, seed: int, step: int):
    return [compress_rtn_row(G[i], B, p, seed, step, i) for i in range(G.shape[0])]


def aggregate_rtn(msgs, B, d: int, alpha: float) -> np.ndarray:
    acc = np.zeros(d, dtype=np.float32)
    for msg in msgs:
        acc = acc + decode_rtn_row(msg, B, d)
    return (np.float32(alpha) * acc).astype(np.float32)


def message_bits_rtn(B: Sequence[int], level: int, d: int) -> int:
    """Bits of an RTN MLMC message: per entry the codes sent, plus c, the coefficient (32 bits each) and the level."""
    per = B[0] + (B[level - 1] if level > 1 else 0) + B[level]
    return d * per + 64 + _ceil_log2(len(B) - 1)


# ----------------------------------------------------------------------------------------------
# server aggregate
# ----------------------------------------------------------------------------------------------
def aggregate_sparse(msgs, d: int, alpha: float) -> np.ndarray:
    """out_j = fp32(alpha * acc_j); acc_j = fp32 sum over workers in worker order of the entries at j
    (a worker without an entry at j is skipped)."""
    acc = np.zeros(d, dtype=np.float32)
    for msg in msgs:
        idx = msg["idx"].astype(np.int64)
        acc[idx] = acc[idx] + msg["val"]
    return (np.float32(alpha) * acc).astype(np.float32)


def aggregate_bits(msgs, F, d: int, alpha: float) -> np.ndarray:
    acc = np.zeros(d, dtype=np.float32)
    for msg in msgs:
        acc = acc + decode_bits_row(msg, F, d)
    return (np.float32(alpha) * acc).astype(np.float32)


# ----------------------------------------------------------------------------------------------
# server update and message sizes
# ----------------------------------------------------------------------------------------------
def server_update(x: np.ndarray, gtilde: np.ndarray, eta: float) -> np.ndarray:
    """Alg. 2 / Alg. 3 "Server updates": x_{t+1} = x_t - eta * g~_t, per entry one fp32 multiply, then one fp32
    subtract (two roundings, no fused multiply-add)."""
    x = np.asarray(x, dtype=np.float32)
    step = (np.float32(eta) * np.asarray(gtilde, dtype=np.float32)).astype(np.float32)
    return (x - step).astype(np.float32)


def message_bits_topk(ladder: Sequence[int], level: int, d: int, value_bits: int = 32) -> int:
    """Bits one worker sends for a Top-k MLMC message (Sec. 3, Sec. 3.2: the residual is the entries of one rank
    band): every entry as a value and an index into d, plus the level: nnz * (value_bits + ceil(log2 d)) + ceil(log2 L)."""
    L = len(ladder) - 1
    nnz = ladder[0] + ladder[level] - ladder[level - 1]
    return nnz * (value_bits + _ceil_log2(d)) + _ceil_log2(L)


def message_bits_fixed_point(F: Sequence[int], level: int, d: int, scale_bits: int = 32) -> int:
    """Bits one worker sends for a fixed-point MLMC message (Sec. 3.1): per entry the sign, the F_0 base bits and the
    F_l - F_{l-1} bits of the level field, plus the scale and the level.  With the unit ladder F = 0..63 and a 64-bit
    scale this is the paper's 2 d + 64 + ceil(log2 63)."""
    L = len(F) - 1
    return d * (1 + F[0] + F[level] - F[level - 1]) + scale_bits + _ceil_log2(L)

