"""Seeded synthetic gradient workloads (inputs only -- none of the method's arithmetic lives here).

Both the CPU oracle's tests and the HIP path's tests / benchmark draw their inputs from this module so
that the two sides see byte-identical data.  Everything is generated on the host with numpy's PCG64
and is a pure function of (workload name, seed).

The workloads stand in for the gradient shapes of the paper's experiments (Sec. 5, App. G): d ~ 1.1e7
parameters (ResNet-18), d ~ 2.6e7 (ResNet-50 scale), d ~ 1.2e8 (BERT scale), M in {4, 8, 16} workers, with
"Gaussian-like, far from uniform" entries (Sec. 3.2, Sec. 3.3): a model is a list of tensors, each with
its own scale, so a row is a concatenation of segments with widely spread standard deviations.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str                 # "topk" | "stopk" | "bits" (fixed-point ladder) | "vbits" (the same, divided by the largest entry) | "fbits" (floating-point ladder) | "rtn" (Round-to-Nearest ladder)
    M: int                    # workers (rows)
    d: int                    # gradient dimension
    dtype: str                # "f32" | "bf16"
    L: int                    # number of drawable levels
    ladder: tuple             # k_0..k_L (topk) or F_0..F_L (bits)
    adaptive: bool            # level probabilities from per-level residual norms
    gen: str                  # generator recipe name
    seed: int = 0
    steps: int = 1
    extra: dict = field(default_factory=dict)


def geometric_rank_ladder(d: int, L: int) -> tuple:
    """k_l = floor(d / 2^(L-l)), l = 0..L, so k_L = d."""
    return tuple(int(d) >> (L - l) for l in range(L + 1))


def _mk(name, kind, M, d, dtype, L, ladder, adaptive, gen, seed=0, steps=1, **extra):
    return Workload(name, kind, M, d, dtype, L, tuple(int(x) for x in ladder), adaptive, gen, seed, steps, extra)


WORKLOADS = {
    # Tiny Top-k MLMC, iid N(0,1), k_l = 2^(6+l)
    "tiny_topk": _mk("tiny_topk", "topk", 4, 65536, "f32", 10, [2 ** (6 + l) for l in range(11)], False,
                     "iid_normal", seed=0, steps=100),
    # ResNet-18 scale, fixed p
    "resnet18_topk": _mk("resnet18_topk", "topk", 8, 11_689_512, "f32", 10,
                         geometric_rank_ladder(11_689_512, 10), False, "segmented_normal",
                         seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1),
    # ResNet-50 scale, adaptive p, 0.1% x100 outliers
    "resnet50_adaptive_topk": _mk("resnet50_adaptive_topk", "topk", 16, 25_557_032, "f32", 12,
                                  geometric_rank_ladder(25_557_032, 12), True, "segmented_normal_outliers",
                                  seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1,
                                  outlier_every=1000, outlier_gain=100.0),
    # bit-wise ladder at ResNet-18 scale
    "resnet18_bits": _mk("resnet18_bits", "bits", 8, 11_689_512, "f32", 5, [0, 1, 2, 4, 8, 16], False,
                         "segmented_normal", seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1),
    # the same ladder with entries divided by the largest entry itself (Sec. 3.1 as written)
    "resnet18_vbits": _mk("resnet18_vbits", "vbits", 8, 11_689_512, "f32", 5, [0, 1, 2, 4, 8, 16], False,
                          "segmented_normal", seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1),
    # Round-to-Nearest ladder at the widths the paper's plain RTN runs use (App. G.2: l in {2, 4, 8, 16}), adaptive p
    "resnet18_rtn": _mk("resnet18_rtn", "rtn", 8, 11_689_512, "f32", 4, [0, 2, 4, 8, 16], True,
                        "segmented_normal", seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1),
    # s-segmented Top-k at ResNet-18 scale: s = 0.001 n (the smallest k of App. G.1), 1000 levels, adaptive p over all of them
    "resnet18_stopk": _mk("resnet18_stopk", "stopk", 8, 11_689_512, "f32", 1000,
                          [min(11_690 * l, 11_689_512) for l in range(1001)], True, "segmented_normal",
                          seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1, s=11_690),
    # floating-point bit-wise ladder (one mantissa digit per level) at ResNet-18 scale
    "resnet18_fbits": _mk("resnet18_fbits", "fbits", 8, 11_689_512, "f32", 23, list(range(24)), False,
                          "segmented_normal", seed=0, steps=5, segments=62, std_lo=1e-4, std_hi=1e-1),
    # BERT scale, bf16 inputs, heavy tails
    "bert_adaptive_topk_bf16": _mk("bert_adaptive_topk_bf16", "topk", 4, 124_439_808, "bf16", 16,
                                   geometric_rank_ladder(124_439_808, 16), True, "segmented_student_t",
                                   seed=0, steps=1, segments=148, std_lo=1e-5, std_hi=1e-2, nu=3.0),
}


def scaled(w: Workload, d: int, M: Optional[int] = None, name: Optional[str] = None) -> Workload:
    """Same recipe at another size (used by parity tests: same structure, oracle-sized)."""
    M = w.M if M is None else M
    if w.kind == "stopk":
        s_len = max(1, d // 1000)
        L = -(-d // s_len)
        extra = dict(w.extra, s=s_len)
        return Workload(name or f"{w.name}@d{d}m{M}", w.kind, M, d, w.dtype, L, tuple(min(s_len * l, d) for l in range(L + 1)),
                        w.adaptive, w.gen, w.seed, w.steps, extra)
    if w.kind == "topk":
        if w.gen == "iid_normal":
            ladder = tuple(min(d, k) for k in w.ladder)
            # keep the ladder strictly increasing after clamping
            lad = [ladder[0]]
            for k in ladder[1:]:
                if k > lad[-1]:
                    lad.append(k)
            if lad[-1] != d:
                lad.append(d)
            ladder = tuple(lad)
        else:
            ladder = geometric_rank_ladder(d, w.L)
        L = len(ladder) - 1
    else:
        ladder, L = w.ladder, w.L
    return Workload(name or f"{w.name}@d{d}m{M}", w.kind, M, d, w.dtype, L, ladder, w.adaptive, w.gen,
                    w.seed, w.steps, dict(w.extra))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def segment_layout(d: int, n_seg: int, std_lo: float, std_hi: float, seed: int):
    """Segment lengths and per-segment scales, shared by all rows (workers share the model).

    weights exp(U(0, ln 1e4)); lengths max(1, floor(d*w/sum w)); the remainder goes to the last
    segment; scales log-uniform in [std_lo, std_hi].
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    n_seg = max(1, min(n_seg, d))
    w = np.exp(rng.uniform(0.0, math.log(1e4), size=n_seg))
    lens = np.maximum(1, np.floor(d * w / w.sum()).astype(np.int64))
    # fix the total: trim the largest segments while too long, then put the remainder on the last one
    excess = int(lens.sum()) - d
    while excess > 0:
        j = int(np.argmax(lens))
        take = min(excess, int(lens[j]) - 1)
        lens[j] -= take
        excess -= take
    lens[-1] += d - int(lens.sum())
    std = np.exp(rng.uniform(math.log(std_lo), math.log(std_hi), size=n_seg))
    assert lens.sum() == d and (lens >= 1).all()
    return lens, std


def _row_rng(seed: int, row: int):
    return np.random.Generator(np.random.PCG64(seed + 1 + row))


def generate_row(w: Workload, row: int, layout=None) -> np.ndarray:
    """One worker's gradient: float32 array, or uint16 bf16 bit patterns when w.dtype == 'bf16'."""
    rng = _row_rng(w.seed, row)
    d = w.d
    if w.gen == "iid_normal":
        g = rng.standard_normal(d, dtype=np.float32)
    elif w.gen in ("segmented_normal", "segmented_normal_outliers"):
        lens, std = layout if layout is not None else segment_layout(
            d, w.extra["segments"], w.extra["std_lo"], w.extra["std_hi"], w.seed)
        g = rng.standard_normal(d, dtype=np.float32)
        g *= np.repeat(std.astype(np.float32), lens)
        if w.gen == "segmented_normal_outliers":
            n_out = d // int(w.extra["outlier_every"])
            if n_out > 0:
                pos = rng.choice(d, size=n_out, replace=False)
                g[pos] *= np.float32(w.extra["outlier_gain"])
    elif w.gen == "segmented_student_t":
        lens, std = layout if layout is not None else segment_layout(
            d, w.extra["segments"], w.extra["std_lo"], w.extra["std_hi"], w.seed)
        g = np.empty(d, dtype=np.float32)
        # chunked so the float64 intermediates stay small
        scale = np.repeat(std.astype(np.float32), lens)
        step = 1 << 22
        for s in range(0, d, step):
            e = min(d, s + step)
            g[s:e] = rng.standard_t(w.extra["nu"], size=e - s).astype(np.float32)
        g *= scale
    else:
        raise ValueError(f"unknown generator {w.gen}")
    if w.dtype == "bf16":
        return f32_to_bf16_bits(g)
    return g


def generate(w: Workload) -> np.ndarray:
    """All M rows: array [M, d] float32, or uint16 bf16 bit patterns."""
    layout = None
    if w.gen != "iid_normal":
        layout = segment_layout(w.d, w.extra["segments"], w.extra["std_lo"], w.extra["std_hi"], w.seed)
    out = np.empty((w.M, w.d), dtype=np.uint16 if w.dtype == "bf16" else np.float32)
    for i in range(w.M):
        out[i] = generate_row(w, i, layout)
    return out


def adversarial_rows(d: int, seed: int = 0) -> List[np.ndarray]:
    """Float32 rows of length d that stress ordering rules: ties, signed zeros, denormals, constants."""
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    rows = []
    rows.append(np.full(d, 0.75, dtype=np.float32))                                 # all equal
    rows.append(np.zeros(d, dtype=np.float32))                                      # all zero
    z = np.zeros(d, dtype=np.float32); z[::2] = -0.0; z[::7] = 1e-3; rows.append(z)  # signed zeros + few values
    q = rng.integers(-3, 4, size=d).astype(np.float32) * np.float32(0.125); rows.append(q)  # heavy ties
    den = (rng.integers(0, 1 << 10, size=d).astype(np.uint32)).view(np.float32).copy()
    den[::3] *= -1; rows.append(den)                                                # denormals with ties
    mix = rng.standard_normal(d).astype(np.float32)
    mix[rng.integers(0, d, size=max(1, d // 8))] = mix[0]                           # a large tie class in Gaussian data
    rows.append(mix)
    nar = (np.float32(1.0) + rng.integers(0, 1 << 12, size=d).astype(np.float32) * np.float32(2.0 ** -23))
    nar[::2] *= -1; rows.append(nar.astype(np.float32))                             # one exponent, low mantissa bits only
    wide = np.exp(rng.uniform(-80, 80, size=d)).astype(np.float32); rows.append(wide)  # every exponent populated
    return rows
