"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy
as 1, 2, 3", SC'11), written from the published definition with Python integers.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  The paper being reproduced only says "sample l ~ p"
(Alg. 2, Alg. 3); a counter-based generator makes that draw a pure function of (seed, step, worker).
"""

_MASK32 = 0xFFFFFFFF
_MUL_A = 0xD2511F53   # multiplier applied to counter word 0
_MUL_B = 0xCD9E8D57   # multiplier applied to counter word 2
_WEYL_A = 0x9E3779B9  # key schedule increment for key word 0 (golden ratio)
_WEYL_B = 0xBB67AE85  # key schedule increment for key word 1 (sqrt(3) - 1)


def philox4x32_10(counter, key):
    """counter: 4 uint32 words, key: 2 uint32 words -> 4 uint32 output words."""
    c0, c1, c2, c3 = (int(x) & _MASK32 for x in counter)
    k0, k1 = (int(x) & _MASK32 for x in key)
    for r in range(10):
        if r > 0:
            k0 = (k0 + _WEYL_A) & _MASK32
            k1 = (k1 + _WEYL_B) & _MASK32
        pa = _MUL_A * c0
        pb = _MUL_B * c2
        c0, c1, c2, c3 = ((pb >> 32) ^ c1 ^ k0) & _MASK32, pb & _MASK32, ((pa >> 32) ^ c3 ^ k1) & _MASK32, pa & _MASK32
    return c0, c1, c2, c3


def level_uniform(seed: int, step: int, worker: int) -> int:
    """The one 32-bit uniform used per (worker, step): output word 0 with
    key = (seed_lo, seed_hi) and counter = (step_lo, step_hi, worker, 0)."""
    seed &= 0xFFFFFFFFFFFFFFFF
    step &= 0xFFFFFFFFFFFFFFFF
    return philox4x32_10((step & _MASK32, step >> 32, worker & _MASK32, 0), (seed & _MASK32, seed >> 32))[0]
