"""CPU-side checks of the built library: it loads, exports every declared symbol, and validates plans.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

import paper_2507_05508_amd as P
from paper_2507_05508_amd import binding
from oracle import mlmc as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "mlmc.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = set(re.findall(r"\b(mlmc_[a-z_0-9]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    assert os.path.exists(binding.LIB_PATH), "build first: python -m paper_2507_05508_amd.build"
    lib = ctypes.CDLL(binding.LIB_PATH)
    declared = _declared_functions()
    assert set(declared) == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_geometric_p_matches_lemma_3_3_form():
    for L in (1, 5, 10, 16):
        assert P.mlmc_geometric_p(L) == O.geometric_p(L)


def test_plan_validation():
    ok = P.Plan(P.MLMC_TOPK, 4, 65536, P.MLMC_F32, [2 ** (6 + l) for l in range(11)], P.mlmc_geometric_p(10), allocate=False)
    assert ok.sparse_capacity_worst == 4 * (64 + 32768) and ok.num_tiles == 16 and ok.workspace_bytes > 4 * 65536 * 4
    bad = [
        dict(kind=P.MLMC_TOPK, M=0, d=10, ladder=[0, 10], p=[1.0]),
        dict(kind=P.MLMC_TOPK, M=1, d=10, ladder=[0, 11], p=[1.0]),          # k_L > d
        dict(kind=P.MLMC_TOPK, M=1, d=10, ladder=[3, 3, 10], p=[0.5, 0.5]),   # not strictly increasing
        dict(kind=P.MLMC_TOPK, M=1, d=10, ladder=[-1, 10], p=[1.0]),
        dict(kind=P.MLMC_TOPK, M=1, d=10, ladder=[0, 5, 10], p=[0.5, 0.4]),   # does not sum to 1
        dict(kind=P.MLMC_TOPK, M=1, d=10, ladder=[0, 5, 10], p=[1.0, 0.0]),   # zero probability
        dict(kind=P.MLMC_TOPK, M=1, d=1 << 31, ladder=[0, 5], p=[1.0]),
        dict(kind=P.MLMC_TOPK, M=1, d=100, ladder=list(range(40)), p=None),   # L > MLMC_MAX_LEVELS
        dict(kind=P.MLMC_BITS, M=1, d=10, ladder=[0, 8, 25], p=[0.5, 0.5]),   # more than 24 bits
        dict(kind=P.MLMC_BITS, M=1, d=10, ladder=[0, 8, 16], p=None),         # adaptive bits not defined
        dict(kind=P.MLMC_VBITS, M=1, d=10, ladder=[0, 8, 25], p=[0.5, 0.5]),  # more than 24 bits
        dict(kind=P.MLMC_VBITS, M=1, d=10, ladder=[0, 8, 16], p=None),        # adaptive not defined
        dict(kind=P.MLMC_RTN, M=1, d=10, ladder=[0, 8, 17], p=None),          # codes wider than 16 bits
        dict(kind=P.MLMC_RTN, M=1, d=10, ladder=list(range(10)), p=None),     # more than 8 levels
        dict(kind=P.MLMC_RTN, M=1, d=10, ladder=[4, 14, 16], p=None),         # 4 + 14 + 16 code planes in one message
        dict(kind=P.MLMC_FBITS, M=1, d=10, ladder=[0, 8, 24], p=[0.5, 0.5]),  # more than 23 mantissa digits
        dict(kind=P.MLMC_FBITS, M=1, d=10, ladder=[0, 8, 16], p=None),        # adaptive not defined
        dict(kind=7, M=1, d=10, ladder=[0, 10], p=[1.0]),
    ]
    for b in bad:
        with pytest.raises(P.MlmcError):
            P.Plan(b["kind"], b["M"], b["d"], P.MLMC_F32, b["ladder"], b["p"], allocate=False)
    bits = P.Plan(P.MLMC_BITS, 8, 1000, P.MLMC_F32, [0, 1, 2, 4, 8, 16], P.mlmc_geometric_p(5), allocate=False)
    assert bits.num_planes == 9 and bits.sparse_capacity_worst == 0
    bits2 = P.Plan(P.MLMC_BITS, 8, 1000, P.MLMC_F32, [2, 3, 8, 12], P.mlmc_geometric_p(3), allocate=False)
    assert bits2.num_planes == 1 + 2 + 5
    vb = P.Plan(P.MLMC_VBITS, 8, 1000, P.MLMC_F32, [2, 3, 8, 12], P.mlmc_geometric_p(3), allocate=False)
    assert vb.num_planes == 1 + 2 + 5 and vb.sparse_capacity_worst == 0
    with pytest.raises(P.MlmcError):
        vb.set_sampling(2)   # the largest entry is read exactly
    rt = P.Plan(P.MLMC_RTN, 8, 1000, P.MLMC_F32, [0, 2, 4, 8, 16], None, allocate=False)
    assert rt.num_planes == 8 + 16 and rt.sparse_capacity_worst == 0     # the previous and the drawn level's codes
    rt2 = P.Plan(P.MLMC_RTN, 8, 1000, P.MLMC_F32, [2, 3, 5, 9], P.mlmc_geometric_p(3), allocate=False)
    assert rt2.num_planes == 2 + 5 + 9
    fb = P.Plan(P.MLMC_FBITS, 8, 1000, P.MLMC_F32, list(range(24)), P.mlmc_geometric_p(23), allocate=False)
    assert fb.num_planes == 10 and fb.sparse_capacity_worst == 0   # sign + 8 exponent bits + one mantissa digit (App. B)
    # tuning hooks are refused for the kinds they do not apply to
    tk = P.Plan(P.MLMC_TOPK, 4, 100_000, P.MLMC_F32, [10, 100, 100_000], None, allocate=False)
    tk.set_overlap(True)
    tk.set_overlap(False)
    with pytest.raises(P.MlmcError):
        bits.set_overlap(True)
