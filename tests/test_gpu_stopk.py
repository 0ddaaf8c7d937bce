"""GPU parity of s-segmented Top-k MLMC (uniform ladder k_l = s l, thousands of levels, Lemma 3.4 probabilities over
all of them) against the CPU oracle, bit for bit: norms of every band, drawn levels, the drawn segment, aggregate."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from gpu_util import check_topk_against_oracle, to_device

pytestmark = pytest.mark.gpu


def _run_and_check(G, s, dtype=P.MLMC_F32, steps=(0, 1, 2), seed=42, ld=None):
    M, d = G.shape
    plan = P.Plan(P.MLMC_STOPK, M, d, dtype, [s], None)
    ladder = O.stopk_ladder(d, s)
    assert plan.ladder == ladder and plan.L == len(ladder) - 1 and plan.sparse_capacity_worst == M * min(s, d)
    g = to_device(G, ld=ld)
    norms = P.mlmc_level_norms(plan, g)
    torch.cuda.synchronize()
    assert plan.status() == 0
    got = norms.cpu().numpy()
    for i in range(M):
        want, _ = O.level_norms_row(G[i], ladder)
        assert np.array_equal(got[i].view(np.uint64), np.array(want, dtype=np.float64).view(np.uint64)), f"row {i}: norms differ"
    for step in steps:
        msg = P.mlmc_compress_topk(plan, g, seed=seed, step=step)
        want = check_topk_against_oracle(plan, G, seed, step, msg, adaptive=True)
        assert plan.status() == 0
        assert np.array_equal(msg.norms.cpu().numpy().view(np.uint64), got.view(np.uint64))
        for use_tile in (True, False):
            out = P.mlmc_aggregate(plan, msg, 1.0 / M, use_tile_off=use_tile)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, d, 1.0 / M).view(np.uint32))
        bits = P.mlmc_message_bits(plan, msg).cpu().numpy()
        assert bits.tolist() == [O.message_bits_topk(ladder, m["level"], d) for m in want]


@pytest.mark.parametrize("name,d,M,s", [("resnet18_topk", 3 * 8192 + 777, 3, 64), ("resnet50_adaptive_topk", 100_003, 2, 100),
                                         ("tiny_topk", 20_000, 2, 7), ("resnet18_topk", 40_000, 2, 1)])
def test_stopk_segmented_workloads(name, d, M, s):
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    print(f"stopk {name} d={d} M={M} s={s}", flush=True)
    _run_and_check(W.generate(w), s)


def test_stopk_ties_zeros_denormals_and_padding():
    d = 2 * 8192 + 300
    G = np.stack(W.adversarial_rows(d))
    for s, ld in ((33, None), (1000, d + 3), (d, None), (d + 5, None), (d - 1, d + 1)):
        print(f"stopk adversarial s={s} ld={ld}", flush=True)
        _run_and_check(G, s, steps=(0, 5), ld=ld)


def test_stopk_bf16_rows():
    w = W.scaled(W.WORKLOADS["bert_adaptive_topk_bf16"], d=70_000, M=2)
    _run_and_check(W.generate(w), 512, dtype=P.MLMC_BF16)


def test_stopk_exponential_decay_draws_many_levels():
    """Assumption 3.5 input: the level probabilities decay geometrically, so repeated steps draw many distinct levels."""
    d, s = 4 * 8192, 32
    rng = np.random.default_rng(9)
    g = np.empty(d, dtype=np.float32)
    g[rng.permutation(d)] = (2.0 * np.exp(-0.5 * 0.0004 * np.arange(d))).astype(np.float32) * rng.choice(np.array([-1, 1], dtype=np.float32), size=d)
    G = np.stack([g, g[::-1].copy()])
    plan = P.Plan(P.MLMC_STOPK, 2, d, P.MLMC_F32, [s], None)
    gd = to_device(G)
    seen = set()
    for step in range(12):
        msg = P.mlmc_compress_topk(plan, gd, seed=3, step=step)
        want = check_topk_against_oracle(plan, G, 3, step, msg, adaptive=True)
        seen |= {m["level"] for m in want}
    assert len(seen) >= 10


def test_stopk_plan_validation():
    for bad in (dict(d=1000, s=0), dict(d=10_000_000, s=100)):   # s < 1; more than MLMC_MAX_SLEVELS levels
        with pytest.raises(P.MlmcError):
            P.Plan(P.MLMC_STOPK, 2, bad["d"], P.MLMC_F32, [bad["s"]], None, allocate=False)
    with pytest.raises(P.MlmcError):
        P.Plan(P.MLMC_STOPK, 2, 1000, P.MLMC_F32, [10], [0.5, 0.5], allocate=False)   # fixed p is not defined here
