"""GPU parity of the floating-point bit-wise MLMC path (App. B: sign + exponent + mantissa digits of the drawn level)
and of its aggregate / fused update / message sizes against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _check(plan, G, F, p, seed, step, msg):
    torch.cuda.synchronize()
    level = msg.level.cpu().numpy()
    planes = msg.planes.cpu().numpy().view(np.uint64)
    want = O.compress_fbits(G, F, p, seed, step)
    for i in range(G.shape[0]):
        assert level[i] == want[i]["level"], (i, level[i], want[i]["level"])
        n = want[i]["planes"].shape[0]
        assert np.array_equal(planes[i, :n], want[i]["planes"]), f"row {i}: planes differ"
    return want


@pytest.mark.parametrize("F", [list(range(24)), [0, 1, 2, 4, 8, 16, 23], [3, 5, 12, 20], [0, 23]])
@pytest.mark.parametrize("d", [3 * 4096 + 77, 64, 100_003])
def test_fbits_compress_aggregate_update(F, d):
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=3)
    G = W.generate(w)
    G[1] *= np.float32(1e-3)
    p = O.geometric_p(len(F) - 1)
    plan = P.Plan(P.MLMC_FBITS, 3, d, P.MLMC_F32, F, p)
    assert plan.num_planes == 9 + F[0] + max(F[l] - F[l - 1] for l in range(1, len(F)))
    g = to_device(G)
    x_ref = np.zeros(d, dtype=np.float32)
    x = torch.zeros(d, dtype=torch.float32, device="cuda:0")
    for step in range(4):
        print(f"fbits F={F} d={d} step={step}", flush=True)
        msg = P.mlmc_compress_bits(plan, g, seed=11, step=step)
        want = _check(plan, G, F, p, 11, step, msg)
        assert plan.status() == 0
        out = P.mlmc_aggregate(plan, msg, 1.0 / 3)
        torch.cuda.synchronize()
        ref = O.aggregate_fbits(want, F, d, 1.0 / 3)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
        x_ref = O.server_update(x_ref, ref, 0.1)
        P.mlmc_aggregate_update(plan, msg, 1.0 / 3, 0.1, x)
        torch.cuda.synchronize()
        assert np.array_equal(x.cpu().numpy().view(np.uint32), x_ref.view(np.uint32))
        bits = P.mlmc_message_bits(plan, msg).cpu().numpy()
        assert bits.tolist() == [O.message_bits_floating_point(F, m["level"], d) for m in want]


def test_fbits_adversarial_padded_and_bf16_rows():
    d = 2 * 4096 + 300
    G = np.stack(W.adversarial_rows(d))
    F = list(range(24))
    p = O.geometric_p(23)
    plan = P.Plan(P.MLMC_FBITS, G.shape[0], d, P.MLMC_F32, F, p)
    for ld in (d, d + 1, d + 6):
        g = to_device(G, ld=ld)
        for step in range(3):
            print(f"fbits adversarial ld={ld} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=2, step=step)
            want = _check(plan, G, F, p, 2, step, msg)
            out = P.mlmc_aggregate(plan, msg, 1.0)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_fbits(want, F, d, 1.0).view(np.uint32))
    w = W.scaled(W.WORKLOADS["bert_adaptive_topk_bf16"], d=50_000, M=2)
    Gb = W.generate(w)
    Fb = [0, 1, 2, 4, 7]   # bf16 has seven mantissa digits: deeper levels would be all zero
    pb = O.geometric_p(4)
    planb = P.Plan(P.MLMC_FBITS, 2, w.d, P.MLMC_BF16, Fb, pb)
    gb = to_device(Gb)
    for step in range(3):
        msg = P.mlmc_compress_bits(planb, gb, seed=1, step=step)
        want = _check(planb, Gb, Fb, pb, 1, step, msg)
        out = P.mlmc_aggregate(planb, msg, 0.5)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_fbits(want, Fb, w.d, 0.5).view(np.uint32))


@pytest.mark.parametrize("seed", [5, 6])
def test_fbits_random_plans_and_inputs(seed):
    rng = np.random.default_rng(seed)
    for case in range(20):
        M = int(rng.choice([1, 2, 3, 5, 9]))
        d = int(rng.choice([rng.integers(1, 200), rng.integers(200, 20000), rng.integers(20000, 150000)]))
        nF = int(rng.integers(2, 8))
        F = np.sort(rng.choice(np.arange(0, 24), size=nF, replace=False)).tolist()
        kind = int(rng.integers(0, 3))
        if kind == 0:
            G = rng.standard_normal((M, d)).astype(np.float32)
        elif kind == 1:
            G = (rng.standard_normal((M, d)) * np.exp(rng.uniform(-80, 30, size=(M, 1)))).astype(np.float32)
            G[rng.random((M, d)) < 0.4] = 0.0
        else:
            G = rng.integers(-5, 6, size=(M, d)).astype(np.float32)
        p = O.geometric_p(len(F) - 1)
        plan = P.Plan(P.MLMC_FBITS, M, d, P.MLMC_F32, F, p)
        g = to_device(G, ld=d + int(rng.integers(1, 4)) if rng.random() < 0.3 else None)
        call_seed = int(rng.integers(0, 2**40))
        for step in range(2):
            print(f"fbits random case {case}: M={M} d={d} F={F} kind={kind} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=call_seed, step=step)
            want = _check(plan, G, F, p, call_seed, step, msg)
            assert plan.status() == 0
            out = P.mlmc_aggregate(plan, msg, 0.25)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_fbits(want, F, d, 0.25).view(np.uint32))
