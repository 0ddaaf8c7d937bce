"""GPU parity of the fixed-point bit-wise MLMC path that divides by the largest entry itself (Sec. 3.1 as written)
and of its aggregate against the CPU oracle, bit for bit."""
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
    M, d = G.shape
    level = msg.level.cpu().numpy()
    vbits = msg.scale_exp.cpu().numpy().view(np.uint32)
    planes = msg.planes.cpu().numpy().view(np.uint64)
    want = O.compress_vbits(as_f32_rows(G), F, p, seed, step)
    for i in range(M):
        assert level[i] == want[i]["level"], (i, level[i], want[i]["level"])
        assert vbits[i] == np.float32(want[i]["vmax"]).view(np.uint32), (i, hex(vbits[i]), want[i]["vmax"])
        n = want[i]["planes"].shape[0]
        assert np.array_equal(planes[i, :n], want[i]["planes"]), f"row {i}: planes differ"
    return want


def as_f32_rows(G):
    return np.stack([O.as_f32(G[i]) for i in range(G.shape[0])])


@pytest.mark.parametrize("F", [[0, 1, 2, 4, 8, 16], [2, 3, 8, 12], [0, 24], list(range(17))])
@pytest.mark.parametrize("d", [3 * 4096 + 77, 64, 100_003])
def test_vbits_compress_and_aggregate(F, d):
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=3)
    G = W.generate(w)
    p = O.geometric_p(len(F) - 1)
    plan = P.Plan(P.MLMC_VBITS, 3, d, P.MLMC_F32, F, p)
    g = to_device(G)
    for step in range(5):
        print(f"vbits F={F} d={d} step={step}", flush=True)
        msg = P.mlmc_compress_bits(plan, g, seed=11, step=step)
        want = _check(plan, G, F, p, 11, step, msg)
        assert plan.status() == 0
        out = P.mlmc_aggregate(plan, msg, 1.0 / 3)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_vbits(want, F, d, 1.0 / 3).view(np.uint32))


def test_vbits_adversarial_padded_and_bf16_rows():
    d = 2 * 4096 + 300
    G = np.stack(W.adversarial_rows(d))
    F = [0, 1, 2, 4, 8, 16]
    p = O.geometric_p(5)
    plan = P.Plan(P.MLMC_VBITS, G.shape[0], d, P.MLMC_F32, F, p)
    for ld in (d, d + 1, d + 6):
        g = to_device(G, ld=ld)
        for step in range(3):
            print(f"vbits adversarial ld={ld} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=2, step=step)
            want = _check(plan, G, F, p, 2, step, msg)
            out = P.mlmc_aggregate(plan, msg, 1.0)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_vbits(want, F, d, 1.0).view(np.uint32))
    w = W.scaled(W.WORKLOADS["bert_adaptive_topk_bf16"], d=50_000, M=2)
    Gb = W.generate(w)
    Fb = [0, 1, 2, 4, 8]
    pb = O.geometric_p(4)
    planb = P.Plan(P.MLMC_VBITS, 2, w.d, P.MLMC_BF16, Fb, pb)
    gb = to_device(Gb)
    for step in range(3):
        print(f"vbits bf16 step={step}", flush=True)
        msg = P.mlmc_compress_bits(planb, gb, seed=1, step=step)
        _check(planb, Gb, Fb, pb, 1, step, msg)


@pytest.mark.parametrize("seed", [3, 4])
def test_vbits_random_plans_and_inputs(seed):
    """Randomised valid calls (row counts, lengths, ladders up to 24 bits, value families with zeros, ties at the
    maximum and very small or large scales, padded rows), the update of a model and the message sizes included."""
    rng = np.random.default_rng(seed)
    for case in range(25):
        M = int(rng.choice([1, 2, 3, 5, 9]))
        d = int(rng.choice([rng.integers(1, 200), rng.integers(200, 20000), rng.integers(20000, 150000)]))
        nF = int(rng.integers(2, 8))
        F = np.sort(rng.choice(np.arange(0, 25), size=nF, replace=False)).tolist()
        L = len(F) - 1
        kind = int(rng.integers(0, 3))
        if kind == 0:
            G = rng.standard_normal((M, d)).astype(np.float32)
        elif kind == 1:
            G = (rng.standard_normal((M, d)) * np.exp(rng.uniform(-60, 40, size=(M, 1)))).astype(np.float32)
            G[rng.random((M, d)) < 0.4] = 0.0
        else:
            G = rng.integers(-5, 6, size=(M, d)).astype(np.float32)   # the largest magnitude many times over
            if M > 1:
                G[0] = 0.0   # an all-zero row
        p = O.geometric_p(L)
        plan = P.Plan(P.MLMC_VBITS, M, d, P.MLMC_F32, F, p)
        g = to_device(G, ld=d + int(rng.integers(1, 4)) if rng.random() < 0.3 else None)
        call_seed = int(rng.integers(0, 2**40))
        x0 = rng.standard_normal(d).astype(np.float32)
        for step in range(2):
            print(f"vbits random case {case}: M={M} d={d} F={F} kind={kind} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=call_seed, step=step)
            want = _check(plan, G, F, p, call_seed, step, msg)
            assert plan.status() == 0
            x = torch.from_numpy(x0.copy()).to("cuda:0")
            out = torch.empty(d, dtype=torch.float32, device="cuda:0")
            P.mlmc_aggregate_update(plan, msg, 0.25, 0.1, x, out=out)
            bits = P.mlmc_message_bits(plan, msg)
            torch.cuda.synchronize()
            ref = O.aggregate_vbits(want, F, d, 0.25)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
            assert np.array_equal(x.cpu().numpy().view(np.uint32), O.server_update(x0, ref, 0.1).view(np.uint32))
            assert bits.cpu().numpy().tolist() == [O.message_bits_fixed_point(F, m["level"], d) for m in want]
