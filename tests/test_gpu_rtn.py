"""GPU parity of Round-to-Nearest MLMC (Sec. 3.3, App. G.2: codes, residual norms, adaptive draw, code planes) and of
its aggregate against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _check(plan, G, B, p, seed, step, msg):
    torch.cuda.synchronize()
    M, d = G.shape
    level = msg.level.cpu().numpy()
    scale = msg.scale_exp.cpu().numpy().view(np.uint32)
    norms = msg.norms.cpu().numpy()
    planes = msg.planes.cpu().numpy().view(np.uint64)
    want = O.compress_rtn(G, B, p, seed, step)
    for i in range(M):
        assert np.array_equal(norms[i].view(np.uint64), np.array(want[i]["norms"], dtype=np.float64).view(np.uint64)), (i, norms[i], want[i]["norms"])
        assert level[i] == want[i]["level"], (i, level[i], want[i]["level"])
        assert scale[i, 0] == np.float32(want[i]["c"]).view(np.uint32) and scale[i, 1] == np.float32(want[i]["coef"]).view(np.uint32), (i, scale[i], want[i]["c"], want[i]["coef"])
        n = want[i]["planes"].shape[0]
        assert np.array_equal(planes[i, :n], want[i]["planes"]), f"row {i}: planes differ"
    return want


@pytest.mark.parametrize("B", [[0, 2, 4, 8, 16], [2, 3, 5, 9], [0, 16], [0, 1, 2, 3, 4, 5, 6, 7, 8]])
@pytest.mark.parametrize("d", [3 * 4096 + 77, 64, 100_003])
@pytest.mark.parametrize("adaptive", [True, False])
def test_rtn_compress_and_aggregate(B, d, adaptive):
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=3)
    G = W.generate(w)
    p = None if adaptive else O.geometric_p(len(B) - 1)
    plan = P.Plan(P.MLMC_RTN, 3, d, P.MLMC_F32, B, p)
    g = to_device(G)
    for step in range(4):
        print(f"rtn B={B} d={d} adaptive={adaptive} step={step}", flush=True)
        msg = P.mlmc_compress_rtn(plan, g, seed=11, step=step)
        want = _check(plan, G, B, p, 11, step, msg)
        assert plan.status() == 0
        out = P.mlmc_aggregate(plan, msg, 1.0 / 3)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_rtn(want, B, d, 1.0 / 3).view(np.uint32))


def test_rtn_ties_adversarial_padded_and_bf16_rows():
    d = 2 * 4096 + 300
    rows = W.adversarial_rows(d)
    tie = np.zeros(d, dtype=np.float32)   # c = 3.5 and width 3: the quotient is the entry itself, half-integers are ties
    tie[: 4 * (d // 4)] = np.tile(np.array([0.5, -1.5, 2.5, -0.5], dtype=np.float32), d // 4)
    tie[5] = 3.5
    G = np.stack(rows + [tie])
    B = [0, 3, 8]
    plan = P.Plan(P.MLMC_RTN, G.shape[0], d, P.MLMC_F32, B, None)
    for ld in (d, d + 1, d + 6):
        g = to_device(G, ld=ld)
        for step in range(3):
            print(f"rtn adversarial ld={ld} step={step}", flush=True)
            msg = P.mlmc_compress_rtn(plan, g, seed=2, step=step)
            want = _check(plan, G, B, None, 2, step, msg)
            out = P.mlmc_aggregate(plan, msg, 1.0)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_rtn(want, B, d, 1.0).view(np.uint32))
    w = W.scaled(W.WORKLOADS["bert_adaptive_topk_bf16"], d=50_000, M=2)
    Gb = W.generate(w)
    Gf = np.stack([O.as_f32(Gb[i]) for i in range(2)])
    planb = P.Plan(P.MLMC_RTN, 2, w.d, P.MLMC_BF16, [0, 2, 4, 8], None)
    gb = to_device(Gb)
    for step in range(3):
        print(f"rtn bf16 step={step}", flush=True)
        msg = P.mlmc_compress_rtn(planb, gb, seed=1, step=step)
        _check(planb, Gf, [0, 2, 4, 8], None, 1, step, msg)


@pytest.mark.parametrize("seed", [7, 8])
def test_rtn_random_plans_and_inputs(seed):
    """Randomised valid calls (row counts, lengths, ladders, value families with zeros and extreme scales, padded rows),
    with the norms-only entry point, the update of a model and the message sizes."""
    rng = np.random.default_rng(seed)
    for case in range(20):
        M = int(rng.choice([1, 2, 3, 5, 9]))
        d = int(rng.choice([rng.integers(1, 200), rng.integers(200, 20000), rng.integers(20000, 150000)]))
        while True:
            nB = int(rng.integers(2, 7))
            B = np.sort(rng.choice(np.arange(0, 17), size=nB, replace=False)).tolist()
            if B[0] + max((B[l - 1] if l > 1 else 0) + B[l] for l in range(1, nB)) <= 32:
                break
        L = len(B) - 1
        kind = int(rng.integers(0, 3))
        if kind == 0:
            G = rng.standard_normal((M, d)).astype(np.float32)
        elif kind == 1:
            G = (rng.standard_normal((M, d)) * np.exp(rng.uniform(-60, 40, size=(M, 1)))).astype(np.float32)
            G[rng.random((M, d)) < 0.4] = 0.0
        else:
            G = rng.integers(-5, 6, size=(M, d)).astype(np.float32)
            if M > 1:
                G[0] = 0.0
        p = None if case % 3 else O.geometric_p(L)
        plan = P.Plan(P.MLMC_RTN, M, d, P.MLMC_F32, B, p)
        g = to_device(G, ld=d + int(rng.integers(1, 4)) if rng.random() < 0.3 else None)
        call_seed = int(rng.integers(0, 2**40))
        x0 = rng.standard_normal(d).astype(np.float32)
        print(f"rtn random case {case}: M={M} d={d} B={B} kind={kind}", flush=True)
        nr = P.mlmc_level_norms(plan, g)
        torch.cuda.synchronize()
        for i in range(M):
            assert np.array_equal(nr[i].cpu().numpy().view(np.uint64), np.array(O.rtn_level_norms_row(G[i], B), dtype=np.float64).view(np.uint64))
        for step in range(2):
            msg = P.mlmc_compress_rtn(plan, g, seed=call_seed, step=step)
            want = _check(plan, G, B, p, call_seed, step, msg)
            assert plan.status() == 0
            x = torch.from_numpy(x0.copy()).to("cuda:0")
            out = torch.empty(d, dtype=torch.float32, device="cuda:0")
            P.mlmc_aggregate_update(plan, msg, 0.25, 0.1, x, out=out)
            bits = P.mlmc_message_bits(plan, msg)
            torch.cuda.synchronize()
            ref = O.aggregate_rtn(want, B, d, 0.25)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
            assert np.array_equal(x.cpu().numpy().view(np.uint32), O.server_update(x0, ref, 0.1).view(np.uint32))
            assert bits.cpu().numpy().tolist() == [O.message_bits_rtn(B, m["level"], d) for m in want]
