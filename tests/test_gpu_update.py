"""GPU parity of the fused server update (Alg. 2 "Server updates") and of the per-worker message sizes against the
CPU oracle, for rank-band and bit-wise messages, bit for bit."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from gpu_util import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,d,M,adaptive", [("resnet50_adaptive_topk", 5 * 4096 + 123, 5, True), ("resnet18_topk", 70_001, 3, False),
                                                ("tiny_topk", 4096, 2, False)])
def test_topk_server_update_and_message_bits(name, d, M, adaptive):
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    G = W.generate(w)
    p = None if adaptive else O.geometric_p(w.L)
    plan = P.Plan(P.MLMC_TOPK, w.M, w.d, P.MLMC_F32, w.ladder, p)
    g = to_device(G)
    rng = np.random.default_rng(3)
    x0 = rng.standard_normal(d).astype(np.float32)
    x_ref = x0.copy()
    x = torch.from_numpy(x0).to("cuda:0")
    alpha, eta = 1.0 / M, 0.0123
    for step in range(4):   # a few steps of Alg. 2 on the same gradients: the model carries over
        print(f"{name} update step {step}", flush=True)
        msg = P.mlmc_compress_topk(plan, g, seed=7, step=step)
        want = O.compress_topk(G, w.ladder, p, 7, step)
        gt = O.aggregate_sparse(want, d, alpha)
        x_ref = O.server_update(x_ref, gt, eta)
        out = torch.empty(d, dtype=torch.float32, device="cuda:0") if step % 2 == 0 else None   # with and without g~ written
        P.mlmc_aggregate_update(plan, msg, alpha, eta, x, out=out, use_tile_off=(step != 1))
        torch.cuda.synchronize()
        assert plan.status() == 0
        assert np.array_equal(x.cpu().numpy().view(np.uint32), x_ref.view(np.uint32))
        if out is not None:
            assert np.array_equal(out.cpu().numpy().view(np.uint32), gt.view(np.uint32))
        bits = P.mlmc_message_bits(plan, msg).cpu().numpy()
        assert bits.tolist() == [O.message_bits_topk(w.ladder, m["level"], d) for m in want]


@pytest.mark.parametrize("F", [[0, 1, 2, 4, 8, 16], [2, 3, 8, 12]])
def test_bits_server_update_and_message_bits(F):
    d, M = 3 * 4096 + 77, 4
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=M)
    G = W.generate(w)
    p = O.geometric_p(len(F) - 1)
    plan = P.Plan(P.MLMC_BITS, M, d, P.MLMC_F32, F, p)
    g = to_device(G)
    x_ref = np.linspace(-1, 1, d).astype(np.float32)
    x = torch.from_numpy(x_ref.copy()).to("cuda:0")
    for step in range(3):
        msg = P.mlmc_compress_bits(plan, g, seed=2, step=step)
        want = O.compress_bits(G, F, p, 2, step)
        gt = O.aggregate_bits(want, F, d, 0.25)
        x_ref = O.server_update(x_ref, gt, 0.5)
        out = torch.empty(d, dtype=torch.float32, device="cuda:0")
        P.mlmc_aggregate_update(plan, msg, 0.25, 0.5, x, out=out)
        torch.cuda.synchronize()
        assert np.array_equal(x.cpu().numpy().view(np.uint32), x_ref.view(np.uint32))
        assert np.array_equal(out.cpu().numpy().view(np.uint32), gt.view(np.uint32))
        bits = P.mlmc_message_bits(plan, msg).cpu().numpy()
        assert bits.tolist() == [O.message_bits_fixed_point(F, m["level"], d) for m in want]


def test_update_argument_checks():
    plan = P.Plan(P.MLMC_BITS, 2, 1000, P.MLMC_F32, [0, 1, 2], P.mlmc_geometric_p(2))
    msg = P.BitsMessage(plan)
    x = torch.zeros(1000, dtype=torch.float32, device="cuda:0")
    with pytest.raises(P.MlmcError):
        P.mlmc_aggregate_update(plan, msg, 1.0, 1.0, x, out=x)        # out must not alias x
    with pytest.raises(P.MlmcError):
        P.mlmc_aggregate_update(plan, msg, 1.0, 1.0, x[:500])         # wrong length
