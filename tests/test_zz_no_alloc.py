"""mlmc_compress_bits_static (the entry point that allocates nothing: its scratch is a device array inside the
library) against mlmc_compress_bits, through the C ABI, bit for bit, on two calls in a row, the second one with a
smaller input; and the limit of the static scratch."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from gpu_util import to_device


def test_static_scratch_limit_is_checked_on_the_host():
    """A plan whose workspace exceeds the static array is refused before anything touches a GPU."""
    big = P.Plan(P.MLMC_BITS, 512, 1000, P.MLMC_F32, [0, 1, 2, 4, 8, 16], P.mlmc_geometric_p(5), allocate=False)
    assert big.workspace_bytes > P.MLMC_STATIC_SCRATCH_BYTES
    rc = P.lib().mlmc_compress_bits_static(big.handle, None, 1000, 0, 0, None, None, None, None, None)
    assert rc == P.MLMC_ELIMIT
    topk = P.Plan(P.MLMC_TOPK, 2, 1000, P.MLMC_F32, [10, 100, 1000], None, allocate=False)
    assert P.lib().mlmc_compress_bits_static(topk.handle, None, 1000, 0, 0, None, None, None, None, None) == P.binding.MLMC_EINVAL


@pytest.mark.gpu
def test_static_scratch_matches_workspace_variant_twice():
    torch.cuda.set_device(0)
    cases = [(8, 5 * 4096 + 77, [0, 1, 2, 4, 8, 16], 3), (3, 1000, [2, 3, 8, 12], 4)]   # the second input is smaller
    for M, d, F, step in cases:
        print(f"static scratch: M={M} d={d} F={F}", flush=True)
        w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=M)
        G = W.generate(w)
        G[M - 1] *= np.float32(1e-3)   # rows with different scales
        g = to_device(G)
        p = P.mlmc_geometric_p(len(F) - 1)
        plan = P.Plan(P.MLMC_BITS, M, d, P.MLMC_F32, F, p)
        assert plan.workspace_bytes <= P.MLMC_STATIC_SCRATCH_BYTES
        ref = P.mlmc_compress_bits(plan, g, seed=9, step=step)
        torch.cuda.synchronize()
        assert plan.status() == 0
        got = P.BitsMessage(plan)
        got.level.fill_(-1)
        got.scale_exp.fill_(12345)
        status = torch.full((1,), 77, dtype=torch.int32, device="cuda:0")
        before = torch.cuda.memory_allocated()
        P.mlmc_compress_bits_static(plan, g, seed=9, step=step, out=got, dev_status=status)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert int(status.item()) == 0
        assert torch.equal(got.level, ref.level) and torch.equal(got.scale_exp, ref.scale_exp)
        assert torch.equal(got.planes, ref.planes)
        assert len(set(ref.level.cpu().tolist())) >= 1 and int(ref.planes.ne(0).sum()) > 0
