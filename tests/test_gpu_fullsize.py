"""Parity at the full BASELINE sizes, in the launch configuration bench.py times: every row of every full-size
workload is compared with the CPU oracle element by element (levels, norms, indices, values, offsets), and the dense
update with the oracle's aggregate of its own messages.  The oracle runs in worker processes, one row per task."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from oracle_pool import OracleTopkRows

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]


def _upload(G):
    if G.dtype == np.uint16:
        return torch.from_numpy(G.view(np.int16)).to("cuda:0").view(torch.bfloat16)
    return torch.from_numpy(G).to("cuda:0")


def _compare_with_oracle(tag, w, plan, msg, out, want_rows, alpha):
    """One compress + aggregate call against the oracle's messages of all rows (bit for bit)."""
    level = msg.level.cpu().numpy()
    row_off = msg.row_off.cpu().numpy()
    idx = msg.idx.cpu().numpy().view(np.uint32)
    val = msg.val.cpu().numpy().view(np.uint32)
    norms = msg.norms.cpu().numpy() if w.adaptive else None
    tile_off = msg.tile_off.cpu().numpy().view(np.uint32)
    off = 0
    for i in range(w.M):
        m = want_rows[i]
        assert level[i] == m["level"], (tag, i, level[i], m["level"])
        if w.adaptive:
            assert np.array_equal(norms[i].view(np.uint64), np.array(m["norms"], dtype=np.float64).view(np.uint64)), (tag, i)
        n = len(m["idx"])
        assert n == w.ladder[0] + w.ladder[m["level"]] - w.ladder[m["level"] - 1]
        assert row_off[i] == off, (tag, i)
        assert np.array_equal(idx[off:off + n], m["idx"]), f"{tag} row {i}: indices differ"
        assert np.array_equal(val[off:off + n], m["val"].view(np.uint32)), f"{tag} row {i}: values differ"
        bounds = np.searchsorted(m["idx"], np.arange(plan.num_tiles + 1, dtype=np.int64) * P.MLMC_TILE, side="left")
        assert np.array_equal(tile_off[i], bounds.astype(np.uint32)), f"{tag} row {i}: tile offsets differ"
        off += n
    assert row_off[w.M] == off
    ref = O.aggregate_sparse([want_rows[i] for i in range(w.M)], w.d, alpha)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), f"{tag}: dense update differs"


# steps: one ordinary step, and one in which (by the oracle's own draw) some row draws level 1 and some row level L
@pytest.mark.parametrize("name,steps", [("resnet50_adaptive_topk", (3, 15)), ("resnet18_topk", (3, 266))])
def test_topk_full_size(name, steps):
    w = W.WORKLOADS[name]
    pf = None if w.adaptive else O.geometric_p(w.L)
    print(f"{name}: oracle on all {w.M} rows, steps {steps} (worker processes)", flush=True)
    pool = OracleTopkRows(name, w.seed, steps, p_fixed=pf)
    print(f"{name}: generating the rows", flush=True)
    g = _upload(W.generate(w))
    want = pool.result()
    drawn = {want[i][s]["level"] for i in range(w.M) for s in range(len(steps))}
    assert 1 in drawn and w.L in drawn, drawn      # the narrowest and the widest band both reach full size
    plan = P.Plan(P.MLMC_TOPK, w.M, w.d, P.MLMC_F32, w.ladder, pf)
    msg = P.SparseMessage(plan, with_norms=w.adaptive)
    alpha = 1.0 / w.M
    for si, step in enumerate(steps):
        for staging in (True, False):
            tag = f"{name} step {step} staging {'on' if staging else 'off'}"
            print(tag, flush=True)
            plan.set_staging(staging)
            msg.idx.fill_(-1)
            msg.val.fill_(float("nan"))
            P.mlmc_compress_topk(plan, g, seed=w.seed, step=step, out=msg)
            out = P.mlmc_aggregate(plan, msg, alpha)
            torch.cuda.synchronize()
            assert plan.status() == 0
            _compare_with_oracle(tag, w, plan, msg, out, {i: want[i][si] for i in range(w.M)}, alpha)


def test_topk_largest_chunk():
    """A shape whose plan takes the largest chunk (2^18 elements per workgroup of the selection read: the widest LDS
    bitmap of the message kernel, eight count chunks per thread in the planner), every row against the oracle."""
    name, d, M, step = "resnet50_adaptive_topk", 46_000_000, 16, 1
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    pool = OracleTopkRows(name, w.seed, (step,), d=d, M=M)
    print("largest chunk: generating the rows", flush=True)
    g = _upload(W.generate(w))
    plan = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_F32, w.ladder, None)
    assert plan.chunk == 1 << 18
    want = pool.result()
    msg = P.SparseMessage(plan, with_norms=True)
    for staging in (True, False):
        print(f"largest chunk: staging {staging}", flush=True)
        plan.set_staging(staging)
        P.mlmc_compress_topk(plan, g, seed=w.seed, step=step, out=msg)
        out = P.mlmc_aggregate(plan, msg, 1.0 / M)
        torch.cuda.synchronize()
        assert plan.status() == 0
        _compare_with_oracle(f"largest chunk staging {staging}", w, plan, msg, out, {i: want[i][0] for i in range(M)}, 1.0 / M)


def test_stopk_full_size():
    """s-segmented Top-k at s = 0.001 n: 1000 levels, every row against the oracle (one step)."""
    w = W.WORKLOADS["resnet18_stopk"]
    pool = OracleTopkRows(w.name, w.seed, (2,))
    g = _upload(W.generate(w))
    want = pool.result()
    plan = P.Plan(P.MLMC_STOPK, w.M, w.d, P.MLMC_F32, [w.extra["s"]], None)
    assert tuple(plan.ladder) == w.ladder
    msg = P.SparseMessage(plan, with_norms=True)
    P.mlmc_compress_topk(plan, g, seed=w.seed, step=2, out=msg)
    out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
    torch.cuda.synchronize()
    assert plan.status() == 0
    _compare_with_oracle("stopk step 2", w, plan, msg, out, {i: want[i][0] for i in range(w.M)}, 1.0 / w.M)


def test_bits_full_size():
    w = W.WORKLOADS["resnet18_bits"]
    G = W.generate(w)
    g = _upload(G)
    p = O.geometric_p(w.L)
    plan = P.Plan(P.MLMC_BITS, w.M, w.d, P.MLMC_F32, w.ladder, p)
    for step in (0, 1):
        print(f"bits full size step {step}", flush=True)
        msg = P.mlmc_compress_bits(plan, g, seed=w.seed, step=step)
        out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
        torch.cuda.synchronize()
        assert plan.status() == 0
        want = O.compress_bits(G, w.ladder, p, w.seed, step)
        planes = msg.planes.cpu().numpy().view(np.uint64)
        for i in range(w.M):
            assert int(msg.level[i]) == want[i]["level"] and int(msg.scale_exp[i]) == want[i]["scale_exp"]
            n = want[i]["planes"].shape[0]
            assert np.array_equal(planes[i, :n], want[i]["planes"])
        ref = O.aggregate_bits(want, w.ladder, w.d, 1.0 / w.M)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_vbits_full_size():
    w = W.WORKLOADS["resnet18_vbits"]
    G = W.generate(w)
    g = _upload(G)
    p = O.geometric_p(w.L)
    plan = P.Plan(P.MLMC_VBITS, w.M, w.d, P.MLMC_F32, w.ladder, p)
    for step in (0, 1):
        print(f"largest-entry fixed point full size step {step}", flush=True)
        msg = P.mlmc_compress_bits(plan, g, seed=w.seed, step=step)
        out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
        torch.cuda.synchronize()
        assert plan.status() == 0
        want = O.compress_vbits(G, w.ladder, p, w.seed, step)
        planes = msg.planes.cpu().numpy().view(np.uint64)
        vbits = msg.scale_exp.cpu().numpy().view(np.uint32)
        for i in range(w.M):
            assert int(msg.level[i]) == want[i]["level"] and vbits[i] == np.float32(want[i]["vmax"]).view(np.uint32)
            n = want[i]["planes"].shape[0]
            assert np.array_equal(planes[i, :n], want[i]["planes"])
        ref = O.aggregate_vbits(want, w.ladder, w.d, 1.0 / w.M)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_rtn_full_size():
    w = W.WORKLOADS["resnet18_rtn"]
    G = W.generate(w)
    g = _upload(G)
    plan = P.Plan(P.MLMC_RTN, w.M, w.d, P.MLMC_F32, w.ladder, None)
    for step in (0, 1):
        print(f"Round-to-Nearest full size step {step}", flush=True)
        msg = P.mlmc_compress_rtn(plan, g, seed=w.seed, step=step)
        out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
        torch.cuda.synchronize()
        assert plan.status() == 0
        want = O.compress_rtn(G, w.ladder, None, w.seed, step)
        planes = msg.planes.cpu().numpy().view(np.uint64)
        scale = msg.scale_exp.cpu().numpy().view(np.uint32)
        norms = msg.norms.cpu().numpy()
        for i in range(w.M):
            assert np.array_equal(norms[i].view(np.uint64), np.array(want[i]["norms"], dtype=np.float64).view(np.uint64))
            assert int(msg.level[i]) == want[i]["level"]
            assert scale[i, 0] == np.float32(want[i]["c"]).view(np.uint32) and scale[i, 1] == np.float32(want[i]["coef"]).view(np.uint32)
            n = want[i]["planes"].shape[0]
            assert np.array_equal(planes[i, :n], want[i]["planes"])
        ref = O.aggregate_rtn(want, w.ladder, w.d, 1.0 / w.M)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_fbits_full_size():
    w = W.WORKLOADS["resnet18_fbits"]
    G = W.generate(w)
    g = _upload(G)
    p = O.geometric_p(w.L)
    plan = P.Plan(P.MLMC_FBITS, w.M, w.d, P.MLMC_F32, w.ladder, p)
    for step in (0, 1):
        print(f"floating-point bits full size step {step}", flush=True)
        msg = P.mlmc_compress_bits(plan, g, seed=w.seed, step=step)
        out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
        torch.cuda.synchronize()
        assert plan.status() == 0
        want = O.compress_fbits(G, w.ladder, p, w.seed, step)
        planes = msg.planes.cpu().numpy().view(np.uint64)
        for i in range(w.M):
            assert int(msg.level[i]) == want[i]["level"]
            n = want[i]["planes"].shape[0]
            assert np.array_equal(planes[i, :n], want[i]["planes"])
        ref = O.aggregate_fbits(want, w.ladder, w.d, 1.0 / w.M)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_topk_bf16_full_size():
    w = W.WORKLOADS["bert_adaptive_topk_bf16"]
    print("bert_adaptive_topk_bf16: oracle on all 4 rows of 1.2e8 entries (worker processes, a few minutes)", flush=True)
    pool = OracleTopkRows(w.name, 0, (0,), workers=4)
    print("bert_adaptive_topk_bf16: generating the rows", flush=True)
    g = _upload(W.generate(w))
    want = pool.result()
    plan = P.Plan(P.MLMC_TOPK, w.M, w.d, P.MLMC_BF16, w.ladder, None)
    msg = P.SparseMessage(plan, with_norms=True)
    P.mlmc_compress_topk(plan, g, seed=0, step=0, out=msg)
    out = P.mlmc_aggregate(plan, msg, 0.25)
    torch.cuda.synchronize()
    assert plan.status() == 0
    _compare_with_oracle("bf16 step 0", w, plan, msg, out, {i: want[i][0] for i in range(w.M)}, 0.25)
