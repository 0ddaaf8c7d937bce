"""GPU parity of the fixed-point bit-wise MLMC path and its aggregate against the CPU oracle."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _check_bits(plan, G, F, p, seed, step, msg):
    torch.cuda.synchronize()
    M, d = G.shape
    level = msg.level.cpu().numpy()
    sexp = msg.scale_exp.cpu().numpy()
    planes = msg.planes.cpu().numpy().view(np.uint64)
    want = O.compress_bits(G, F, p, seed, step)
    for i in range(M):
        assert level[i] == want[i]["level"] and sexp[i] == want[i]["scale_exp"], (i, level[i], sexp[i], want[i]["level"], want[i]["scale_exp"])
        n = want[i]["planes"].shape[0]
        assert np.array_equal(planes[i, :n], want[i]["planes"]), f"row {i}: planes differ"
    return want


@pytest.mark.parametrize("F", [[0, 1, 2, 4, 8, 16], [2, 3, 8, 12], [0, 24], list(range(17))])
@pytest.mark.parametrize("d", [3 * 4096 + 77, 64, 100_003])
def test_bits_compress_and_aggregate(F, d):
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=3)
    G = W.generate(w)
    L = len(F) - 1
    p = O.geometric_p(L)
    plan = P.Plan(P.MLMC_BITS, 3, d, P.MLMC_F32, F, p)
    g = to_device(G)
    for step in range(5):
        print(f"bits F={F} d={d} step={step}", flush=True)
        msg = P.mlmc_compress_bits(plan, g, seed=11, step=step)
        want = _check_bits(plan, G, F, p, 11, step, msg)
        assert plan.status() == 0
        out = P.mlmc_aggregate(plan, msg, 1.0 / 3)
        torch.cuda.synchronize()
        ref = O.aggregate_bits(want, F, d, 1.0 / 3)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_bits_adversarial_and_padded_rows():
    d = 2 * 4096 + 300
    G = np.stack(W.adversarial_rows(d))
    F = [0, 1, 2, 4, 8, 16]
    p = O.geometric_p(5)
    plan = P.Plan(P.MLMC_BITS, G.shape[0], d, P.MLMC_F32, F, p)
    for ld in (d, d + 1, d + 6):
        g = to_device(G, ld=ld)
        for step in range(3):
            print(f"bits adversarial ld={ld} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=2, step=step)
            want = _check_bits(plan, G, F, p, 2, step, msg)
            out = P.mlmc_aggregate(plan, msg, 1.0)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_bits(want, F, d, 1.0).view(np.uint32))


def test_bits_bf16_rows():
    w = W.scaled(W.WORKLOADS["bert_adaptive_topk_bf16"], d=50_000, M=2)
    G = W.generate(w)
    F = [0, 1, 2, 4, 8]
    p = O.geometric_p(4)
    plan = P.Plan(P.MLMC_BITS, 2, w.d, P.MLMC_BF16, F, p)
    g = to_device(G)
    for step in range(3):
        msg = P.mlmc_compress_bits(plan, g, seed=1, step=step)
        _check_bits(plan, G, F, p, 1, step, msg)


@pytest.mark.parametrize("seed", [3, 4])
def test_bits_random_plans_and_inputs(seed):
    """Randomised valid calls of the bit-wise path (row counts, lengths, bit ladders up to 24 bits, value families
    with zeros and very small or large scales, padded rows) against the oracle, bit for bit, aggregate included."""
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
            G = rng.integers(-5, 6, size=(M, d)).astype(np.float32)
            if M > 1:
                G[0] = 0.0   # an all-zero row
        p = O.geometric_p(L)
        plan = P.Plan(P.MLMC_BITS, M, d, P.MLMC_F32, F, p)
        if case % 2:
            plan.set_sampling(int(rng.integers(1, 5)))   # scale predicted from a sample of the blocks
        g = to_device(G, ld=d + int(rng.integers(1, 4)) if rng.random() < 0.3 else None)
        call_seed = int(rng.integers(0, 2**40))
        for step in range(2):
            print(f"bits random case {case}: M={M} d={d} F={F} kind={kind} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=call_seed, step=step)
            want = _check_bits(plan, G, F, p, call_seed, step, msg)
            assert plan.status() == 0
            out = P.mlmc_aggregate(plan, msg, 0.25)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_bits(want, F, d, 0.25).view(np.uint32))


@pytest.mark.parametrize("shift", [1, 2, 4])
def test_bits_sampled_scale_is_proven_or_redone(shift):
    """The row scale is predicted from a sample of the blocks and the message extracted under it in the one full
    read; rows whose true maximum needs a larger scale are extracted again.  Rows are built so that the maximum
    lies in a sampled block, in an unsampled block (larger exponent: redone), in an unsampled block with the same
    exponent (not redone), and in the ragged last block; the result never depends on the sampling."""
    S = 1 << shift
    d = 40 * 1024 + 333
    rng = np.random.default_rng(shift)
    G = (rng.standard_normal((6, d)) * 0.01).astype(np.float32)
    sampled_blk, unsampled_blk = (S >> 1) + S, (S >> 1) + S + 1
    G[0, sampled_blk * 1024 + 5] = 3.0                      # maximum inside the sample
    G[1, unsampled_blk * 1024 + 700] = -3.0                 # outside, several binades above the sample's maximum
    G[2, unsampled_blk * 1024 + 1] = np.abs(G[2]).max() * np.float32(1.01)   # outside, (almost surely) same binade
    G[3, d - 1] = 1e20                                      # last, partial block
    G[4] = 0.0
    G[4, unsampled_blk * 1024] = 1e-41                      # a denormal maximum outside the sample: scale exponent stays -125
    F = [0, 1, 2, 4, 8, 16]
    p = O.geometric_p(5)
    for Fl, pl in ((F, p), ([2, 3, 8, 12], O.geometric_p(3))):
        plan = P.Plan(P.MLMC_BITS, G.shape[0], d, P.MLMC_F32, Fl, pl)
        plan.set_sampling(shift)
        g = to_device(G)
        for step in range(4):
            print(f"bits sampled scale shift={shift} F={Fl} step={step}", flush=True)
            msg = P.mlmc_compress_bits(plan, g, seed=5, step=step)
            want = _check_bits(plan, G, Fl, pl, 5, step, msg)
            assert plan.status() == 0
            out = P.mlmc_aggregate(plan, msg, 0.5)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_bits(want, Fl, d, 0.5).view(np.uint32))


@pytest.mark.parametrize("kind", ["bits", "vbits", "fbits", "rtn"])
@pytest.mark.parametrize("d", [100_003, (1 << 21) + 3 * 4096 + 77])
def test_workspace_contents_on_entry_do_not_matter(kind, d):
    """The calls expect nothing in the workspace: with every byte of it set to 0xFF or 0x5A beforehand the message,
    the status word and the aggregate are those of a call on a workspace as allocated.  (The fixed-point kinds start
    with the maximum kernel, no clearing launch before it; the longer rows take the sampled maximum.)"""
    M = 3
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=M)
    G = W.generate(w)
    G[1] *= np.float32(1e-3)
    g = to_device(G)
    if kind == "rtn":
        plan = P.Plan(P.MLMC_RTN, M, d, P.MLMC_F32, [0, 2, 4, 8], None)
        compress = P.mlmc_compress_rtn
    else:
        F = [0, 1, 2, 4, 8, 16] if kind != "fbits" else [0, 1, 2, 4, 8, 16, 23]
        code = {"bits": P.MLMC_BITS, "vbits": P.MLMC_VBITS, "fbits": P.MLMC_FBITS}[kind]
        plan = P.Plan(code, M, d, P.MLMC_F32, F, O.geometric_p(len(F) - 1))
        compress = P.mlmc_compress_bits

    def run(step):
        msg = compress(plan, g, seed=21, step=step)
        out = P.mlmc_aggregate(plan, msg, 1.0 / M)
        torch.cuda.synchronize()
        got = [msg.level.cpu().numpy(), msg.scale_exp.cpu().numpy(), msg.planes.cpu().numpy(), out.cpu().numpy().view(np.uint32)]
        if msg.norms is not None:
            got.append(msg.norms.cpu().numpy().view(np.uint64))
        return got, plan.status(informational=True)

    for step in range(3):
        print(f"workspace {kind} d={d} step={step}", flush=True)
        want, want_status = run(step)
        for fill in (0xFF, 0x5A):
            plan.ws.fill_(fill)
            got, status = run(step)
            assert status == want_status
            for a, b in zip(got, want):
                assert np.array_equal(a, b), (kind, step, hex(fill))


@pytest.mark.parametrize("where", ["first", "middle", "last"])
def test_bits_one_long_row_every_workgroup_maximum_counts(where):
    """One worker and a row long enough that the maximum kernel runs with its largest grid (1024 workgroups for the
    row, each leaving its own maximum): the row's largest entry sits in the first block, in a middle one or in the
    ragged last one, and both fixed-point kinds (power-of-two scale from every block; largest entry itself) must find it."""
    d = 8192 * 1024 + 3 * 1024 + 77
    w = W.scaled(W.WORKLOADS["resnet18_bits"], d=d, M=1)
    G = W.generate(w)
    at = {"first": 3, "middle": 4099 * 1024 + 511, "last": d - 2}[where]
    G[0, at] = np.float32(-7.25) * np.abs(G[0]).max()
    g = to_device(G)
    F = [0, 1, 2, 4, 8, 16]
    p = O.geometric_p(5)
    print(f"long row, maximum in the {where} block: bits", flush=True)
    plan = P.Plan(P.MLMC_BITS, 1, d, P.MLMC_F32, F, p)
    plan.set_sampling(0)
    msg = P.mlmc_compress_bits(plan, g, seed=9, step=1)
    want = _check_bits(plan, G, F, p, 9, 1, msg)
    assert plan.status(informational=True) == 0   # every block was read: nothing to redo
    out = P.mlmc_aggregate(plan, msg, 1.0)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_bits(want, F, d, 1.0).view(np.uint32))
    print(f"long row, maximum in the {where} block: vbits", flush=True)
    planv = P.Plan(P.MLMC_VBITS, 1, d, P.MLMC_F32, F, p)
    msgv = P.mlmc_compress_bits(planv, g, seed=9, step=1)
    torch.cuda.synchronize()
    wantv = O.compress_vbits(G, F, p, 9, 1)
    assert int(msgv.level.cpu().numpy()[0]) == wantv[0]["level"]
    assert msgv.scale_exp.cpu().numpy().view(np.uint32)[0] == np.float32(wantv[0]["vmax"]).view(np.uint32)
    n = wantv[0]["planes"].shape[0]
    assert np.array_equal(msgv.planes.cpu().numpy().view(np.uint64)[0, :n], wantv[0]["planes"])
    assert planv.status() == 0
