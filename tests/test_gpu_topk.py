"""GPU parity of the Top-k MLMC path against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import mlmc_workloads as W
import paper_2507_05508_amd as P
from oracle import mlmc as O
from gpu_util import check_topk_against_oracle, to_device, u32

pytestmark = pytest.mark.gpu


def _plan_for(w, p_fixed):
    return P.Plan(P.MLMC_TOPK, w.M, w.d, P.MLMC_BF16 if w.dtype == "bf16" else P.MLMC_F32, w.ladder, p_fixed)


@pytest.mark.parametrize("d", [65536, 5 * 4096 + 123, 1000])
def test_fixed_p_tiny_workload(d):
    w = W.scaled(W.WORKLOADS["tiny_topk"], d=d)
    G = W.generate(w)
    p = O.geometric_p(w.L)
    plan = _plan_for(w, p)
    g = to_device(G)
    seen = set()
    for step in range(100 if d == 65536 else 12):   # the tiny workload as configured: all of its 100 steps
        if step % 10 == 0:
            print(f"tiny_topk d={d} step={step}", flush=True)
        msg = P.mlmc_compress_topk(plan, g, seed=0, step=step)
        want = check_topk_against_oracle(plan, G, 0, step, msg, adaptive=False)
        assert plan.status() == 0
        seen |= {m["level"] for m in want}
        out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
        torch.cuda.synchronize()
        ref = O.aggregate_sparse(want, w.d, 1.0 / w.M)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    assert len(seen) >= 3


@pytest.mark.parametrize("name,d,M", [("resnet18_topk", 3 * 65536 + 4096 + 77, 3), ("resnet50_adaptive_topk", 300_001, 2)])
def test_fixed_p_segmented(name, d, M):
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    G = W.generate(w)
    p = O.geometric_p(w.L)
    plan = _plan_for(w, p)
    g = to_device(G)
    for step in (0, 1, 2, 7, 100, 2 ** 40 + 5):
        print(f"{name} fixed d={d} step={step}", flush=True)
        msg = P.mlmc_compress_topk(plan, g, seed=1234567890123, step=step)
        want = check_topk_against_oracle(plan, G, 1234567890123, step, msg, adaptive=False)
        assert plan.status() == 0
        for use_tile in (True, False):
            out = P.mlmc_aggregate(plan, msg, 0.5, use_tile_off=use_tile)
            torch.cuda.synchronize()
            ref = O.aggregate_sparse(want, w.d, 0.5)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("name,d,M", [("resnet50_adaptive_topk", 5 * 65536 + 999, 3), ("resnet18_topk", 70_000, 2),
                                       ("tiny_topk", 20_000, 2)])
def test_adaptive_norms_and_compress(name, d, M):
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    G = W.generate(w)
    plan = _plan_for(w, None)
    g = to_device(G)
    print(f"{name} adaptive norms d={d}", flush=True)
    norms = P.mlmc_level_norms(plan, g)
    torch.cuda.synchronize()
    assert plan.status() == 0
    got = norms.cpu().numpy()
    for i in range(M):
        want, _ = O.level_norms_row(G[i], w.ladder)
        assert np.array_equal(got[i].view(np.uint64), np.array(want, dtype=np.float64).view(np.uint64)), (i, got[i], want)
    for step in range(6):
        print(f"{name} adaptive compress d={d} step={step}", flush=True)
        msg = P.mlmc_compress_topk(plan, g, seed=42, step=step)
        want = check_topk_against_oracle(plan, G, 42, step, msg, adaptive=True)
        assert plan.status() == 0
        assert np.array_equal(msg.norms.cpu().numpy().view(np.uint64), got.view(np.uint64))
        out = P.mlmc_aggregate(plan, msg, 1.0)
        torch.cuda.synchronize()
        ref = O.aggregate_sparse(want, w.d, 1.0)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    # caller-supplied norms / probabilities take the three-threshold path and give the same message
    msg2 = P.mlmc_compress_topk(plan, g, seed=42, step=3, p=norms, p_is_norms=True)
    check_topk_against_oracle(plan, G, 42, 3, msg2, adaptive=True)
    pt = torch.tensor([O.adaptive_p(list(got[i])) for i in range(M)], dtype=torch.float64, device=g.device)
    msg3 = P.mlmc_compress_topk(plan, g, seed=42, step=4, p=pt, p_is_norms=False)
    check_topk_against_oracle(plan, G, 42, 4, msg3, adaptive=True)


@pytest.mark.parametrize("shift", [1, 3, 6])
@pytest.mark.parametrize("name,d,M", [("resnet50_adaptive_topk", 9 * 65536 + 999, 3), ("tiny_topk", 150_000, 2),
                                       ("bert_adaptive_topk_bf16", 6 * 65536 + 4096 + 5, 2)])
def test_sampled_threshold_search_gives_the_same_message(name, d, M, shift):
    """Thresholds located from a histogram of one block in 2^shift, proven by exact counts (or redone exactly when
    the sample was too thin to bracket them): the message must not depend on the sampling."""
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    G = W.generate(w)
    g = to_device(G)
    redone = set()
    for pf in (None, O.geometric_p(w.L)):
        plan = _plan_for(w, pf)
        plan.set_sampling(shift)
        if pf is None:
            print(f"{name} sampled shift={shift} norms d={d}", flush=True)
            norms = P.mlmc_level_norms(plan, g).cpu().numpy()
            assert plan.status() == 0
            for i in range(M):
                want, _ = O.level_norms_row(G[i], w.ladder)
                assert np.array_equal(norms[i].view(np.uint64), np.array(want, dtype=np.float64).view(np.uint64)), (i, norms[i], want)
        for step in range(5):
            print(f"{name} sampled shift={shift} adaptive={pf is None} d={d} step={step}", flush=True)
            msg = P.mlmc_compress_topk(plan, g, seed=11, step=step)
            want = check_topk_against_oracle(plan, G, 11, step, msg, adaptive=pf is None)
            assert plan.status() == 0
            redone.add(bool(plan.status(informational=True) & P.MLMC_DEV_REDONE))
            out = P.mlmc_aggregate(plan, msg, 0.5)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, w.d, 0.5).view(np.uint32))
    print(f"{name} shift={shift}: exact redo seen {sorted(redone)}", flush=True)
    if shift <= 3:
        assert redone == {False}    # an eighth of the blocks is plenty: the zones must hold


@pytest.mark.parametrize("name,d,M", [("resnet50_adaptive_topk", 7 * 65536 + 4096 + 17, 3), ("tiny_topk", 90_000, 2)])
def test_message_from_second_read_equals_message_from_staged_lists(name, d, M):
    """Staging off: every row's message is written by the second read of the row; staging on: from the lists the
    selection read set aside (or, after a wrong level prediction, by the second read).  Same message either way."""
    w = W.scaled(W.WORKLOADS[name], d=d, M=M)
    G = W.generate(w)
    g = to_device(G)
    for pf in (None, O.geometric_p(w.L)):
        for staging in (False, True):
            plan = _plan_for(w, pf)
            plan.set_staging(staging)
            for step in range(8):
                print(f"{name} staging={staging} adaptive={pf is None} d={d} step={step}", flush=True)
                msg = P.mlmc_compress_topk(plan, g, seed=21, step=step)
                want = check_topk_against_oracle(plan, G, 21, step, msg, adaptive=pf is None)
                assert plan.status() == 0
                out = P.mlmc_aggregate(plan, msg, 1.0 / M)
                torch.cuda.synchronize()
                assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, w.d, 1.0 / M).view(np.uint32))


def test_message_kernels_side_by_side_or_in_turn():
    """The second read of unstaged rows runs on the plan's side stream beside the assembly from the staged lists
    (overlap on, the default) or after it on the caller's stream (off).  Same message either way, also on a stream
    other than the default one and with other work of the caller queued right behind the call."""
    w = W.scaled(W.WORKLOADS["resnet50_adaptive_topk"], d=9 * 65536 + 4096 + 33, M=5)
    G = W.generate(w)
    g = to_device(G)
    side = torch.cuda.Stream()
    for overlap in (True, False):
        plan = _plan_for(w, None)
        plan.set_overlap(overlap)
        for step in range(10):
            print(f"overlap={overlap} step={step}", flush=True)
            if step % 2:
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    msg = P.mlmc_compress_topk(plan, g, seed=5, step=step)
                    out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)   # reads the message right behind the join
                torch.cuda.current_stream().wait_stream(side)
            else:
                msg = P.mlmc_compress_topk(plan, g, seed=5, step=step)
                out = P.mlmc_aggregate(plan, msg, 1.0 / w.M)
            want = check_topk_against_oracle(plan, G, 5, step, msg, adaptive=True)
            assert plan.status() == 0
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, w.d, 1.0 / w.M).view(np.uint32))


@pytest.mark.parametrize("shift", [0, 2])
def test_adversarial_rows_ties_zeros_denormals(shift):
    d = 3 * 4096 + 517
    rows = W.adversarial_rows(d)
    G = np.stack(rows)
    M = G.shape[0]
    ladder = [5, 100, 101, 1000, 4096, 9000, d - 1, d]
    L = len(ladder) - 1
    g = to_device(G)
    plan_a = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_F32, ladder, None)
    plan_a.set_sampling(shift)
    print("adversarial norms", flush=True)
    norms = P.mlmc_level_norms(plan_a, g).cpu().numpy()
    for i in range(M):
        want, _ = O.level_norms_row(G[i], ladder)
        assert np.array_equal(norms[i].view(np.uint64), np.array(want).view(np.uint64)), (i, norms[i], want)
    plan_f = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_F32, ladder, O.geometric_p(L))
    plan_f.set_sampling(shift)
    for step in range(10):
        print(f"adversarial step={step}", flush=True)
        msg = P.mlmc_compress_topk(plan_f, g, seed=9, step=step)
        check_topk_against_oracle(plan_f, G, 9, step, msg, adaptive=False)
        assert plan_f.status() == 0
        msg = P.mlmc_compress_topk(plan_a, g, seed=9, step=step)
        want = check_topk_against_oracle(plan_a, G, 9, step, msg, adaptive=True)
        assert plan_a.status() == 0
        out = P.mlmc_aggregate(plan_a, msg, 0.125)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, d, 0.125).view(np.uint32))


def _tie_rows(d, M, n_above, n_tie, bf16, seed):
    """Rows with n_above entries larger than one value, n_tie entries equal to it in magnitude (random signs, random
    places), the rest smaller: a rank threshold inside the tie block is decided by the index alone."""
    rng = np.random.default_rng(seed)
    rows = []
    for i in range(M):
        perm = rng.permutation(d)
        x = np.empty(d, np.float32)
        x[perm[:n_above]] = (2.0 + rng.random(n_above)).astype(np.float32)
        x[perm[n_above:n_above + n_tie]] = np.float32(0.375)
        x[perm[n_above + n_tie:]] = (0.25 * rng.random(d - n_above - n_tie)).astype(np.float32)
        x *= rng.choice(np.array([-1.0, 1.0], np.float32), d)
        rows.append(x)
    G = np.stack(rows)
    if bf16:   # every value above is a bf16 number after truncation of the random parts; the tie value is one exactly
        G = (G.view(np.uint32) >> 16).astype(np.uint16)
    return G


@pytest.mark.parametrize("bf16", [False, True])
def test_one_key_holds_the_threshold_massive_ties(bf16):
    """A threshold whose key is shared by far more entries than a workgroup can rank: the index cut is found from the
    per-chunk counts of the tie block and the one chunk that holds it.  Cases: the cut inside a chunk (first, middle,
    ragged last chunk), the threshold being the last of its key, two thresholds inside the same key."""
    d, M = 6 * 65536 + 3 * 4096 + 77, 3
    n_above, n_tie = d // 5, (3 * d) // 5
    G = _tie_rows(d, M, n_above, n_tie, bf16, 11)
    g = to_device(G)
    dt = P.MLMC_BF16 if bf16 else P.MLMC_F32
    ladders = [[100, n_above + 5, d],                    # the cut right after the block's first entries
               [100, n_above + n_tie // 2, d],           # in the middle
               [100, n_above + n_tie - 3, d],            # near its end
               [100, n_above + n_tie, d],                # the last of its key: every equal entry is inside
               [n_above + 1000, n_above + n_tie // 3, n_above + n_tie - 1000, d]]   # several thresholds in one key
    for ladder in ladders:
        L = len(ladder) - 1
        for pf in (None, O.geometric_p(L)):
            plan = P.Plan(P.MLMC_TOPK, M, d, dt, ladder, pf)
            if pf is None:
                norms = P.mlmc_level_norms(plan, g).cpu().numpy()
                for i in range(M):
                    want, _ = O.level_norms_row(G[i], ladder)
                    assert np.array_equal(norms[i].view(np.uint64), np.array(want).view(np.uint64)), (ladder, i)
            for step in range(4):
                print(f"massive ties bf16={bf16} ladder={ladder} adaptive={pf is None} step={step}", flush=True)
                msg = P.mlmc_compress_topk(plan, g, seed=3, step=step)
                check_topk_against_oracle(plan, G, 3, step, msg, adaptive=pf is None)
                assert plan.status() == 0


@pytest.mark.parametrize("ld_pad", [1, 2, 3, 8])
def test_padded_and_misaligned_rows(ld_pad):
    w = W.scaled(W.WORKLOADS["resnet18_topk"], d=2 * 4096 + 1001, M=3)
    G = W.generate(w)
    g = to_device(G, ld=w.d + ld_pad)
    plan = _plan_for(w, None)
    for step in range(3):
        print(f"padded ld=d+{ld_pad} step={step}", flush=True)
        msg = P.mlmc_compress_topk(plan, g, seed=5, step=step)
        check_topk_against_oracle(plan, G, 5, step, msg, adaptive=True)
        assert plan.status() == 0


def test_bf16_rows():
    w = W.scaled(W.WORKLOADS["bert_adaptive_topk_bf16"], d=4 * 65536 + 4096 * 3 + 5, M=2)
    G = W.generate(w)
    assert G.dtype == np.uint16
    g = to_device(G)
    plan = _plan_for(w, None)
    print("bf16 norms", flush=True)
    norms = P.mlmc_level_norms(plan, g).cpu().numpy()
    for i in range(w.M):
        want, _ = O.level_norms_row(G[i], w.ladder)
        assert np.array_equal(norms[i].view(np.uint64), np.array(want).view(np.uint64))
    for step in range(6):
        print(f"bf16 step={step}", flush=True)
        msg = P.mlmc_compress_topk(plan, g, seed=77, step=step)
        check_topk_against_oracle(plan, G, 77, step, msg, adaptive=True)
        assert plan.status() == 0
    g2 = to_device(G, ld=w.d + 3)
    msg = P.mlmc_compress_topk(plan, g2, seed=77, step=1)
    check_topk_against_oracle(plan, G, 77, 1, msg, adaptive=True)


@pytest.mark.parametrize("d,ladder", [(1, [0, 1]), (5, [0, 2, 5]), (64, [0, 1, 2, 3, 64]), (4097, [0, 4097]),
                                       (9000, [10, 20, 8000]), (4096, [4095, 4096])])
def test_degenerate_shapes(d, ladder):
    rng = np.random.default_rng(d)
    G = rng.standard_normal((2, d)).astype(np.float32)
    L = len(ladder) - 1
    g = to_device(G)
    for pf in (O.geometric_p(L), None):
        plan = P.Plan(P.MLMC_TOPK, 2, d, P.MLMC_F32, ladder, pf)
        for step in range(4):
            print(f"degenerate d={d} ladder={ladder} adaptive={pf is None} step={step}", flush=True)
            msg = P.mlmc_compress_topk(plan, g, seed=3, step=step)
            want = check_topk_against_oracle(plan, G, 3, step, msg, adaptive=pf is None)
            assert plan.status() == 0
            out = P.mlmc_aggregate(plan, msg, 0.5)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, d, 0.5).view(np.uint32))


def test_many_levels_many_rows():
    """The limits of the plan: L = 32 levels (33 thresholds, most of them crowded into a few buckets) and more rows
    than any other test, sampled and exact threshold search, adaptive and fixed p."""
    rng = np.random.default_rng(7)
    M, d, L = 37, 3 * 16384 + 811, 32
    G = (rng.standard_normal((M, d)) * np.exp(rng.uniform(-6, 2, size=(M, 1)))).astype(np.float32)
    ladder = [3] + [10 + 37 * l + (l * l * l) // 2 for l in range(1, L)] + [d]
    assert all(a < b for a, b in zip(ladder, ladder[1:]))
    g = to_device(G)
    for pf in (None, O.geometric_p(L)):
        for shift in (0, 2):
            plan = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_F32, ladder, pf)
            plan.set_sampling(shift)
            for step in range(3):
                print(f"L=32 M={M} adaptive={pf is None} shift={shift} step={step}", flush=True)
                msg = P.mlmc_compress_topk(plan, g, seed=5, step=step)
                want = check_topk_against_oracle(plan, G, 5, step, msg, adaptive=pf is None)
                assert plan.status() == 0
                out = P.mlmc_aggregate(plan, msg, 1.0 / M)
                torch.cuda.synchronize()
                assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, d, 1.0 / M).view(np.uint32))


@pytest.mark.parametrize("M", [70, 300])
def test_more_rows_than_a_wave_or_a_workgroup(M):
    """Row counts beyond 64 and beyond 256: the per-row loops that lanes or threads share (message starts, the order in
    which the message kernels take the rows, the aggregate's row table) wrap around."""
    rng = np.random.default_rng(M)
    d = 16384 + 77
    G = (rng.standard_normal((M, d)) * np.exp(rng.uniform(-3, 3, size=(M, 1)))).astype(np.float32)
    ladder = [5, 40, 300, 2000, d // 2, d]
    L = len(ladder) - 1
    g = to_device(G)
    for pf in (None, O.geometric_p(L)):
        plan = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_F32, ladder, pf)
        for step in range(2):
            print(f"rows M={M} adaptive={pf is None} step={step}", flush=True)
            msg = P.mlmc_compress_topk(plan, g, seed=11, step=step)
            want = check_topk_against_oracle(plan, G, 11, step, msg, adaptive=pf is None)
            assert plan.status() == 0
            out = P.mlmc_aggregate(plan, msg, 1.0 / M)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, d, 1.0 / M).view(np.uint32))


@pytest.mark.parametrize("seed", [1, 2])
def test_random_plans_and_inputs(seed):
    """Randomised valid calls (row counts, lengths from 1 to 120 000, ladders, fp32 / bf16, padded rows, value
    families with zeros, massive ties and heavy tails, sampled and exact threshold search, staging on and off)
    against the oracle, bit for bit, aggregate included."""
    rng = np.random.default_rng(seed)
    for case in range(30):
        M = int(rng.choice([1, 2, 3, 5, 9]))
        d = int(rng.choice([rng.integers(1, 200), rng.integers(200, 20000), rng.integers(20000, 120000)]))
        ladder = np.sort(rng.choice(np.arange(0, d + 1), size=min(int(rng.integers(2, 12)), d + 1), replace=False)).tolist()
        if rng.random() < 0.5:
            ladder[-1] = d
        L = len(ladder) - 1
        kind = int(rng.integers(0, 4))
        if kind == 0:
            G = rng.standard_normal((M, d)).astype(np.float32)
        elif kind == 1:
            G = (rng.standard_normal((M, d)) * np.exp(rng.uniform(-20, 10, size=(M, 1)))).astype(np.float32)
            G[rng.random((M, d)) < 0.5] = 0.0
        elif kind == 2:
            G = rng.integers(-3, 4, size=(M, d)).astype(np.float32)
        else:
            G = (rng.standard_t(2, size=(M, d)) * np.exp(rng.uniform(-8, 2, size=(1, d)))).astype(np.float32)
        bf16 = rng.random() < 0.3
        if bf16:
            Gb = (G.view(np.uint32) >> 16).astype(np.uint16)
            G = (Gb.astype(np.uint32) << 16).view(np.float32)
            g = to_device(Gb)
        else:
            g = to_device(G, ld=d + int(rng.integers(1, 4)) if rng.random() < 0.3 else None)
        adaptive = rng.random() < 0.5
        plan = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_BF16 if bf16 else P.MLMC_F32, ladder, None if adaptive else O.geometric_p(L))
        shift = int(rng.choice([0, 0, 1, 2, 4]))
        plan.set_sampling(shift)
        staging = rng.random() >= 0.25
        plan.set_staging(staging)
        call_seed = int(rng.integers(0, 2**40))
        for step in range(2):
            print(f"random case {case}: M={M} d={d} ladder={ladder} kind={kind} bf16={bf16} adaptive={adaptive} "
                  f"shift={shift} staging={staging} step={step}", flush=True)
            msg = P.mlmc_compress_topk(plan, g, seed=call_seed, step=step)
            want = check_topk_against_oracle(plan, G, call_seed, step, msg, adaptive=adaptive)
            assert plan.status() == 0
            out = P.mlmc_aggregate(plan, msg, 0.5)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy().view(np.uint32), O.aggregate_sparse(want, d, 0.5).view(np.uint32))


def test_identity_ladder_is_dense_mean():
    """L = 1, k_0 = 0, k_1 = d, p = 1: the message is the gradient and the aggregate is Alg. 1's mean."""
    rng = np.random.default_rng(0)
    M, d = 4, 10_000
    G = rng.standard_normal((M, d)).astype(np.float32)
    plan = P.Plan(P.MLMC_TOPK, M, d, P.MLMC_F32, [0, d], [1.0])
    g = to_device(G)
    msg = P.mlmc_compress_topk(plan, g, seed=0, step=0)
    out = P.mlmc_aggregate(plan, msg, 0.25).cpu().numpy()
    acc = np.zeros(d, dtype=np.float32)
    for i in range(M):
        acc = acc + G[i]
    assert np.array_equal(out, acc * np.float32(0.25))


def test_capacity_and_nonfinite_flags():
    w = W.scaled(W.WORKLOADS["resnet18_topk"], d=20_000, M=2)
    G = W.generate(w)
    plan = _plan_for(w, O.geometric_p(w.L))
    g = to_device(G)
    small = P.SparseMessage(plan, capacity=10)
    guard = torch.full_like(small.idx, -1)
    P.mlmc_compress_topk(plan, g, seed=0, step=0, out=small)
    assert plan.status() & P.MLMC_DEV_CAPACITY
    want = O.compress_topk(G, w.ladder, plan.p_fixed, 0, 0)
    assert np.array_equal(u32(small.idx)[:10], want[0]["idx"][:10])   # what fits is still correct
    for use_tile in (True, False):   # the aggregate must not follow the offsets past what the buffers hold
        out = P.mlmc_aggregate(plan, small, 1.0, use_tile_off=use_tile)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all())
    G2 = G.copy()
    G2[1, 17] = np.inf
    G2[0, 5] = np.nan
    g2 = to_device(G2)
    msg = P.mlmc_compress_topk(plan, g2, seed=0, step=1)
    assert plan.status() & P.MLMC_DEV_NONFINITE
    want = O.compress_topk(G2, w.ladder, plan.p_fixed, 0, 1)
    off = 0
    for i in range(2):
        n = len(want[i]["idx"])
        assert np.array_equal(u32(msg.idx)[off:off + n], want[i]["idx"])   # ordered by bit pattern
        off += n
