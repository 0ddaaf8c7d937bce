#!/usr/bin/env python3
"""Benchmark of the MLMC compress + aggregate hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of M synthetic gradient rows that are already
resident in HBM: (adaptive: per-level norms +) level draw + compress + server aggregate.  The step index
changes every step, so different levels (hence different message sizes) are drawn.

Prints ONE JSON line: metric = GB/s of gradient input (M * d * sizeof(input) / step time), with
  roofline     -- the dominant kernel's algorithmic bytes per launch / its HIP-event duration vs 8 TB/s HBM
  cpu_baseline -- the CPU oracle timed on a bounded sample of the same workload (rows are independent)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import mlmc_workloads as W  # noqa: E402

HBM_PEAK_GBPS = 8000.0
DEFAULT_WORKLOAD = "resnet50_adaptive_topk"


def algorithmic_bytes(w, kernel, nnz_total, planes_bytes):
    """Bytes the method itself has to move in one launch of `kernel`: one read of what it consumes, one write of what it
    produces (no re-reads, no scratch lists)."""
    s_in = 2 if w.dtype == "bf16" else 4
    in_bytes = w.M * w.d * s_in
    if kernel in ("k_main", "k_bits_max", "k_bits_smax", "k_rtn_norms"):
        return in_bytes                                   # one read of every input element
    if kernel == "k_rs_scatter":
        return 16 * w.M * w.d                             # a sort pass: every {key, index} pair read and written
    if kernel == "k_rs_hist":
        return 8 * w.M * w.d
    if kernel == "k_write":
        return in_bytes + 8 * nnz_total                   # read the rows, write (idx, val)
    if kernel == "k_agg_sparse":
        return 8 * nnz_total + 4 * w.d                    # read the messages, write the dense update
    if kernel == "k_bits_extract":
        return in_bytes + planes_bytes
    if kernel == "k_agg_bits":
        return planes_bytes + 4 * w.d
    return 0


def kernel_sources_digest():
    """sha256 over the kernel sources and the C header: names the code a profile was taken from."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_05508_amd", "csrc")
    files = sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".h")))
    for path in files + [os.path.join(ROOT, "include", "mlmc.h")]:
        h.update(os.path.basename(path).encode() + b"\0")
        h.update(open(path, "rb").read())
    return h.hexdigest()


# kernels that the library times under one name (mlmc_profile_*) and the kernel trace lists under their own
_TRACE_NAME = {"k_main2": "k_main", "k_rtn_extract": "k_bits_extract", "k_sb_clear": "k_zero"}


def measured_traffic(workload, kernel):
    """(HBM bytes per launch of `kernel`, provenance) from the committed rocprofv3 summary of this workload
    (FETCH_SIZE + WRITE_SIZE, scaled as the summary says).  The summary names the digest of the kernel sources it
    was measured on; when the sources have changed since (or no summary covers the kernel) the bytes are None:
    a stale counter reading is not reported."""
    path = os.path.join(ROOT, "profiles", f"{workload}.txt")
    if not os.path.exists(path):
        return None, {"profile": None, "reason": "no summary for this workload"}
    digest_now, digest_prof, value = kernel_sources_digest(), None, None
    for line in open(path):
        f = line.split()
        if line.startswith("kernel sources sha256:"):
            digest_prof = f[-1]
        elif value is None and f and _TRACE_NAME.get(f[0].split("<")[0], f[0].split("<")[0]) == kernel and len(f) >= 3:   # first line of the kernel: its working launches
            try:
                value = int((float(f[-2]) + float(f[-1])) * 1e6)
            except ValueError:
                value = None
    prov = {"profile": f"profiles/{workload}.txt", "kernel_sources_sha256": digest_prof}
    if digest_prof != digest_now:
        prov["reason"] = "kernel sources changed since the profile was taken"
        return None, prov
    return value, prov


def _oracle_row(w, row_data, i):
    from oracle import mlmc as O
    p = None if w.adaptive else O.geometric_p(w.L)
    if w.kind in ("topk", "stopk"):
        return O.compress_topk_row(row_data, w.ladder, p, w.seed, 0, i)
    if w.kind == "fbits":
        return O.compress_fbits_row(row_data, w.ladder, p, w.seed, 0, i)
    if w.kind == "vbits":
        return O.compress_vbits_row(row_data, w.ladder, p, w.seed, 0, i)
    if w.kind == "rtn":
        return O.compress_rtn_row(row_data, w.ladder, p, w.seed, 0, i)
    return O.compress_bits_row(row_data, w.ladder, p, w.seed, 0, i)


def _oracle_aggregate(w, msgs):
    from oracle import mlmc as O
    if w.kind in ("topk", "stopk"):
        return O.aggregate_sparse(msgs, w.d, 1.0 / w.M)
    if w.kind == "fbits":
        return O.aggregate_fbits(msgs, w.ladder, w.d, 1.0 / w.M)
    if w.kind == "vbits":
        return O.aggregate_vbits(msgs, w.ladder, w.d, 1.0 / w.M)
    if w.kind == "rtn":
        return O.aggregate_rtn(msgs, w.ladder, w.d, 1.0 / w.M)
    return O.aggregate_bits(msgs, w.ladder, w.d, 1.0 / w.M)


def _cpu_child(w, G, rows, barrier, conn):
    """One process of the all-cores leg: waits until every process is ready, then compresses its rows."""
    try:
        barrier.wait()
        t0 = time.perf_counter()
        msgs = [_oracle_row(w, G[i], i) for i in rows]
        dt = time.perf_counter() - t0
        keep = ("level", "idx", "val", "scale_exp", "planes", "p_level")
        conn.send((dt, [{k: m[k] for k in keep if k in m} for m in msgs]))
    finally:
        conn.close()


def cpu_baseline(w, G, budget_s=25.0, max_cores=16):
    """The oracle as it stands on a bounded sample of the same workload, step 0: compress of every sampled row +
    the aggregate of their messages.  Two legs: one thread, and one worker row per task over the host cores
    (processes forked before anything touches the GPU; each times its own rows from a common start, the leg's time
    is the slowest process + the single-threaded aggregate).  Must be called before the GPU is initialised."""
    import multiprocessing as mp
    s_in = 2 if w.dtype == "bf16" else 4
    # leg 1: a single thread, first rows until about a third of the budget is spent
    t0 = time.perf_counter()
    msgs = []
    for i in range(w.M):
        msgs.append(_oracle_row(w, G[i], i))
        if time.perf_counter() - t0 > budget_s / 3 * 0.8:
            break
    rows1 = len(msgs)
    _oracle_aggregate(w, msgs)
    dt1 = time.perf_counter() - t0
    per_row = dt1 / rows1
    single = {"value": rows1 * w.d * s_in / dt1 / 1e9, "unit": "GB/s", "cores": 1,
              "sample": f"{rows1} of {w.M} rows of {w.name} (d={w.d}), step 0: compress + aggregate, {dt1:.1f} s"}
    del msgs
    # leg 2: rows over the cores; as many rows as fit the rest of the budget (a process slows down when all run)
    cores = max(1, min(max_cores, os.cpu_count() or 1, w.M))
    rounds = max(1, int((budget_s * 2 / 3) / (per_row * 1.6)))
    rows2 = min(w.M, cores * rounds)
    ctx = mp.get_context("fork")
    barrier = ctx.Barrier(cores + 1)
    procs, conns = [], []
    for c in range(cores):
        parent, child = ctx.Pipe(duplex=False)
        pr = ctx.Process(target=_cpu_child, args=(w, G, list(range(c, rows2, cores)), barrier, child))
        pr.start()
        child.close()
        procs.append(pr)
        conns.append(parent)
    barrier.wait()
    results = [c.recv() for c in conns]
    for pr in procs:
        pr.join()
    slowest = max(r[0] for r in results)
    by_row = {}
    for c, (_, ms) in enumerate(results):
        for k, m in enumerate(ms):
            by_row[c + k * cores] = m
    t2 = time.perf_counter()
    _oracle_aggregate(w, [by_row[i] for i in range(rows2)])
    dt2 = slowest + time.perf_counter() - t2
    return {"value": rows2 * w.d * s_in / dt2 / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{rows2} of {w.M} rows of {w.name} (d={w.d}), step 0, one row per task over {cores} processes: "
                      f"compress {slowest:.1f} s (slowest process) + aggregate, {dt2:.1f} s",
            "single_thread": single}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(W.WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-staging", action="store_true",
                    help="Top-k: write every message by a second read of the rows (tuning hook off; same results)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="Top-k: both message kernels on the caller's stream (tuning hook off; same results)")
    ap.add_argument("--fused-update", action="store_true",
                    help="server side as mlmc_aggregate_update: x <- x - eta * g~ inside the aggregate, g~ itself not written")
    ap.add_argument("--cpu-budget", type=float, default=25.0)
    ap.add_argument("--print-kernel-digest", action="store_true",
                    help="print the sha256 that names the kernel sources (profile summaries quote it) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (a known-size kernel to scale profiler byte counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (M workers are M rows on one MI355X); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.print_kernel_digest:
        print(kernel_sources_digest())
        return

    w = W.WORKLOADS[args.workload]
    t_gen = time.perf_counter()
    G = W.generate(w)
    print(f"[bench] generated {w.name}: M={w.M} d={w.d} {w.dtype} in {time.perf_counter() - t_gen:.1f} s", file=sys.stderr, flush=True)
    # the CPU baseline runs first: its worker processes are forked while this process holds no GPU state
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, G, args.cpu_budget)
        print(f"[bench] cpu baseline: {cpu['value']:.4f} GB/s on {cpu['cores']} cores, "
              f"{cpu['single_thread']['value']:.4f} GB/s on one", file=sys.stderr, flush=True)

    import torch
    import paper_2507_05508_amd as P
    dev = torch.device("cuda:0")
    if w.dtype == "bf16":
        g = torch.from_numpy(G.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        g = torch.from_numpy(G).to(dev)
    s_in = 2 if w.dtype == "bf16" else 4
    in_bytes = w.M * w.d * s_in
    alpha = 1.0 / w.M

    sparse = w.kind in ("topk", "stopk")
    if w.kind == "stopk":
        plan = P.Plan(P.MLMC_STOPK, w.M, w.d, P.MLMC_BF16 if w.dtype == "bf16" else P.MLMC_F32, [w.extra["s"]], None)
        msg = P.SparseMessage(plan, with_norms=True)
    elif w.kind == "topk":
        plan = P.Plan(P.MLMC_TOPK, w.M, w.d, P.MLMC_BF16 if w.dtype == "bf16" else P.MLMC_F32, w.ladder,
                      None if w.adaptive else P.mlmc_geometric_p(w.L))
        msg = P.SparseMessage(plan, with_norms=w.adaptive)
        if args.no_staging:
            plan.set_staging(False)
        if args.no_overlap:
            plan.set_overlap(False)
    else:
        kind = {"bits": P.MLMC_BITS, "fbits": P.MLMC_FBITS, "vbits": P.MLMC_VBITS, "rtn": P.MLMC_RTN}[w.kind]
        plan = P.Plan(kind, w.M, w.d, P.MLMC_F32, w.ladder, None if w.adaptive else P.mlmc_geometric_p(w.L))
        msg = P.BitsMessage(plan)
    out = torch.empty(w.d, dtype=torch.float32, device=dev)
    x_model = torch.zeros(w.d, dtype=torch.float32, device=dev) if args.fused_update else None

    def step(i):
        if sparse:
            P.mlmc_compress_topk(plan, g, seed=w.seed, step=i, out=msg)
        else:
            (P.mlmc_compress_rtn if w.kind == "rtn" else P.mlmc_compress_bits)(plan, g, seed=w.seed, step=i, out=msg)
        if args.fused_update:
            P.mlmc_aggregate_update(plan, msg, alpha, 0.01, x_model)
        else:
            P.mlmc_aggregate(plan, msg, alpha, out=out)

    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    assert plan.status() == 0, f"device status {plan.status()}"

    # timed region: K steps, whole-job wall clock between two synchronisations
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    redone = bool(plan.status(informational=True) & P.MLMC_DEV_REDONE)   # of the last step
    ms_per_step = dt * 1e3 / args.steps
    assert plan.status() == 0, f"device status {plan.status()}"

    # same K steps again with a HIP-event pair around every kernel (on the launch stream)
    nnz_total, planes_bytes = 0, 0
    drawn = {}   # drawn level -> rows that drew it over the timed steps (the message size, hence the bytes, depends on it)
    P.mlmc_profile_reset()
    P.mlmc_profile_enable(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    dt_ev = time.perf_counter() - t1
    P.mlmc_profile_enable(False)
    prof = P.mlmc_profile_get()
    # message sizes of those steps (needed for the algorithmic bytes): replay the draws, cheap
    for i in range(args.steps):
        if sparse:
            P.mlmc_compress_topk(plan, g, seed=w.seed, step=args.warmup + i, out=msg)
            nnz_total += int(msg.row_off[-1].item())
            for l in msg.level.cpu().numpy().tolist():
                drawn[l] = drawn.get(l, 0) + 1
        else:
            (P.mlmc_compress_rtn if w.kind == "rtn" else P.mlmc_compress_bits)(plan, g, seed=w.seed, step=args.warmup + i, out=msg)
            lv = msg.level.cpu().numpy()
            for l in lv.tolist():
                drawn[l] = drawn.get(l, 0) + 1
            if w.kind == "rtn":     # the codes of the base, the previous and the drawn level
                per_row = [w.ladder[0] + (w.ladder[l - 1] if l > 1 else 0) + w.ladder[l] for l in lv]
            else:
                per_row = [(9 if w.kind == "fbits" else 1) + w.ladder[0] + w.ladder[l] - w.ladder[l - 1] for l in lv]
            planes_bytes += sum(n * ((w.d + 63) // 64) * 8 for n in per_row)
    nnz_avg = nnz_total / args.steps
    planes_avg = planes_bytes / args.steps

    kern = {k: {"avg_us": ms * 1e3 / n, "launches": n, "share": ms / sum(v[0] for v in prof.values())}
            for k, (ms, n) in prof.items()}
    dominant = max(prof, key=lambda k: prof[k][0])
    dom_avg_s = prof[dominant][0] / prof[dominant][1] / 1e3
    dom_bytes = algorithmic_bytes(w, dominant, nnz_avg, planes_avg)
    achieved = dom_bytes / dom_avg_s / 1e9
    if sparse:
        step_alg_bytes = in_bytes + 16 * nnz_avg + 4 * w.d
    else:
        step_alg_bytes = in_bytes + 2 * planes_avg + 4 * w.d

    value = in_bytes / (ms_per_step * 1e-3) / 1e9
    traffic, traffic_from = measured_traffic(w.name, dominant)
    result = {
        "metric": "mlmc_compress_aggregate_input_throughput",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "d": w.d, "L": w.L, "kind": w.kind,
                   "p": "adaptive" if w.adaptive else "fixed_geometric", "input_bytes": in_bytes,
                   "avg_nnz_per_step": round(nnz_avg, 1), "alpha": alpha,
                   "server": "aggregate + fused model update" if args.fused_update else "aggregate"},
        "hbm_peak_frac_input": round(value / HBM_PEAK_GBPS, 4),
        "hbm_peak_frac_algorithmic": round(step_alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "ms_per_step_with_events": round(dt_ev * 1e3 / args.steps, 4),
        "exact_redo_in_last_step": redone,
        "drawn_levels": {str(l): n for l, n in sorted(drawn.items())},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_from": traffic_from,
                     "avg_us": round(dom_avg_s * 1e6, 2), "algorithmic_bytes_per_launch": int(dom_bytes)},
        "kernels": {k: {"avg_us": round(v["avg_us"], 2), "launches": v["launches"], "share": round(v["share"], 4)}
                    for k, v in sorted(kern.items(), key=lambda kv: -kv[1]["share"])},
    }
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
