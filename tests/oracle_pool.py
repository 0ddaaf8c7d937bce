"""Runs the CPU oracle on the rows of a named workload in worker processes (one row per task).

The children import numpy, the seeded generators and the oracle only -- nothing that touches a GPU -- and rebuild
their row from (workload, row index), so no input crosses the process boundary.  They are started with the
"spawn" method: a fresh interpreter, not a fork of a process that may hold GPU state.
"""
import multiprocessing as mp
import os
from concurrent.futures import ProcessPoolExecutor

import numpy as np

import mlmc_workloads as W
from oracle import mlmc as O


def _layout(w):
    if w.gen == "iid_normal":
        return None
    return W.segment_layout(w.d, w.extra["segments"], w.extra["std_lo"], w.extra["std_hi"], w.seed)


def _topk_row(args):
    name, d, M, row, seed, steps, p_fixed = args
    w = W.WORKLOADS[name] if d is None else W.scaled(W.WORKLOADS[name], d=d, M=M)
    g = W.generate_row(w, row, _layout(w))
    out = []
    for step in steps:
        m = O.compress_topk_row(g, w.ladder, p_fixed, seed, step, row)
        out.append(dict(level=m["level"], idx=m["idx"], val=m["val"], norms=m["norms"], p=m["p"]))
    return row, out


def oracle_topk_rows(name, seed, steps, rows=None, p_fixed=None, d=None, M=None, workers=None):
    """{row: [message of every step in `steps`]} from O.compress_topk_row, rows of WORKLOADS[name] (or of its
    scaled version).  `workers` processes, default min(rows, cores, 8)."""
    w = W.WORKLOADS[name] if d is None else W.scaled(W.WORKLOADS[name], d=d, M=M)
    rows = list(range(w.M)) if rows is None else list(rows)
    if workers is None:
        workers = max(1, min(len(rows), os.cpu_count() or 1, 8))
    tasks = [(name, d, M, r, seed, tuple(steps), p_fixed) for r in rows]
    if workers == 1:
        return dict(_topk_row(t) for t in tasks)
    with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as ex:
        return dict(ex.map(_topk_row, tasks))
