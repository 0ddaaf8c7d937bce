"""Runs the CPU oracle on the rows of a named workload in worker processes (one row per task).

The children import numpy, the seeded generators and the oracle only -- nothing that touches a GPU -- and rebuild
their row from (workload, row index), so no input crosses the process boundary.  They are started with the
"spawn" method: a fresh interpreter, not a fork of a process that may hold GPU state.
"""
import multiprocessing as mp
import os
from concurrent.futures import ProcessPoolExecutor, as_completed

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


class OracleTopkRows:
    """O.compress_topk_row on rows of WORKLOADS[name] (or of its scaled version) for every step in `steps`, started
    in `workers` processes (default min(rows, cores, 8)) when the object is made; result() waits and returns
    {row: [message of every step]}, printing a line per finished row."""

    def __init__(self, name, seed, steps, rows=None, p_fixed=None, d=None, M=None, workers=None):
        w = W.WORKLOADS[name] if d is None else W.scaled(W.WORKLOADS[name], d=d, M=M)
        rows = list(range(w.M)) if rows is None else list(rows)
        if workers is None:
            workers = max(1, min(len(rows), os.cpu_count() or 1, 8))
        self.name = name
        self.tasks = [(name, d, M, r, seed, tuple(steps), p_fixed) for r in rows]
        self.ex = ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn"))
        self.futures = [self.ex.submit(_topk_row, t) for t in self.tasks]

    def result(self):
        out = {}
        try:
            for f in as_completed(self.futures):
                row, msgs = f.result()
                out[row] = msgs
                print(f"oracle: {self.name} row {row} done ({len(out)} of {len(self.futures)})", flush=True)
        finally:
            self.ex.shutdown(wait=True, cancel_futures=True)
        return out


def oracle_topk_rows(name, seed, steps, rows=None, p_fixed=None, d=None, M=None, workers=None):
    return OracleTopkRows(name, seed, steps, rows, p_fixed, d, M, workers).result()
