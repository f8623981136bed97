"""The oracle over blocks of whole rows in worker processes.  TEST INFRASTRUCTURE ONLY.

With row or group statistics every row of a matrix is quantized independently of the others
(Eq. 3 is taken per row, Eq. 2 and Adam per unit of a row), so ``quantize_matrix`` applied to
blocks of rows and concatenated IS ``quantize_matrix`` of the whole matrix.  This module does
only that: it hands blocks of rows to ``easyquant_oracle.quantize_matrix`` in a pool of
processes and stitches the results together (the outlier list's row pointers get their
offsets).  It holds none of the method's arithmetic.  Whole-matrix statistics are refused.

Workers are started with the ``forkserver`` method from a process that has not touched a GPU
yet: create the pool before the first GPU call of the program (a test session's first fixture,
the first lines of the benchmark).  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module.
"""
from __future__ import annotations

import multiprocessing
import os
import time
from concurrent.futures import ProcessPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import easyquant_oracle as eqo


def _worker_ready(_: int) -> int:
    return os.getpid()


def _quantize_block(args) -> Tuple[int, Dict[str, np.ndarray], float]:
    key, raw, p_kwargs, keep = args
    t0 = time.perf_counter()
    q = eqo.quantize_matrix(raw, eqo.Params(**p_kwargs))
    dt = time.perf_counter() - t0
    return key, {k: q[k] for k in keep}, dt


KEEP_ALL = ("codes", "scales", "zero_points", "out_row_ptr", "out_col", "out_val", "mask", "u")


class RowPool:
    def __init__(self, workers: int):
        self.workers = max(1, int(workers))
        ctx = multiprocessing.get_context("forkserver")
        self.pool = ProcessPoolExecutor(max_workers=self.workers, mp_context=ctx)
        # start every worker now (imports NumPy and the oracle there), so that none is forked later
        self.pids = sorted(set(self.pool.map(_worker_ready, range(4 * self.workers))))

    def close(self):
        self.pool.shutdown(wait=True, cancel_futures=True)

    def quantize_blocks(self, blocks: Sequence[np.ndarray], p: eqo.Params, keep=KEEP_ALL) -> List[Dict[str, np.ndarray]]:
        """quantize_matrix of every block (each a rows x cols array of raw patterns), in order."""
        if p.stat_scope == eqo.STAT_MATRIX:
            raise ValueError("whole-matrix statistics couple the rows: not for the row pool")
        kw = dict(p.__dict__)
        jobs = [(i, np.ascontiguousarray(b), kw, tuple(keep)) for i, b in enumerate(blocks)]
        out: List[Optional[Dict[str, np.ndarray]]] = [None] * len(jobs)
        self.last_cpu_seconds = 0.0
        for key, q, dt in self.pool.map(_quantize_block, jobs):
            out[key] = q
            self.last_cpu_seconds += dt
        return out  # type: ignore[return-value]

    def quantize_matrix(self, raw: np.ndarray, p: eqo.Params, rows_per_block: int = 16) -> Dict[str, np.ndarray]:
        """quantize_matrix(raw, p), its rows spread over the workers."""
        rows = raw.shape[0]
        cuts = list(range(0, rows, rows_per_block)) or [0]
        parts = self.quantize_blocks([raw[a:a + rows_per_block] for a in cuts], p)
        return stitch(parts)


def stitch(parts: Sequence[Dict[str, np.ndarray]]) -> Dict[str, np.ndarray]:
    """Results of consecutive row blocks -> the result of the matrix they tile."""
    out = {k: np.concatenate([q[k] for q in parts], axis=0) for k in ("codes", "scales", "zero_points", "mask", "u")
           if k in parts[0]}
    out["out_col"] = np.concatenate([q["out_col"] for q in parts])
    out["out_val"] = np.concatenate([q["out_val"] for q in parts])
    ptr = [np.zeros(1, np.uint32)]
    base = 0
    for q in parts:
        ptr.append((q["out_row_ptr"][1:].astype(np.int64) + base).astype(np.uint32))
        base += int(q["out_row_ptr"][-1])
    out["out_row_ptr"] = np.concatenate(ptr)
    return out
