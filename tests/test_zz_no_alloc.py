"""The allocation-free entry point eq_quantize_matrix_noalloc against eq_quantize_matrix.

Both run the same kernels; they differ in where the scratch memory lives (the library's built-in
device array instead of a caller's workspace) and in how descriptors, work items and Adam's
bias-correction table get there (a kernel, from by-value arguments, instead of copies from host
memory).  The outputs must be the same bits.  Calls on one GPU share the array, which keeps the
previous call's contents: consecutive calls, the later ones smaller, must not see them."""
import ctypes

import numpy as np
import pytest
import torch

import eq_inputs
import paper_2403_02775_amd as eqg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(W, gp, capacity):
    rows, cols = W.shape
    a = eqg.alloc_outputs(rows, cols, gp, capacity, DEV)
    b = eqg.alloc_outputs(rows, cols, gp, capacity, DEV)
    for o in (a, b):                       # different garbage in both, so that equal bits were written
        for t in (o.codes, o.out_row_ptr, o.out_col, o.status):
            t.fill_(0x5A5A5A5A if o is a else 0x33333333)
        o.out_val.fill_(0x1111 if o is a else 0x2222)
        o.scales.fill_(-1.0 if o is a else -2.0)
        o.zero_points.fill_(200 if o is a else 100)
    ws = torch.empty(eqg.eq_workspace_bytes([rows], [cols], [capacity], gp), dtype=torch.uint8, device=DEV)
    eqg.eq_quantize_matrix(W, gp, a, ws)
    eqg.eq_quantize_matrix_noalloc(W, gp, b)
    torch.cuda.synchronize()
    return a, b


def _same(a, b, what):
    n = int(a.out_row_ptr[-1].item()) & 0xFFFFFFFF
    assert int(a.status.item()) == 0 and int(b.status.item()) == 0, what
    assert torch.equal(a.out_row_ptr, b.out_row_ptr), what
    assert n == (int(b.out_row_ptr[-1].item()) & 0xFFFFFFFF) and n <= a.capacity
    assert torch.equal(a.out_col[:n], b.out_col[:n]) and torch.equal(a.out_val[:n], b.out_val[:n]), what
    assert torch.equal(a.codes, b.codes), what
    assert torch.equal(a.scales.view(torch.int32), b.scales.view(torch.int32)), what
    assert torch.equal(a.zero_points, b.zero_points), what
    return n


# (rows, cols, parameters): every kernel family, the later calls smaller than the first
CASES = [
    (1536, 4096, dict(group_size=128, iters=20)),                       # one lane per unit
    (300, 2048, dict(group_size=128, iters=20)),                        # the same, smaller: stale items and counts
    (257, 1024, dict(group_size=128, iters=0, bits=3)),                 # no optimisation steps
    (40, 4096, dict(group_size=0, iters=12)),                           # one range per row over lanes
    (7, 11008, dict(group_size=0, iters=5)),                            # ... cut into equal pieces
    (64, 256, dict(group_size=0, iters=30, mode=eqg.EQ_ASYMMETRIC)),    # general kernel
    (96, 1024, dict(group_size=128, iters=8, stat_scope=eqg.EQ_STAT_MATRIX, dtype=eqg.EQ_BF16)),
    (48, 512, dict(group_size=64, iters=6, select=eqg.EQ_SELECT_LAST)),
]


def test_noalloc_matches_the_workspace_entry_point_call_after_call():
    for k, (rows, cols, kw) in enumerate(CASES):
        gp = eqg.Params(**kw)
        rec = eq_inputs.with_dtype(eq_inputs.RECIPES["c2"], "bf16" if gp.dtype == eqg.EQ_BF16 else "f16")
        W = eq_inputs.gen_matrix(rows, cols, rec, seed=100 + k, device=DEV)
        cap = eqg.eq_outlier_capacity_bound(rows, cols, gp.n_sigma)
        print(f"[noalloc] case {k}: {rows} x {cols} {kw}", flush=True)
        a, b = _both(W, gp, cap)
        n = _same(a, b, (k, rows, cols, kw))
        assert n > 0


def test_noalloc_twice_in_a_row_second_call_smaller():
    gp = eqg.Params(group_size=128, iters=10)
    big = eq_inputs.gen_matrix(2048, 4096, eq_inputs.RECIPES["c2"], seed=7, device=DEV)
    small = eq_inputs.gen_matrix(130, 1024, eq_inputs.RECIPES["c2"], seed=8, device=DEV)
    for W in (big, small):
        rows, cols = W.shape
        a, b = _both(W, gp, eqg.eq_outlier_capacity_bound(rows, cols, gp.n_sigma))
        _same(a, b, (rows, cols))
    # back to back on one stream without a synchronisation in between: stream order is enough
    o1 = eqg.alloc_outputs(2048, 4096, gp, 200000, DEV)
    o2 = eqg.alloc_outputs(130, 1024, gp, 20000, DEV)
    eqg.eq_quantize_matrix_noalloc(big, gp, o1)
    eqg.eq_quantize_matrix_noalloc(small, gp, o2)
    torch.cuda.synchronize()
    r1 = eqg.alloc_outputs(2048, 4096, gp, 200000, DEV)
    r2 = eqg.alloc_outputs(130, 1024, gp, 20000, DEV)
    for W, r, cap in ((big, r1, 200000), (small, r2, 20000)):
        ws = torch.empty(eqg.eq_workspace_bytes([W.shape[0]], [W.shape[1]], [cap], gp), dtype=torch.uint8, device=DEV)
        eqg.eq_quantize_matrix(W, gp, r, ws)
    torch.cuda.synchronize()
    _same(r1, o1, "big")
    _same(r2, o2, "small")


def test_noalloc_outlier_overflow_and_empty_matrix():
    gp = eqg.Params(group_size=128, iters=3)
    W = eq_inputs.gen_matrix(64, 1024, eq_inputs.RECIPES["c2"], seed=9, device=DEV)
    o = eqg.alloc_outputs(64, 1024, gp, 5, DEV)          # far too few entries
    eqg.eq_quantize_matrix_noalloc(W, gp, o)
    torch.cuda.synchronize()
    assert int(o.status.item()) & eqg.EQ_S_OUTLIER_OVERFLOW
    full = eqg.alloc_outputs(64, 1024, gp, 8000, DEV)
    eqg.eq_quantize_matrix_noalloc(W, gp, full)
    torch.cuda.synchronize()
    assert int(full.status.item()) == 0
    assert torch.equal(o.out_row_ptr, full.out_row_ptr)  # the true counts, so that the caller can re-size
    e = eqg.alloc_outputs(0, 1024, gp, 0, DEV)
    e.out_row_ptr.fill_(77)
    eqg.eq_quantize_matrix_noalloc(torch.empty((0, 1024), dtype=torch.float16, device=DEV), gp, e)
    torch.cuda.synchronize()
    assert int(e.out_row_ptr[0].item()) == 0 and int(e.status.item()) == 0


def test_noalloc_replays_from_a_hip_graph():
    """What the entry point is for: it enqueues kernels only, so a whole quantization can be recorded
    into a HIP graph.  Every replay, with fresh weights in the same buffer and eager work and
    synchronisations in between, must give the bits of the eager workspace call."""
    rows, cols = 512, 4096
    gp = eqg.Params(group_size=128, iters=6)
    cap = 60000
    W = eq_inputs.gen_matrix(rows, cols, eq_inputs.RECIPES["c2"], seed=40, device=DEV)
    out = eqg.alloc_outputs(rows, cols, gp, cap, DEV)
    ref = eqg.alloc_outputs(rows, cols, gp, cap, DEV)
    ws = torch.empty(eqg.eq_workspace_bytes([rows], [cols], [cap], gp), dtype=torch.uint8, device=DEV)
    eqg.eq_quantize_matrix_noalloc(W, gp, out)        # first call outside the capture: looks up the array's address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            eqg.eq_quantize_matrix_noalloc(W, gp, out)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        W.copy_(eq_inputs.gen_matrix(rows, cols, eq_inputs.RECIPES["c2"], seed=41 + rep, device=DEV))
        eqg.eq_quantize_matrix(W, gp, ref, ws)
        for t in (out.codes, out.out_row_ptr, out.out_col, out.status):
            t.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _same(ref, out, rep) > 0


