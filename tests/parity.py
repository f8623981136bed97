"""Helpers of the GPU parity tests: run the HIP path through the C ABI, fetch its outputs,
and compare them with the CPU oracle under the stated bar.

The bar (written here once, used by every parity test):
  * outlier list (row_ptr, columns, raw values) and integer codes: bit-exact, except that a
    mask decision may differ for an element whose |x - mean| lies within 1e-6 (relative) of
    n*sigma, and a code may differ for an element whose pre-rounding value x/s lies within
    1e-6 (relative) of a rounding boundary.  A differing mask changes the sums of its whole
    unit, so that unit is excused as a whole; excused ELEMENTS are counted and must stay
    below 1e-5 of all elements;
  * scales: 1e-4 relative; zero-points: exact;
  * per-row reconstruction error: 1e-4 relative (rows that hold an excused unit are skipped).
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2403_02775_amd as eqg
from oracle import easyquant_oracle as eqo

BAND = 1e-6
MAX_EXCUSED_FRACTION = 1e-5
SCALE_RTOL = 1e-4
SSE_RTOL = 1e-4


def to_gpu_params(p: eqo.Params) -> eqg.Params:
    return eqg.Params(dtype=p.dtype, bits=p.bits, group_size=p.group_size, mode=p.mode, stat_scope=p.stat_scope,
                      n_sigma=p.n_sigma, iters=p.iters, lr=p.lr, beta1=p.beta1, beta2=p.beta2, eps=p.eps,
                      select=p.select)


def raw_of(w: torch.Tensor) -> np.ndarray:
    return w.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def run_gpu(Ws, p: eqo.Params, capacities=None, batch=True):
    """Quantize the CUDA tensors `Ws` with the HIP path; returns (list of QMatrix, list of dicts of numpy arrays)."""
    gp = to_gpu_params(p)
    dev = Ws[0].device
    if capacities is None:
        capacities = [eqg.eq_outlier_capacity_bound(W.shape[0], W.shape[1], p.n_sigma) for W in Ws]
    outs = [eqg.alloc_outputs(W.shape[0], W.shape[1], gp, cap, dev) for W, cap in zip(Ws, capacities)]
    nbytes = eqg.eq_workspace_bytes([W.shape[0] for W in Ws], [W.shape[1] for W in Ws], capacities, gp)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    if batch:
        eqg.eq_quantize_batch(Ws, gp, outs, ws)
    else:
        assert len(Ws) == 1
        eqg.eq_quantize_matrix(Ws[0], gp, outs[0], ws)
    torch.cuda.synchronize()
    return outs, [fetch(o, W.shape[0], W.shape[1], p) for o, W in zip(outs, Ws)]


def fetch(o, rows, cols, p):
    rp = o.out_row_ptr.cpu().numpy().view(np.uint32)
    n = int(rp[-1]) if rows >= 0 else 0
    n = min(n, o.capacity)
    codes = o.codes.cpu().numpy().view(np.uint32)
    return {
        "codes": codes,
        "scales": o.scales.cpu().numpy(),
        "zero_points": o.zero_points.cpu().numpy(),
        "out_row_ptr": rp,
        "out_col": o.out_col[:n].cpu().numpy().view(np.uint32),
        "out_val": o.out_val[:n].cpu().numpy().view(np.uint16),
        "status": int(o.status.cpu().item()),
    }


def gpu_dequantize(o, rows, cols, p: eqo.Params, dev) -> np.ndarray:
    gp = to_gpu_params(p)
    out = torch.empty((rows, cols), dtype=torch.float16 if p.dtype == eqo.F16 else torch.bfloat16, device=dev)
    eqg.eq_dequantize(o, rows, cols, gp, out)
    torch.cuda.synchronize()
    return raw_of(out)


def compare(raw: np.ndarray, got: dict, want: dict, p: eqo.Params, what: str = "") -> dict:
    """Applies the bar of this module; returns the counts it found, raises AssertionError otherwise."""
    rows, cols = raw.shape
    G = p.group_size if p.group_size else cols
    upr = cols // G if cols else 1
    assert got["status"] == 0, (what, "status", got["status"])
    # ---- masks -------------------------------------------------------------------------
    def dense_mask(q):
        m = np.zeros((rows, cols), bool)
        rp = q["out_row_ptr"].astype(np.int64)
        rr = np.repeat(np.arange(rows), np.diff(rp))
        m[rr, q["out_col"].astype(np.int64)] = True
        return m
    assert got["out_row_ptr"].shape == want["out_row_ptr"].shape
    assert (np.diff(got["out_row_ptr"].astype(np.int64)) >= 0).all(), (what, "row_ptr not monotone")
    assert len(got["out_col"]) == int(got["out_row_ptr"][-1]), what
    mg, mw = dense_mask(got), want["mask"]
    assert mg.sum() == len(got["out_col"]), (what, "duplicate or unsorted outlier columns")
    excused_unit = np.zeros((rows, upr), bool)
    excused_elems = 0
    diff = mg != mw
    if diff.any():
        x = eqo.widen(raw, p.dtype).astype(np.float64)
        n = np.float64(np.float32(p.n_sigma))
        for r, c in zip(*np.nonzero(diff)):
            if p.stat_scope == eqo.STAT_ROW or (p.stat_scope == eqo.STAT_GROUP and p.group_size == 0):
                v = x[r]
            elif p.stat_scope == eqo.STAT_GROUP:
                v = x[r, (c // G) * G:(c // G + 1) * G]
            else:
                v = x.reshape(-1)
            thr = n * v.std()
            rel = abs(abs(x[r, c] - v.mean()) - thr) / thr
            assert rel <= BAND, (what, "mask differs outside the band", r, c, rel)
            excused_unit[r, c // G] = True
            excused_elems += 1
    # outlier columns sorted within each row and values verbatim
    rp = got["out_row_ptr"].astype(np.int64)
    rr = np.repeat(np.arange(rows), np.diff(rp))
    cc = got["out_col"].astype(np.int64)
    if len(cc):
        same_row = rr[1:] == rr[:-1]
        assert (np.diff(cc)[same_row] > 0).all(), (what, "columns not ascending within a row")
        assert (raw[rr, cc] == got["out_val"]).all(), (what, "outlier values not verbatim")
    if not diff.any():
        assert (got["out_row_ptr"] == want["out_row_ptr"]).all() and (got["out_col"] == want["out_col"]).all()
        assert (got["out_val"] == want["out_val"]).all()
    # ---- zero-points, scales -------------------------------------------------------------
    ok_unit = ~excused_unit
    assert (got["zero_points"].reshape(rows, upr)[ok_unit] == want["zero_points"].reshape(rows, upr)[ok_unit]).all(), what
    sg, sw = got["scales"].reshape(rows, upr).astype(np.float64), want["scales"].reshape(rows, upr).astype(np.float64)
    rel = np.abs(sg - sw) / np.abs(sw)
    assert (rel[ok_unit] <= SCALE_RTOL).all(), (what, "scale", rel[ok_unit].max())
    scale_exact = int((got["scales"].reshape(rows, upr)[ok_unit] == want["scales"].reshape(rows, upr)[ok_unit]).sum())
    # ---- codes -------------------------------------------------------------------------
    ug = eqo.unpack_codes(got["codes"], cols, p.bits) if cols else np.zeros((rows, 0), np.int32)
    uw = want["u"].astype(np.int32)
    cd = (ug != uw) & np.repeat(ok_unit, G, axis=1)
    code_mismatch = int(cd.sum())
    if code_mismatch:
        x32 = eqo.widen(raw, p.dtype)
        for r, c in zip(*np.nonzero(cd)):
            s = np.float32(want["scales"].reshape(rows, upr)[r, c // G])
            # the pre-rounding value as the oracle forms it: the exact product of the element and
            # the binary32 reciprocal of the scale (exact in binary64)
            t = float(np.float64(x32[r, c]) * np.float64(np.float32(1.0) / s))
            dist = abs(abs(t - np.floor(t)) - 0.5)
            assert dist <= BAND * max(abs(t), 1.0), (what, "code differs outside the band", r, c, t, ug[r, c], uw[r, c])
            excused_elems += 1
    total = max(rows * cols, 1)
    assert excused_elems <= MAX_EXCUSED_FRACTION * total or excused_elems == 0, (what, "excused", excused_elems)
    if cols and (got["codes"].shape == want["codes"].shape) and not excused_unit.any() and not code_mismatch:
        assert (got["codes"] == want["codes"]).all(), (what, "packed words (padding bits?)")
    return {"excused_elems": excused_elems, "excused_units": int(excused_unit.sum()), "scale_exact": scale_exact,
            "units": rows * upr, "code_mismatch": code_mismatch, "rows_ok": ~excused_unit.any(axis=1)}


def compare_sse(raw, deq_gpu, deq_oracle, p, rows_ok, what=""):
    a = eqo.reconstruction_sse(raw, deq_gpu, p.dtype)
    b = eqo.reconstruction_sse(raw, deq_oracle, p.dtype)
    ok = rows_ok & (b > 0)
    rel = np.abs(a[ok] - b[ok]) / b[ok]
    assert (rel <= SSE_RTOL).all(), (what, "per-row reconstruction error", rel.max())
    assert (a[rows_ok & (b == 0)] == 0).all()
