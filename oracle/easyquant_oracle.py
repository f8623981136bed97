"""Plain CPU oracle for the EasyQuant quantization path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module.  It shares no code with the HIP path and never calls it.

What it computes (EasyQuant, Algorithm 1, "Quantize" and "Dequantize"):

1. the n-sigma outlier index set of a weight            (Eq. 3)
2. an Adam optimisation of the quantization range of every unit (one output
   channel, or one group of consecutive input positions of it) using the
   gradient of the reconstruction error                  (Eq. 2, Section 4.2)
3. round-to-nearest codes of the normal values at that range (Eq. 1)
4. the composite reconstruction: outliers verbatim, the rest dequantized (Eq. 4)

The method is an iteration, so the oracle takes the algorithm's steps in order,
vectorised over units with NumPy (every unit sees the same scalar sequence of
operations; nothing is blocked, fused or reordered).  The iteration is chaotic
at the last bit, therefore the arithmetic is pinned as well:

* the scale s = r / D and its reciprocal are binary32 (one rounding each); the level
  of an element is the EXACT product x * (1/s) rounded ONCE to the nearest integer,
  ties to even, as Eq. 1 rounds a real number (the product of a 16-bit value and a
  binary32 value is exact in binary64, so no intermediate rounding takes part);
* the two sums of Eq. 2, ``A = sum c_i^2`` and ``B = sum x_i c_i``, are EXACT
  (integers, and a binary64 accumulation of exact binary32 products that is
  checked to be exact; ``math.fsum`` otherwise);
* the scalar recurrence (loss, gradient, Adam) in binary64, one rounding per
  operation, no fused multiply-add; the range is rounded to binary32 each step.

Readings of the paper that this file implements (the paper is silent or
ambiguous on each; they are listed once more in the design notes):

* Eq. 3 prints ``n * var(W)`` but calls it the n-sigma criterion and reports
  fewer than 1 % outliers at n = 3, which only the standard deviation gives;
  population sigma (divide by N); ``>=`` as printed; a constant scope (sigma = 0)
  has no outliers.
* mean / sigma are taken over one row by default (also: one group, or the whole
  matrix as Eq. 3 literally says).
* "Quantization range" (Section 3.1, Table 10) is the clipping bound ``r``; the
  scale of Eq. 1 is ``s = r / D``.  Adam steps ``r``.  Table 10's range moving by
  about one learning rate per step early on is what Adam does to the variable it
  updates.
* Adam: beta1 = 0.9, beta2 = 0.999, eps = 1e-8 unless given, bias-corrected.
* Symmetric mode (the paper's): integer levels ``-(2^(k-1)-1) .. 2^(k-1)``
  (Eq. 1's l_min, l_max); initial range = max |x| over the normal values, mapped
  to level ``D = 2^(k-1)-1`` so that nothing clips at step 0.
* Asymmetric mode is an extension: an integer zero-point fixed at initialisation
  from min/max (including 0), ``D = 2^k-1``; only the range is optimised.
* The rounding operator of Eq. 1 is round-half-to-even.
* The code inside the gradient is the clamped one (the true derivative of Eq. 1).
* Only normal values enter the range, A and B (Section 4.2).
* The returned range is the best iterate of the trajectory, step 0 included
  (``select=BEST``), or the last one as the paper states (``select=LAST``).
* The range never drops below ``r0 * 2^-10``.

Pinned by tests/test_oracle_*.py against: a hand-worked example, the textbook
abs-max round-to-nearest quantizer, a finite-difference gradient of Eq. 1's loss,
``torch.optim.Adam``, a brute-force scan over scales, the Gaussian 3-sigma tail
mass, and structural invariants.  The paper's own numeric tables need real model
weights and datasets: parity against them is unpinned.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

F16, BF16 = 0, 1
SYMMETRIC, ASYMMETRIC = 0, 1
STAT_ROW, STAT_GROUP, STAT_MATRIX = 0, 1, 2
SELECT_BEST, SELECT_LAST = 0, 1

_f32 = np.float32
_f64 = np.float64


@dataclass
class Params:
    dtype: int = F16
    bits: int = 4
    group_size: int = 0          # 0 = one range per row (per output channel)
    mode: int = SYMMETRIC
    stat_scope: int = STAT_ROW
    n_sigma: float = 3.0
    iters: int = 100
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    select: int = SELECT_BEST


# --------------------------------------------------------------------------- #
# storage formats                                                              #
# --------------------------------------------------------------------------- #
def widen(raw: np.ndarray, dtype: int) -> np.ndarray:
    """Raw 16-bit patterns -> binary32 values (exact for both formats)."""
    raw = np.ascontiguousarray(raw, dtype=np.uint16)
    if dtype == F16:
        return raw.view(np.float16).astype(_f32)
    if dtype == BF16:
        return (raw.astype(np.uint32) << np.uint32(16)).view(_f32)
    raise ValueError("dtype")


def narrow(x32: np.ndarray, dtype: int) -> np.ndarray:
    """binary32 -> raw 16-bit patterns, round-to-nearest-even."""
    x32 = np.ascontiguousarray(x32, dtype=_f32)
    if dtype == F16:
        return x32.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        b = x32.view(np.uint32).astype(np.uint64)
        lsb = (b >> np.uint64(16)) & np.uint64(1)
        r = (b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
        return r.astype(np.uint16)
    raise ValueError("dtype")


def pack_codes(u: np.ndarray, bits: int) -> np.ndarray:
    """Unsigned codes (rows x cols) -> per-row little-endian bitstream in uint32 words.

    Code j of a row occupies bits [bits*j, bits*j + bits) of the row's stream;
    each row is padded with zero bits to a whole number of 32-bit words.
    """
    rows, cols = u.shape
    words = (cols * bits + 31) // 32
    planes = ((u[:, :, None].astype(np.uint32) >> np.arange(bits, dtype=np.uint32)) & 1).astype(np.uint8)
    stream = planes.reshape(rows, cols * bits)
    pad = words * 32 - cols * bits
    if pad:
        stream = np.concatenate([stream, np.zeros((rows, pad), np.uint8)], axis=1)
    by = np.packbits(stream, axis=1, bitorder="little")
    return np.ascontiguousarray(by).view("<u4").reshape(rows, words)


def unpack_codes(words: np.ndarray, cols: int, bits: int) -> np.ndarray:
    rows = words.shape[0]
    by = np.ascontiguousarray(words.astype("<u4")).view(np.uint8).reshape(rows, -1)
    stream = np.unpackbits(by, axis=1, bitorder="little")[:, : cols * bits].reshape(rows, cols, bits)
    return (stream.astype(np.uint32) << np.arange(bits, dtype=np.uint32)).sum(axis=2).astype(np.int32)


# --------------------------------------------------------------------------- #
# Eq. 3: outliers                                                              #
# --------------------------------------------------------------------------- #
def outlier_mask(x32: np.ndarray, n_sigma: float, scope: int, group_size: int) -> np.ndarray:
    """Boolean mask of the (n sigma) outliers of a rows x cols matrix (Eq. 3).

    mean and population standard deviation over the scope, two passes, binary64;
    every element of the scope enters them, outliers included.
    """
    rows, cols = x32.shape
    x = x32.astype(_f64)
    n = _f64(_f32(n_sigma))
    if scope == STAT_MATRIX:
        v = x.reshape(1, -1)
    elif scope == STAT_ROW or group_size == 0:
        v = x
    elif scope == STAT_GROUP:
        v = x.reshape(rows * (cols // group_size), group_size)
    else:
        raise ValueError("scope")
    cnt = _f64(v.shape[1])
    mu = v.sum(axis=1, keepdims=True) / cnt
    d = v - mu
    sigma = np.sqrt((d * d).sum(axis=1, keepdims=True) / cnt)
    with np.errstate(invalid="ignore"):
        m = (sigma > 0) & (np.abs(d) >= n * sigma)
    return m.reshape(rows, cols)


# --------------------------------------------------------------------------- #
# Eq. 1 / Eq. 2 at a given range                                               #
# --------------------------------------------------------------------------- #
def _exact_dot(prod32: np.ndarray, unit_ulp: np.ndarray) -> np.ndarray:
    """Row sums of exact binary32 products, as the exact real sum rounded once.

    A binary64 accumulation is exact when every partial sum is a multiple of the
    unit's smallest ulp and stays below 2^53 of them; where that cannot be
    certified the row is summed with ``math.fsum`` (exactly rounded).
    """
    p = prod32.astype(_f64)
    B = p.sum(axis=1)
    bound = np.abs(p).sum(axis=1)
    unsafe = bound >= unit_ulp * _f64(2.0 ** 52)
    for i in np.nonzero(unsafe)[0]:
        B[i] = math.fsum(p[i].tolist())
    return B


class UnitView:
    """Per-unit view of the normal values of one matrix and its level bounds."""

    def __init__(self, x32: np.ndarray, mask: np.ndarray, p: Params):
        rows, cols = x32.shape
        G = p.group_size if p.group_size else cols
        if cols % G:
            raise ValueError("group_size must divide cols")
        self.rows, self.cols, self.G, self.upr = rows, cols, G, cols // G
        L = (1 << p.bits) - 1
        xt = np.where(mask, _f32(0), x32).reshape(rows * self.upr, G)   # outliers leave the unit
        normal = (~mask).reshape(rows * self.upr, G)
        self.xt = xt
        nu = xt.shape[0]
        if p.mode == SYMMETRIC:
            z = np.full(nu, (1 << (p.bits - 1)) - 1, np.int32)
            self.D = _f32((1 << (p.bits - 1)) - 1)
            r0 = np.abs(xt).max(axis=1).astype(_f32)
        elif p.mode == ASYMMETRIC:
            self.D = _f32(L)
            lo = np.minimum(xt.min(axis=1), _f32(0))
            hi = np.maximum(xt.max(axis=1), _f32(0))
            r0 = (hi - lo).astype(_f32)
            with np.errstate(divide="ignore", invalid="ignore"):
                s0 = r0 / self.D
                zf = np.rint((-lo) / s0)
            zf = np.where(r0 > 0, zf, _f32(0))
            z = np.clip(zf, 0, L).astype(np.int32)
        else:
            raise ValueError("mode")
        self.r0 = r0
        # a unit with no normal value, or whose normal values are all zero, keeps s = 1 and is not optimised
        self.active = normal.any(axis=1) & (r0 > 0)
        self.z = z.astype(np.int32)
        self.c_lo = (-self.z).astype(_f32)
        self.c_hi = (L - self.z).astype(_f32)
        # smallest ulp among the non-zero values of each unit (for the exactness check)
        ax = np.abs(xt).astype(_f64)
        ax[ax == 0] = np.inf
        mn = ax.min(axis=1)
        mant = 10 if p.dtype == F16 else 7
        with np.errstate(invalid="ignore"):
            e = np.where(np.isfinite(mn), np.floor(np.log2(np.where(np.isfinite(mn), mn, 1.0))), 0.0)
        floor_e = -14.0 if p.dtype == F16 else -126.0
        self.ulp = np.exp2(np.maximum(e, floor_e) - mant)

    def evaluate(self, r32: np.ndarray):
        """(codes, scale, A, B, J, g) at range ``r32``: J = loss - sum x^2, g = d loss / d range (Eq. 2 through s = r/D)."""
        D = self.D
        s32 = (r32 / D).astype(_f32)
        inv32 = (_f32(1.0) / s32).astype(_f32)
        t = self.xt.astype(_f64) * inv32.astype(_f64)[:, None]       # exact (<= 11 + 24 significant bits)
        tc = np.minimum(np.maximum(t, self.c_lo.astype(_f64)[:, None]), self.c_hi.astype(_f64)[:, None])
        c = np.rint(tc).astype(_f32)
        ci = c.astype(np.int64)
        A = (ci * ci).sum(axis=1)
        B = _exact_dot((self.xt * c).astype(_f32), self.ulp)
        s = s32.astype(_f64)
        e = s * A.astype(_f64) - B
        J = s * (e - B)
        g = (_f64(2.0) * e) / _f64(D)
        return ci.astype(np.int32), s32, A, B, J, g


def optimise_range(units: UnitView, p: Params, trace: Optional[list] = None):
    """Adam on the range of every unit (Section 4.2; Algorithm 1, second step)."""
    nu = units.xt.shape[0]
    act = units.active
    r0 = units.r0.astype(_f32)
    r32 = np.where(act, r0, _f32(1.0) * units.D).astype(_f32)   # inactive: s = 1
    lr, b1, b2, eps = (_f64(_f32(v)) for v in (p.lr, p.beta1, p.beta2, p.eps))
    if not eps > 0:
        raise ValueError("eps must be positive (a zero gradient would step by 0 / 0)")
    m = np.zeros(nu, _f64)
    v = np.zeros(nu, _f64)
    p1 = _f64(1.0)
    p2 = _f64(1.0)
    floor_r = r0.astype(_f64) * _f64(2.0 ** -10)
    J_best = np.full(nu, np.inf, _f64)
    r_best = r32.copy()
    if trace is not None:
        trace.append(r32.copy())
    for _ in range(p.iters):
        _, _, _, _, J, g = units.evaluate(r32)
        better = J < J_best
        J_best = np.where(better, J, J_best)
        r_best = np.where(better, r32, r_best)
        m = b1 * m + (_f64(1.0) - b1) * g
        v = b2 * v + (_f64(1.0) - b2) * (g * g)
        p1 = p1 * b1
        p2 = p2 * b2
        mh = m / (_f64(1.0) - p1)
        vh = v / (_f64(1.0) - p2)
        r64 = r32.astype(_f64) - lr * (mh / (np.sqrt(vh) + eps))
        r_new = np.maximum(r64, floor_r).astype(_f32)
        r32 = np.where(act, r_new, r32)
        if trace is not None:
            trace.append(r32.copy())
    if p.select == SELECT_BEST:
        _, _, _, _, J, _ = units.evaluate(r32)
        better = J < J_best
        r_best = np.where(better, r32, r_best)
        return r_best.astype(_f32)
    if p.select == SELECT_LAST:
        return r32
    raise ValueError("select")


# --------------------------------------------------------------------------- #
# Algorithm 1                                                                  #
# --------------------------------------------------------------------------- #
def quantize_matrix(raw: np.ndarray, p: Params, trace: Optional[list] = None) -> Dict[str, np.ndarray]:
    """Algorithm 1, "Quantize", for one rows x cols matrix of raw 16-bit patterns.

    Returns packed codes, per-unit scale (binary32) and zero-point, and the
    outliers as a CSR-like list (row_ptr, column ascending within a row, raw
    16-bit value), plus the chosen range per unit for diagnostics.
    """
    raw = np.ascontiguousarray(raw, dtype=np.uint16)
    rows, cols = raw.shape
    x32 = widen(raw, p.dtype)
    if not np.isfinite(x32).all():
        raise ValueError("non-finite input")
    mask = outlier_mask(x32, p.n_sigma, p.stat_scope, p.group_size)
    units = UnitView(x32, mask, p)
    r = optimise_range(units, p, trace)
    c, s32, _, _, _, _ = units.evaluate(r)
    u = (c + units.z[:, None]).reshape(rows, cols)
    assert u.min(initial=0) >= 0 and u.max(initial=0) <= (1 << p.bits) - 1
    counts = mask.sum(axis=1)
    row_ptr = np.zeros(rows + 1, np.uint32)
    row_ptr[1:] = np.cumsum(counts)
    rr, cc = np.nonzero(mask)            # row-major order: rows ascending, columns ascending within a row
    return {
        "codes": pack_codes(u.astype(np.uint8), p.bits),
        "scales": s32.reshape(rows, units.upr).astype(_f32),
        "zero_points": units.z.reshape(rows, units.upr).astype(np.uint8),
        "out_row_ptr": row_ptr,
        "out_col": cc.astype(np.uint32),
        "out_val": raw[rr, cc].astype(np.uint16),
        "range": r.reshape(rows, units.upr),
        "mask": mask,
        "u": u.astype(np.uint8),
    }


def dequantize(q: Dict[str, np.ndarray], rows: int, cols: int, p: Params) -> np.ndarray:
    """Algorithm 1, "Dequantize" (Eq. 4): raw 16-bit patterns of the reconstruction."""
    G = p.group_size if p.group_size else cols
    u = unpack_codes(q["codes"], cols, p.bits)
    z = np.repeat(q["zero_points"].astype(np.int32).reshape(rows, cols // G), G, axis=1)
    s = np.repeat(q["scales"].astype(_f32).reshape(rows, cols // G), G, axis=1)
    xh = (s * (u - z).astype(_f32)).astype(_f32)
    out = narrow(xh, p.dtype).reshape(rows, cols)
    row_ptr = q["out_row_ptr"].astype(np.int64)
    rr = np.repeat(np.arange(rows), np.diff(row_ptr))
    out[rr, q["out_col"].astype(np.int64)] = q["out_val"]
    return out


def dequant_matvec(q: Dict[str, np.ndarray], rows: int, cols: int, p: Params, x_raw: np.ndarray) -> np.ndarray:
    """The reconstruction of Eq. 4 applied to a vector: y = W^ x in binary64, W^ = dequantize(q)
    (every element already rounded to the 16-bit type), x given as raw 16-bit patterns."""
    W = widen(dequantize(q, rows, cols, p), p.dtype).astype(_f64)
    x = widen(np.asarray(x_raw).reshape(cols), p.dtype).astype(_f64)
    return W @ x


def reconstruction_sse(raw: np.ndarray, deq_raw: np.ndarray, dtype: int) -> np.ndarray:
    """Per-row squared reconstruction error (the paper's r(W), Section 2), binary64."""
    d = widen(deq_raw, dtype).astype(_f64) - widen(raw, dtype).astype(_f64)
    return (d * d).sum(axis=1)
