"""Pins of the CPU oracle against things other than itself.

Each test fixes one part of ``oracle/easyquant_oracle.py`` to a value or a
property that the paper, the mathematics or an independent library determines:
hand-worked examples (tests/golden), the textbook abs-max quantizer, a finite
difference of Eq. 1's loss, ``torch.optim.Adam``, a brute-force scan over scales,
the Gaussian tail mass and structural invariants.
"""
import math
import os

import numpy as np
import pytest
import torch

import eq_inputs
from oracle import easyquant_oracle as eq

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = v
    return out


def _raw16(a, dtype=eq.F16):
    a = np.asarray(a, np.float32)
    return eq.narrow(a, dtype).reshape(a.shape)


def _units(x, p, mask=None):
    x32 = eq.widen(_raw16(x, p.dtype), p.dtype).reshape(np.asarray(x).shape)
    if mask is None:
        mask = eq.outlier_mask(x32, p.n_sigma, p.stat_scope, p.group_size)
    return eq.UnitView(x32, mask, p), x32, mask


# Independent restatement of Eq. 1 and of the reconstruction error, in binary64.
def _loss_eq1(x, s, l_min, l_max):
    q = s * np.rint(np.clip(x / s, l_min, l_max))
    return float(((q - x) ** 2).sum())


# --------------------------------------------------------------------------- #
# hand-worked examples                                                         #
# --------------------------------------------------------------------------- #
def test_worked_example_codes_sums_gradient_and_packing():
    g = _read_golden("worked_example_sym3.txt")
    x = np.array([[float(v) for v in g["x"]]])
    p = eq.Params(bits=int(g["bits"][0]), group_size=0, n_sigma=float("inf"), iters=0)
    units, x32, _ = _units(x, p)
    assert float(units.r0[0]) == float(g["r0"][0])
    c, s32, A, B, J, grad = units.evaluate(units.r0)
    assert float(s32[0]) == float(g["s0"][0])
    assert c[0].tolist() == [int(v) for v in g["codes"]]
    assert int(A[0]) == int(g["A"][0])
    assert float(B[0]) == float(g["B"][0])
    assert float(J[0]) == float(g["J"][0])
    assert float(J[0]) + float(g["sum_x2"][0]) == float(g["loss"][0])
    # g is d loss / d range; d loss / d s = g * D (chain rule through s = r / D, D = 3)
    assert math.isclose(float(grad[0]) * 3.0, float(g["dloss_ds"][0]), rel_tol=1e-15)
    q = eq.quantize_matrix(_raw16(x), p)
    assert q["u"][0].tolist() == [int(v) for v in g["u"]]
    by = q["codes"].view(np.uint8).reshape(-1)[:3].tolist()
    assert by == [int(v, 16) for v in g["packed_bytes"]]
    # one Adam step
    tr = []
    eq.quantize_matrix(_raw16(x), eq.Params(bits=3, group_size=0, n_sigma=float("inf"), iters=1, lr=1e-3,
                                            select=eq.SELECT_LAST), tr)
    assert float(tr[0][0]) == 0.75
    assert float(tr[1][0]) == float(np.float32(float(g["r1"][0])))


def test_worked_outlier_example():
    g = _read_golden("outlier_example.txt")
    x = np.array([[0.25] * 8 + [-0.25] * 7 + [4.0]])
    p = eq.Params(bits=4, group_size=0, n_sigma=3.0, iters=0)
    units, x32, mask = _units(x, p)
    assert np.nonzero(mask[0])[0].tolist() == [int(g["outlier_index"][0])]
    assert float(units.r0[0]) == float(g["r0"][0])
    # mean / variance as printed in the fixture
    assert x.mean() == float(g["mean"][0]) and x.var() == float(g["variance"][0])
    q = eq.quantize_matrix(_raw16(x), p)
    assert q["out_row_ptr"].tolist() == [0, 1] and q["out_col"].tolist() == [15]
    assert q["out_val"].tolist() == [int(np.float16(4.0).view(np.uint16))]
    # the outlier's code slot holds the zero level
    assert int(q["u"][0, 15]) == 7


def test_sigma_not_variance_reading():
    # With sigma ~ 0.02, n * variance would flag almost everything; Section 5 says < 1 %.
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((64, 1024)) * 0.02).astype(np.float16).astype(np.float32)
    m = eq.outlier_mask(x, 3.0, eq.STAT_ROW, 0)
    assert m.mean() < 0.01


# --------------------------------------------------------------------------- #
# Eq. 3: closed form and bounds                                                #
# --------------------------------------------------------------------------- #
def test_gaussian_three_sigma_tail_mass():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((256, 8192)).astype(np.float32)
    frac = eq.outlier_mask(x, 3.0, eq.STAT_ROW, 0).mean()
    expect = math.erfc(3 / math.sqrt(2))          # 0.26998 %
    n = x.size
    assert abs(frac - expect) < 5 * math.sqrt(expect / n)
    for scope, gs in ((eq.STAT_MATRIX, 0), (eq.STAT_GROUP, 1024)):
        f2 = eq.outlier_mask(x, 3.0, scope, gs).mean()
        assert abs(f2 - expect) < 2e-4


def test_mask_matches_plain_definition_and_chebyshev():
    rng = np.random.default_rng(3)
    x = (rng.standard_t(3, (32, 512)) * 0.05).astype(np.float16).astype(np.float32)
    for n in (1.0, 2.5, 3.0, 6.0):
        m = eq.outlier_mask(x, n, eq.STAT_ROW, 0)
        for r in range(x.shape[0]):
            row = x[r].astype(np.float64)
            ref = np.abs(row - row.mean()) >= n * row.std()          # numpy's own mean / population std
            assert (m[r] == ref).all()
            assert m[r].sum() <= row.size / n ** 2
    # group scope = row scope applied to each group; matrix scope = one row made of everything
    mg = eq.outlier_mask(x, 3.0, eq.STAT_GROUP, 128)
    assert (mg.reshape(-1, 128) == eq.outlier_mask(x.reshape(-1, 128), 3.0, eq.STAT_ROW, 0)).all()
    mm = eq.outlier_mask(x, 3.0, eq.STAT_MATRIX, 0)
    assert (mm.reshape(1, -1) == eq.outlier_mask(x.reshape(1, -1), 3.0, eq.STAT_ROW, 0)).all()
    # Eq. 3 prints >=: a value exactly n sigma from the mean is an outlier (+-a: mean 0, sigma a, all exact)
    pm = np.array([[0.5, -0.5] * 4], np.float32)
    assert eq.outlier_mask(pm, 1.0, eq.STAT_ROW, 0).all()
    assert not eq.outlier_mask(pm, 1.0 + 2.0 ** -10, eq.STAT_ROW, 0).any()
    # constant scope: no outliers; n = infinity: none
    assert not eq.outlier_mask(np.full((2, 64), 0.5, np.float32), 3.0, eq.STAT_ROW, 0).any()
    assert not eq.outlier_mask(x, float("inf"), eq.STAT_ROW, 0).any()


def test_generator_outlier_fraction_in_papers_range():
    lo_hi = [float(l.split()[1]) for l in open(os.path.join(GOLD, "paper_outlier_fractions.txt"))
             if l.strip() and not l.startswith("#")]
    for key in ("c1", "c2", "c3", "c5"):
        rec = eq_inputs.RECIPES[key]
        w = eq_inputs.gen_matrix(128, 4096, rec, seed=5)
        x = w.float().numpy()
        frac = 100 * eq.outlier_mask(x, 3.0, eq.STAT_ROW, 0).mean()
        assert min(lo_hi) * 0.9 < frac < 1.0, (key, frac)
        # every injected outlier (>= 8 sigma_r) is found: the count is at least the injection rate
        assert frac > 100 * rec.p * 0.85


# --------------------------------------------------------------------------- #
# Eq. 1 at a fixed scale: the textbook quantizer                               #
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_rtn_special_case(bits):
    rng = np.random.default_rng(bits)
    x = (rng.standard_normal((16, 256)) * 0.03).astype(np.float16)
    p = eq.Params(bits=bits, group_size=64, n_sigma=float("inf"), iters=0)
    q = eq.quantize_matrix(x.view(np.uint16), p)
    # abs-max round-to-nearest, written out independently
    xg = x.astype(np.float32).reshape(-1, 64)
    D = 2 ** (bits - 1) - 1
    s = np.abs(xg).max(1, keepdims=True) / np.float32(D)
    inv = (np.float32(1) / s).astype(np.float64)
    ref = np.clip(np.rint(xg.astype(np.float64) * inv), -D, D + 1).astype(np.int32) + D
    assert (q["u"].reshape(-1, 64) == ref).all()
    assert (q["scales"].reshape(-1, 1) == s).all()
    assert (q["zero_points"] == D).all()
    assert q["out_row_ptr"][-1] == 0


def test_asymmetric_initialisation():
    x = np.array([[-0.5, 0.25, 1.0, 0.0, 0.75, -0.25, 0.5, 0.125]])
    p = eq.Params(bits=4, group_size=0, mode=eq.ASYMMETRIC, n_sigma=float("inf"), iters=0)
    q = eq.quantize_matrix(_raw16(x), p)
    # range 1.5 over 15 steps: s = 0.1, zero-point = round(0.5 / 0.1) = 5
    assert math.isclose(float(q["scales"][0, 0]), 0.1, rel_tol=1e-6)
    assert int(q["zero_points"][0, 0]) == 5
    # x * 10 = -5 2.5 10 0 7.5 -2.5 5 1.25 ; half-to-even: 2.5 -> 2, 7.5 -> 8, -2.5 -> -2 ; then + 5
    assert q["u"][0].tolist() == [0, 7, 15, 5, 13, 3, 10, 6]
    # all-positive data: the range still includes 0, so zero-point 0
    q2 = eq.quantize_matrix(_raw16(np.abs(x) + 1), p)
    assert int(q2["zero_points"][0, 0]) == 0
    assert float(q2["scales"][0, 0]) == float(np.float32(2.0) / np.float32(15.0))      # range = max - 0, not max - min


# --------------------------------------------------------------------------- #
# Eq. 2: the gradient                                                          #
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("mode", [eq.SYMMETRIC, eq.ASYMMETRIC])
def test_gradient_matches_finite_difference_of_eq1_loss(mode):
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((24, 128)) * 0.02 + (0.01 if mode else 0)).astype(np.float16).astype(np.float64)
    p = eq.Params(bits=4, group_size=0, mode=mode, n_sigma=float("inf"), iters=0)
    units, x32, _ = _units(x, p)
    D = float(units.D)
    checked = 0
    for frac in (1.0, 0.9, 0.8, 0.63):
        r = (units.r0 * np.float32(frac)).astype(np.float32)
        c, s32, A, B, J, g = units.evaluate(r)
        for i in range(x.shape[0]):
            s = float(s32[i])
            lo, hi = float(units.c_lo[i]), float(units.c_hi[i])
            # J is the loss up to the constant sum x^2.  The oracle multiplies by the binary32
            # reciprocal of s where Eq. 1 divides: an element within ~1e-7 of a rounding tie may
            # take the neighbouring level, which moves the loss by a part in ~1e8 at most (the worst
            # case of these rows measures 8.3e-9).
            direct = _loss_eq1(x[i], s, lo, hi)
            assert math.isclose(float(J[i]) + float((x[i] ** 2).sum()), direct, rel_tol=1e-7, abs_tol=1e-15)
            # central difference where no code changes across [s-h, s+h]
            h = s * 1e-6
            cm = np.rint(np.clip(x[i] / (s - h), lo, hi))
            cp = np.rint(np.clip(x[i] / (s + h), lo, hi))
            if not (cm == cp).all():
                continue
            fd = (_loss_eq1(x[i], s + h, lo, hi) - _loss_eq1(x[i], s - h, lo, hi)) / (2 * h)
            assert math.isclose(fd, float(g[i]) * D, rel_tol=1e-5, abs_tol=1e-10), (fd, g[i] * D)
            # on such an interval the loss is quadratic in s with minimiser B / A
            s_star = float(B[i]) / float(A[i])
            assert _loss_eq1(x[i], s_star, -1e9, 1e9) >= 0
            e = s * float(A[i]) - float(B[i])
            assert math.isclose(float(g[i]) * D, 2 * e, rel_tol=1e-12)
            checked += 1
    assert checked > 40


def test_clipped_elements_use_the_clamped_code():
    # one element far outside the range: its code is l_max and it enters A and B as such
    x = np.array([[0.1, -0.1, 0.05, 1.0]])
    p = eq.Params(bits=3, group_size=0, n_sigma=float("inf"), iters=0)
    units, _, _ = _units(x, p)
    r = np.array([0.3], np.float32)                 # s = 0.1 -> 1.0 / 0.1 = 10 clamps to 4
    c, s32, A, B, J, g = units.evaluate(r)
    assert c[0].tolist() == [1, -1, 0, 4]           # 0.5 rounds to even 0
    assert int(A[0]) == 18
    xs = eq.widen(_raw16(x), eq.F16).astype(np.float64)[0]
    assert math.isclose(float(B[0]), float((xs * np.array([1, -1, 0, 4])).sum()), rel_tol=1e-15)


# --------------------------------------------------------------------------- #
# Adam                                                                         #
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("lr", [1e-3, 1e-4])
def test_adam_recurrence_matches_torch_adam(lr):
    rec = eq_inputs.RECIPES["c5"]
    w = eq_inputs.gen_matrix(4, 512, rec, seed=21)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    p = eq.Params(bits=4, group_size=128, iters=120, lr=lr, select=eq.SELECT_LAST)
    trace = []
    eq.quantize_matrix(raw, p, trace)
    x32 = eq.widen(raw, eq.F16)
    units = eq.UnitView(x32, eq.outlier_mask(x32, 3.0, eq.STAT_ROW, 128), p)
    nu = len(units.r0)
    f = lambda v: float(np.float32(v))
    exact = total = 0
    for i in range(nu):
        par = torch.nn.Parameter(torch.tensor([float(trace[0][i])], dtype=torch.float64))
        opt = torch.optim.Adam([par], lr=f(lr), betas=(f(0.9), f(0.999)), eps=f(1e-8))
        for t in range(p.iters):
            r_t = np.float32(par.item())
            assert r_t == trace[t][i]
            one = eq.UnitView(x32.reshape(nu, 128)[i:i + 1], np.zeros((1, 128), bool), p)
            one.xt = units.xt[i:i + 1]; one.c_lo = units.c_lo[i:i + 1]; one.c_hi = units.c_hi[i:i + 1]; one.ulp = units.ulp[i:i + 1]
            g = one.evaluate(np.array([r_t], np.float32))[5][0]
            par.grad = torch.tensor([g], dtype=torch.float64)
            opt.step()
            got = np.float32(max(par.item(), float(units.r0[i]) * 2.0 ** -10))
            want = trace[t + 1][i]
            # torch orders the bias corrections differently (a few 1e-16 relative): the binary32
            # rounding of the range hides that except on a rounding boundary
            assert abs(float(got) - float(want)) <= float(np.spacing(want))
            exact += got == want
            total += 1
            with torch.no_grad():
                par.copy_(torch.tensor([float(want)], dtype=torch.float64))
    assert exact / total > 0.999


def test_first_adam_step_moves_the_range_by_one_learning_rate():
    rec = eq_inputs.RECIPES["c1"]
    w = eq_inputs.gen_matrix(32, 256, rec, seed=2)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    tr = []
    eq.quantize_matrix(raw, eq.Params(bits=4, group_size=0, iters=10, lr=1e-3), tr)
    d1 = np.abs(tr[1].astype(np.float64) - tr[0].astype(np.float64))
    assert np.allclose(d1, 1e-3, rtol=1e-4)
    # Table 10's signature: ~0.9 * 10 * lr in the first ten steps when the gradient keeps its sign
    gold = [l.split() for l in open(os.path.join(GOLD, "paper_table10_range.txt")) if l[0].isdigit()]
    paper_drop = float(gold[0][1]) - float(gold[1][1])
    d10 = tr[0].astype(np.float64) - tr[10].astype(np.float64)
    assert abs(paper_drop - 9e-3) < 1e-9
    assert np.median(d10) > 0.6 * 10 * 1e-3 and d10.max() <= 10 * 1e-3 * 1.05


def test_range_shrinks_then_plateaus_like_table10():
    rec = eq_inputs.RECIPES["c1"]
    w = eq_inputs.gen_matrix(64, 1024, rec, seed=4)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    tr = []
    eq.quantize_matrix(raw, eq.Params(bits=4, group_size=0, iters=400, lr=1e-3, select=eq.SELECT_LAST), tr)
    tr = np.array(tr, np.float64)
    rel = tr / tr[0]
    assert (rel[50] < 0.97).mean() > 0.9                    # shrinks early
    late = np.abs(rel[400] - rel[300])
    early = np.abs(rel[100] - rel[0])
    assert np.median(late) < 0.25 * np.median(early)        # then stabilises


# --------------------------------------------------------------------------- #
# the optimised range against brute force                                      #
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("mode,bits", [(eq.SYMMETRIC, 4), (eq.SYMMETRIC, 3), (eq.ASYMMETRIC, 4)])
def test_optimised_range_vs_brute_force_scan(mode, bits):
    rec = eq_inputs.RECIPES["c1"]
    w = eq_inputs.gen_matrix(24, 128, rec, seed=9 + bits)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    p = eq.Params(bits=bits, group_size=0, mode=mode, iters=300, lr=5e-4)
    q = eq.quantize_matrix(raw, p)
    x32 = eq.widen(raw, eq.F16)
    units = eq.UnitView(x32, q["mask"], p)
    D = float(units.D)
    ratios = []
    for i in range(raw.shape[0]):
        x = units.xt[i].astype(np.float64)[~q["mask"][i]]
        lo, hi = float(units.c_lo[i]), float(units.c_hi[i])
        s0 = float(np.float32(units.r0[i]) / np.float32(D))
        s_ch = float(q["scales"][i, 0])
        l0 = _loss_eq1(x, s0, lo, hi)
        lc = _loss_eq1(x, s_ch, lo, hi)
        assert lc <= l0 * (1 + 1e-9)                            # never worse than plain min/max scaling
        grid = min(_loss_eq1(x, s0 * f, lo, hi) for f in np.linspace(0.3, 1.2, 1801))
        assert lc >= grid * (1 - 1e-3) or lc - grid < 1e-12   # a scan cannot be beaten by much (sanity of the scan)
        ratios.append(lc / grid)
    # the loss is piecewise quadratic, so a gradient method may stop in a local minimum: the
    # typical unit lands close to the scanned global optimum, none is required to reach it
    assert np.median(ratios) < 1.05, (np.median(ratios), max(ratios))


@pytest.mark.parametrize("iters,lr", [(3, 1e-3), (60, 2e-3)])
def test_best_iterate_is_the_argmin_over_the_trajectory(iters, lr):
    """The returned range is the iterate r_0 .. r_T with the smallest Eq. 1 loss, the loss recomputed
    here from its definition.  Few small steps: the last iterate is the best one in some units;
    many larger ones: Adam dithers and an earlier iterate wins."""
    rec = eq_inputs.RECIPES["c1"]
    w = eq_inputs.gen_matrix(16, 128, rec, seed=21)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    p = eq.Params(bits=4, group_size=0, iters=iters, lr=lr)
    tr = []
    q = eq.quantize_matrix(raw, p, tr)
    tr = np.array(tr)                                   # (T + 1) x units, binary32
    assert tr.shape == (iters + 1, 16)
    units = eq.UnitView(eq.widen(raw, eq.F16), q["mask"], p)
    D = np.float32(units.D)
    where = []
    for i in range(16):
        x = units.xt[i].astype(np.float64)[~q["mask"][i]]
        lo, hi = float(units.c_lo[i]), float(units.c_hi[i])
        losses = [_loss_eq1(x, float(np.float32(r) / D), lo, hi) for r in tr[:, i]]
        chosen = _loss_eq1(x, float(q["scales"][i, 0]), lo, hi)
        assert chosen <= min(losses) * (1 + 1e-9) + 1e-15
        assert any(np.float32(q["range"][i, 0]) == np.float32(r) for r in tr[:, i])
        where.append(int(np.argmin(losses)))
    if iters == 3:
        assert where.count(iters) >= 2                  # the iterate after the last step can win
    else:
        assert sum(1 for k in where if 0 < k < iters) >= 8   # ... and so can one in the middle


def test_range_never_drops_below_its_floor():
    """A learning rate far above the range: the first step would make the range negative; it stops
    at r0 / 1024 and stays finite and positive from there on."""
    x = np.array([[0.75] + [0.4375] * 7])               # rounds up at r0: sum (Q - x) c > 0, the range shrinks
    p = eq.Params(bits=3, group_size=0, n_sigma=float("inf"), iters=4, lr=10.0, select=eq.SELECT_LAST)
    tr = []
    eq.quantize_matrix(_raw16(x), p, tr)
    tr = np.array(tr, np.float64).reshape(-1)
    assert tr[0] == 0.75 and tr[1] == 0.75 * 2.0 ** -10
    assert np.isfinite(tr).all() and (tr >= 0.75 * 2.0 ** -10).all()


def test_select_last_is_the_final_iterate_and_best_is_no_worse():
    rec = eq_inputs.RECIPES["c2"]
    w = eq_inputs.gen_matrix(8, 512, rec, seed=13)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    tr = []
    ql = eq.quantize_matrix(raw, eq.Params(bits=4, group_size=128, iters=50, select=eq.SELECT_LAST), tr)
    assert (ql["range"].reshape(-1) == tr[-1]).all()
    qb = eq.quantize_matrix(raw, eq.Params(bits=4, group_size=128, iters=50, select=eq.SELECT_BEST))
    p = eq.Params(bits=4, group_size=128)
    sl = eq.reconstruction_sse(raw, eq.dequantize(ql, 8, 512, p), eq.F16)
    sb = eq.reconstruction_sse(raw, eq.dequantize(qb, 8, 512, p), eq.F16)
    q0 = eq.quantize_matrix(raw, eq.Params(bits=4, group_size=128, iters=0))
    s0 = eq.reconstruction_sse(raw, eq.dequantize(q0, 8, 512, p), eq.F16)
    # the 16-bit rounding of the reconstruction adds noise of relative size ~1e-3 to these sums
    assert (sb <= s0 * 1.002).all() and (sb <= sl * 1.002).all()
    assert sb.sum() < 0.95 * s0.sum()


# --------------------------------------------------------------------------- #
# invariants of the whole path                                                 #
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("dtype,mode,bits,G", [(eq.F16, eq.SYMMETRIC, 4, 128), (eq.BF16, eq.SYMMETRIC, 4, 128),
                                                (eq.F16, eq.ASYMMETRIC, 4, 0), (eq.F16, eq.SYMMETRIC, 3, 128),
                                                (eq.F16, eq.SYMMETRIC, 8, 32)])
def test_invariants(dtype, mode, bits, G):
    rec = eq_inputs.with_dtype(eq_inputs.RECIPES["c3"], "f16" if dtype == eq.F16 else "bf16")
    rows, cols = 48, 1024
    w = eq_inputs.gen_matrix(rows, cols, rec, seed=17)
    raw = w.view(torch.int16).numpy().view(np.uint16)
    p = eq.Params(dtype=dtype, bits=bits, group_size=G, mode=mode, iters=30)
    q = eq.quantize_matrix(raw, p)
    L = 2 ** bits - 1
    assert q["u"].max() <= L
    assert q["codes"].shape == (rows, (cols * bits + 31) // 32)
    assert (eq.unpack_codes(q["codes"], cols, bits) == q["u"]).all()
    # CSR outlier list: sorted, counted, raw values verbatim
    rp = q["out_row_ptr"].astype(np.int64)
    assert rp[0] == 0 and (np.diff(rp) >= 0).all() and rp[-1] == len(q["out_col"]) == len(q["out_val"]) == q["mask"].sum()
    for r in range(rows):
        cc = q["out_col"][rp[r]:rp[r + 1]]
        assert (np.diff(cc.astype(np.int64)) > 0).all()
        assert (raw[r, cc] == q["out_val"][rp[r]:rp[r + 1]]).all()
        assert (np.nonzero(q["mask"][r])[0] == cc).all()
    deq = eq.dequantize(q, rows, cols, p)
    assert (deq[q["mask"]] == raw[q["mask"]]).all()           # outliers reproduced bit-exactly
    # un-clipped normal values sit within half a step of their reconstruction
    Gs = G if G else cols
    x32 = eq.widen(raw, dtype)
    s = np.repeat(q["scales"], Gs, axis=1).astype(np.float64)
    z = np.repeat(q["zero_points"].astype(np.int64), Gs, axis=1)
    c = q["u"].astype(np.int64) - z
    t = x32.astype(np.float64) / s
    unclipped = (~q["mask"]) & (t >= (-z) - 0.5) & (t <= (L - z) + 0.5)
    err = np.abs(s * c - x32)
    assert (err[unclipped] <= 0.5 * s[unclipped] * (1 + 2.0 ** -20)).all()
    clipped = (~q["mask"]) & ~unclipped
    assert ((c[clipped] == -z[clipped]) | (c[clipped] == L - z[clipped])).all()
    assert (q["u"][q["mask"]] == z[q["mask"]]).all()          # outlier slots hold the zero level


def test_degenerate_units():
    p = eq.Params(bits=4, group_size=32, iters=5)
    raw = np.zeros((2, 64), np.uint16)
    raw[1, :32] = np.float16(0.5).view(np.uint16)              # constant group: sigma_row > 0 though
    q = eq.quantize_matrix(raw, p)
    assert q["scales"][0].tolist() == [1.0, 1.0] and (q["u"][0] == 7).all()
    assert q["out_row_ptr"][-1] == 0
    # empty matrix
    q = eq.quantize_matrix(np.zeros((0, 64), np.uint16), p)
    assert q["codes"].shape == (0, 8) and q["out_row_ptr"].tolist() == [0]
    with pytest.raises(ValueError):
        eq.quantize_matrix(np.full((1, 64), 0x7C00, np.uint16), p)   # +inf
    with pytest.raises(ValueError):
        eq.quantize_matrix(raw, eq.Params(bits=4, group_size=32, iters=5, eps=0.0))


def test_pack_unpack_and_bf16_rounding_against_torch():
    rng = np.random.default_rng(0)
    for bits in range(2, 9):
        u = rng.integers(0, 2 ** bits, (5, 72)).astype(np.uint8)
        w = eq.pack_codes(u, bits)
        assert (eq.unpack_codes(w, 72, bits) == u).all()
        # 4-bit: even element in the low nibble
    u = np.array([[1, 2, 3, 4, 5, 6, 7, 8]], np.uint8)
    assert eq.pack_codes(u, 4).view(np.uint8).tolist() == [[0x21, 0x43, 0x65, 0x87]]
    x = (rng.standard_normal(4096) * 3).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]     # ties and a subnormal
    mine = eq.narrow(x, eq.BF16)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (mine == ref).all()
    assert (eq.widen(mine, eq.BF16) == torch.from_numpy(x).to(torch.bfloat16).float().numpy()).all()
    h = rng.integers(0, 0x7C00, 2048).astype(np.uint16)
    assert (eq.widen(h, eq.F16) == torch.from_numpy(h.view(np.int16)).view(torch.float16).float().numpy()).all()
    assert (eq.narrow(eq.widen(h, eq.F16), eq.F16) == h).all()


def test_exact_dot_falls_back_to_exact_summation():
    # a bf16 unit with a 2^60 exponent span: a plain binary64 accumulation would round
    big, tiny = 2.0 ** 30, 2.0 ** -40
    prod = np.array([[big, tiny, -big, tiny]], np.float32)
    got = eq._exact_dot(prod, np.array([2.0 ** -47]))
    assert got[0] == 2.0 ** -39


def test_dequant_matvec_is_the_reconstruction_times_the_vector():
    """Unit vectors pick out the columns of the (already pinned) reconstruction, and a hand-worked
    2 x 8 case: codes 0..7 at zero-point 3 and scale 0.5 give (-1.5 .. 2), one outlier replaces
    column 6 by 10; with x = (1, ..., 1) the first row sums to 2 - 1.5 + 10 = 10.5."""
    p = eq.Params(bits=4, group_size=0)
    u = np.stack([np.arange(8), np.full(8, 3)]).astype(np.int64)
    u[0, 6] = 3                                                   # an outlier's slot holds the zero level
    q = {"codes": eq.pack_codes(u, 4), "scales": np.full((2, 1), 0.5, np.float32),
         "zero_points": np.full((2, 1), 3, np.uint8), "out_row_ptr": np.array([0, 1, 1], np.uint32),
         "out_col": np.array([6], np.uint32), "out_val": eq.narrow(np.array([10.0], np.float32), eq.F16)}
    ones = eq.narrow(np.ones(8, np.float32), eq.F16)
    y = eq.dequant_matvec(q, 2, 8, p, ones)
    assert y.tolist() == [10.5, 0.0]
    W = eq.widen(eq.dequantize(q, 2, 8, p), eq.F16).astype(np.float64)
    for j in range(8):
        e = np.zeros(8, np.float32)
        e[j] = 2.0
        assert np.array_equal(eq.dequant_matvec(q, 2, 8, p, eq.narrow(e, eq.F16)), 2.0 * W[:, j])


def test_rounding_ties_go_to_the_even_level():
    """Eq. 1 rounds to nearest; an exact tie goes to the even level (the reading taken for the
    rounding operator).  Scale 2^-7 exactly (largest magnitude 7 * 2^-7, 4-bit symmetric), values
    at every half level -7.0, -6.5, ..., 7.0: worked by hand, level + zero-point 7."""
    half_levels = np.arange(-14, 15) / 2.0
    x = np.zeros((1, 128), np.float32)
    x[0, :29] = half_levels * 2.0 ** -7
    q = eq.quantize_matrix(eq.narrow(x, eq.F16), eq.Params(bits=4, group_size=0, iters=0, n_sigma=float("inf")))
    assert q["scales"][0, 0] == np.float32(2.0 ** -7)
    expect = [0, 1, 1, 1, 2, 3, 3, 3, 4, 5, 5, 5, 6, 7, 7, 7, 8, 9, 9, 9, 10, 11, 11, 11, 12, 13, 13, 13, 14]
    assert q["u"][0, :29].tolist() == expect
    assert (q["u"][0, 29:] == 7).all()
