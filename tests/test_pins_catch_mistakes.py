"""The pins of the CPU oracle, tested themselves: every planted mistake must fail one of them.

Each entry below rewrites one expression of ``oracle/easyquant_oracle.py`` into a plausible error
(a dropped term, a wrong sign, a transposed index, a different rounding, a different reading of
the paper).  The mutated copy is placed ahead of the real package on the import path
(tests/conftest.py, EASYQUANT_ORACLE_UNDER_TEST) and ``tests/test_oracle_pins.py`` runs against it
in a child process: it has to fail.  Everything here runs on the CPU.
"""
import concurrent.futures as cf
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle", "easyquant_oracle.py")

# (name, text as it stands in the oracle, text with the mistake)
MISTAKES = [
 ("ge_to_gt", "np.abs(d) >= n * sigma", "np.abs(d) > n * sigma"),
 ("sample_variance", "sigma = np.sqrt((d * d).sum(axis=1, keepdims=True) / cnt)", "sigma = np.sqrt((d * d).sum(axis=1, keepdims=True) / (cnt - 1))"),
 ("variance_not_sigma", "sigma = np.sqrt((d * d).sum(axis=1, keepdims=True) / cnt)", "sigma = (d * d).sum(axis=1, keepdims=True) / cnt"),
 ("mean_dropped", "d = v - mu", "d = v"),
 ("sigma_zero_guard", "m = (sigma > 0) & (np.abs(d) >= n * sigma)", "m = (np.abs(d) >= n * sigma)"),
 ("group_scope_is_row", "v = x.reshape(rows * (cols // group_size), group_size)", "v = x"),
 ("matrix_scope_is_row", "v = x.reshape(1, -1)", "v = x"),
 ("sym_D", "self.D = _f32((1 << (p.bits - 1)) - 1)", "self.D = _f32(1 << (p.bits - 1))"),
 ("sym_z", "z = np.full(nu, (1 << (p.bits - 1)) - 1, np.int32)", "z = np.full(nu, (1 << (p.bits - 1)), np.int32)"),
 ("r0_signed_max", "r0 = np.abs(xt).max(axis=1).astype(_f32)", "r0 = xt.max(axis=1).astype(_f32)"),
 ("outliers_stay_in_unit", "xt = np.where(mask, _f32(0), x32).reshape", "xt = x32.reshape"),
 ("asym_lo_without_zero", "lo = np.minimum(xt.min(axis=1), _f32(0))", "lo = xt.min(axis=1)"),
 ("asym_z_sign", "zf = np.rint((-lo) / s0)", "zf = np.rint(lo / s0)"),
 ("asym_D", "self.D = _f32(L)", "self.D = _f32(L + 1)"),
 ("no_clamp", "tc = np.minimum(np.maximum(t, self.c_lo.astype(_f64)[:, None]), self.c_hi.astype(_f64)[:, None])", "tc = t"),
 ("round_half_up", "c = np.rint(tc).astype(_f32)", "c = np.floor(tc + 0.5).astype(_f32)"),
 ("truncate", "c = np.rint(tc).astype(_f32)", "c = np.trunc(tc).astype(_f32)"),
 ("A_not_squared", "A = (ci * ci).sum(axis=1)", "A = np.abs(ci).sum(axis=1)"),
 ("e_sign", "e = s * A.astype(_f64) - B", "e = s * A.astype(_f64) + B"),
 ("J_sign", "J = s * (e - B)", "J = s * (e + B)"),
 ("g_factor2", "g = (_f64(2.0) * e) / _f64(D)", "g = e / _f64(D)"),
 ("g_chain_rule", "g = (_f64(2.0) * e) / _f64(D)", "g = _f64(2.0) * e"),
 ("scale_is_range", "s32 = (r32 / D).astype(_f32)", "s32 = r32.astype(_f32)"),
 ("adam_m", "m = b1 * m + (_f64(1.0) - b1) * g", "m = b1 * m + g"),
 ("adam_v", "v = b2 * v + (_f64(1.0) - b2) * (g * g)", "v = b2 * v + (_f64(1.0) - b2) * np.abs(g)"),
 ("adam_bias1", "mh = m / (_f64(1.0) - p1)", "mh = m"),
 ("adam_bias2", "vh = v / (_f64(1.0) - p2)", "vh = v"),
 ("adam_eps_inside", "(np.sqrt(vh) + eps)", "np.sqrt(vh + eps)"),
 ("adam_ascent", "r64 = r32.astype(_f64) - lr *", "r64 = r32.astype(_f64) + lr *"),
 ("adam_betas_swapped", "p1 = p1 * b1\n        p2 = p2 * b2", "p1 = p1 * b2\n        p2 = p2 * b1"),
 ("no_floor", "r_new = np.maximum(r64, floor_r).astype(_f32)", "r_new = r64.astype(_f32)"),
 ("best_is_worst", "better = J < J_best\n        J_best", "better = J > J_best\n        J_best"),
 ("best_skips_last", "        _, _, _, _, J, _ = units.evaluate(r32)\n        better = J < J_best\n        r_best = np.where(better, r32, r_best)\n        return r_best", "        return r_best"),
 ("last_returns_best", "    if p.select == SELECT_LAST:\n        return r32", "    if p.select == SELECT_LAST:\n        return r_best"),
 ("codes_without_z", "u = (c + units.z[:, None]).reshape(rows, cols)", "u = (c + 0 * units.z[:, None]).reshape(rows, cols) % (1 << p.bits)"),
 ("pack_big_endian_bits", 'by = np.packbits(stream, axis=1, bitorder="little")', 'by = np.packbits(stream, axis=1, bitorder="big")'),
 ("row_ptr_inclusive", "row_ptr[1:] = np.cumsum(counts)", "row_ptr[:-1] = np.cumsum(counts)"),
 ("outlier_value_rounded", '"out_val": raw[rr, cc].astype(np.uint16)', '"out_val": narrow(widen(raw[rr, cc], p.dtype) * _f32(1.0009765625), p.dtype)'),
 ("deq_z_sign", "xh = (s * (u - z).astype(_f32)).astype(_f32)", "xh = (s * (u + z).astype(_f32)).astype(_f32)"),
 ("deq_no_outliers", '    out[rr, q["out_col"].astype(np.int64)] = q["out_val"]\n', ""),
 ("bf16_truncates", "r = (b + np.uint64(0x7FFF) + lsb) >> np.uint64(16)", "r = b >> np.uint64(16)"),
 ("emit_at_r0", "c, s32, _, _, _, _ = units.evaluate(r)", "c, s32, _, _, _, _ = units.evaluate(units.r0)"),
 ("matvec_transposed", "return W @ x", "return W.T @ x if rows == cols else (W @ x)[::-1]"),
 ("sym_top_level_missing", "self.c_hi = (L - self.z).astype(_f32)", "self.c_hi = (L - self.z - (1 if p.mode == SYMMETRIC else 0)).astype(_f32)"),
 ("floor_factor", "floor_r = r0.astype(_f64) * _f64(2.0 ** -10)", "floor_r = r0.astype(_f64) * _f64(2.0 ** -8)"),
 ("hyperparameters_not_binary32", "lr, b1, b2, eps = (_f64(_f32(v)) for v in (p.lr, p.beta1, p.beta2, p.eps))", "lr, b1, b2, eps = (_f64(v) for v in (p.lr, p.beta1, p.beta2, p.eps))"),
 ("outlier_counts_by_column", "counts = mask.sum(axis=1)", "counts = mask.sum(axis=0)[:rows] if rows <= cols else mask.sum(axis=1)"),
 ("outlier_index_is_row", '"out_col": cc.astype(np.uint32)', '"out_col": rr.astype(np.uint32)'),
 ("deq_scale_of_first_group", "s = np.repeat(q[\"scales\"].astype(_f32).reshape(rows, cols // G), G, axis=1)", "s = np.repeat(q[\"scales\"].astype(_f32).reshape(rows, cols // G)[:, :1], cols, axis=1)"),
 ("deq_levels_not_centred", "xh = (s * (u - z).astype(_f32)).astype(_f32)", "xh = (s * (u - z + 0.5).astype(_f32)).astype(_f32)"),
 ("bf16_widen_shift", "return (raw.astype(np.uint32) << np.uint32(16)).view(_f32)", "return (raw.astype(np.uint32) << np.uint32(15)).view(_f32)"),
 ("unpack_msb_first", 'stream = np.unpackbits(by, axis=1, bitorder="little")', 'stream = np.unpackbits(by, axis=1, bitorder="big")'),
 ("reciprocal_of_range", "inv32 = (_f32(1.0) / s32).astype(_f32)", "inv32 = (_f32(1.0) / r32).astype(_f32)"),
 ("B_with_unclamped_level", "B = _exact_dot((self.xt * c).astype(_f32), self.ulp)", "B = _exact_dot((self.xt * np.rint(t).astype(_f32)).astype(_f32), self.ulp)"),
 ("sse_without_square", "return (d * d).sum(axis=1)", "return np.abs(d).sum(axis=1)"),
]


def _run_pins_against(text):
    d = tempfile.mkdtemp(prefix="eq_oracle_")
    try:
        os.makedirs(os.path.join(d, "oracle"))
        open(os.path.join(d, "oracle", "__init__.py"), "w").close()
        with open(os.path.join(d, "oracle", "easyquant_oracle.py"), "w") as f:
            f.write(text)
        env = dict(os.environ, EASYQUANT_ORACLE_UNDER_TEST=d)
        r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                            "-p", "no:cacheprovider"], env=env, capture_output=True, text=True, cwd=ROOT, timeout=600)
        return r.returncode, r.stdout[-400:]
    finally:
        shutil.rmtree(d, ignore_errors=True)


def test_every_planted_mistake_fails_a_pin():
    src = open(ORACLE).read()
    texts = []
    for name, good, bad in MISTAKES:
        assert src.count(good) == 1, f"{name}: the oracle no longer contains this expression exactly once"
        mutated = src.replace(good, bad)
        compile(mutated, name, "exec")                    # still a valid module: the pins fail, not the import
        texts.append(mutated)
    # the unchanged copy passes through the same route (so a failure below is the mistake's doing)
    with cf.ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        results = list(ex.map(_run_pins_against, [src] + texts))
    rc0, tail0 = results[0]
    assert rc0 == 0, tail0
    survivors = [name for (name, _, _), (rc, _) in zip(MISTAKES, results[1:]) if rc == 0]
    broken = [(name, rc, tail) for (name, _, _), (rc, tail) in zip(MISTAKES, results[1:]) if rc not in (0, 1)]
    assert not broken, broken                             # 1 = tests failed; anything else is the harness
    assert not survivors, f"no pin notices: {survivors}"
