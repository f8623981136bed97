"""The C-ABI library loads and exports every symbol that include/easyquant.h declares.
Host-only entry points are also exercised (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "easyquant.h")).read()
    return sorted(set(re.findall(r"EQ_API\s+[\w\s\*]+?\b(eq_\w+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2403_02775_amd as eqg
    if not os.path.exists(eqg.lib_path()):
        from paper_2403_02775_amd.build import build
        build()
    return eqg.lib()


def test_header_declares_the_three_entry_points():
    names = _declared()
    for n in ("eq_quantize_matrix", "eq_quantize_batch", "eq_dequantize"):
        assert n in names
    assert len(names) >= 9


def test_every_declared_symbol_is_exported(lib):
    for name in _declared():
        assert hasattr(lib, name), name


def test_host_only_helpers(lib):
    import paper_2403_02775_amd as eqg
    assert eqg.eq_code_words_per_row(4096, 4) == 512
    assert eqg.eq_code_words_per_row(4096, 3) == 384
    assert eqg.eq_code_words_per_row(8, 3) == 1
    # Chebyshev: at most cols / n^2 elements of a row can lie n sigma from its mean
    assert eqg.eq_outlier_capacity_bound(10, 900, 3.0) == 10 * 101
    assert eqg.eq_outlier_capacity_bound(10, 900, 0.5) == 9000
    assert eqg.eq_outlier_capacity_bound(0, 900, 3.0) == 0
    assert eqg.eq_strerror(0) == "ok" and "NULL" in eqg.eq_strerror(-1)
    p = eqg.Params(group_size=128)
    assert eqg.eq_workspace_bytes([4096], [4096], [1000], p) > 4096 * 8 + 6000
    assert eqg.eq_workspace_bytes([4096], [4096], [1000], eqg.Params(bits=9)) == 0
    cp = eqg.binding._CParams()
    lib.eq_default_params(ctypes.byref(cp))
    assert (cp.bits, cp.group_size, cp.mode, cp.iters, cp.select) == (4, 0, 0, 100, 0)
    assert abs(cp.n_sigma - 3.0) < 1e-7 and abs(cp.lr - 1e-3) < 1e-9


def test_argument_errors_are_reported_without_a_gpu(lib):
    import paper_2403_02775_amd as eqg
    B = eqg.binding
    cp = eqg.Params().c()
    q = B._CQMatrix()
    # NULL output struct / NULL parameter block
    assert lib.eq_quantize_matrix(None, 8, 8, 8, ctypes.byref(cp), None, None, 0, None) == -1
    assert lib.eq_quantize_matrix(None, 8, 8, 8, None, ctypes.byref(q), None, 0, None) == -1
    bad = eqg.Params(bits=1).c()
    assert lib.eq_quantize_matrix(None, 8, 8, 8, ctypes.byref(bad), ctypes.byref(q), None, 0, None) == -3
    # hyper-parameters out of range: epsilon must be positive, the moments' decay below 1, lr finite
    for kw in ({"eps": 0.0}, {"beta1": 1.0}, {"beta2": -0.1}, {"lr": float("inf")}, {"n_sigma": float("nan")}, {"iters": -1}):
        badp = eqg.Params(**kw).c()
        assert lib.eq_quantize_matrix(None, 8, 8, 8, ctypes.byref(badp), ctypes.byref(q), None, 0, None) == -3, kw
    # cols not a multiple of 8, ld < cols, group that does not divide cols, row too long
    assert lib.eq_quantize_matrix(None, 8, 12, 16, ctypes.byref(cp), ctypes.byref(q), None, 0, None) == -2
    assert lib.eq_quantize_matrix(None, 8, 16, 8, ctypes.byref(cp), ctypes.byref(q), None, 0, None) == -2
    g = eqg.Params(group_size=96).c()
    assert lib.eq_quantize_matrix(None, 8, 128, 128, ctypes.byref(g), ctypes.byref(q), None, 0, None) == -2
    assert lib.eq_quantize_matrix(None, 8, 1 << 20, 1 << 20, ctypes.byref(cp), ctypes.byref(q), None, 0, None) == -6
    assert lib.eq_dequantize(None, 8, 8, ctypes.byref(cp), None, 8, None) == -1
    assert lib.eq_quantize_batch(0, None, None, None, None, None, None, None, 0, None) == 0


def test_noalloc_entry_point_rejects_what_does_not_fit_its_scratch(lib):
    """Checked on the host before any HIP call, so no GPU is needed (the pointers are never dereferenced)."""
    import paper_2403_02775_amd as eqg
    gp = eqg.Params(group_size=128, iters=1)
    rows, cols = 8192, 8192
    cap = eqg.eq_outlier_capacity_bound(rows, cols, gp.n_sigma)     # 11 % of the elements: 45 MB of staging
    assert eqg.eq_workspace_bytes([rows], [cols], [cap], gp) > eqg.EQ_STATIC_SCRATCH_BYTES
    text = open(os.path.join(ROOT, "include", "easyquant.h")).read()
    assert re.search(r"#define\s+EQ_STATIC_SCRATCH_BYTES\s+\(32u \* 1024u \* 1024u\)", text) and eqg.EQ_STATIC_SCRATCH_BYTES == 32 << 20
    cp = gp.c()
    q = eqg.binding._CQMatrix(1 << 20, 1 << 20, 1 << 20, 1 << 20, 1 << 20, 1 << 20, cap, 1 << 20)
    rc = lib.eq_quantize_matrix_noalloc(1 << 20, rows, cols, cols, ctypes.byref(cp), ctypes.byref(q), None)
    assert rc == -8 and "scratch" in eqg.eq_strerror(rc)
    assert lib.eq_quantize_matrix_noalloc(1 << 20, rows, cols, cols, ctypes.byref(cp), None, None) == -1
    bad = eqg.Params(bits=9).c()
    assert lib.eq_quantize_matrix_noalloc(1 << 20, rows, cols, cols, ctypes.byref(bad), ctypes.byref(q), None) == -3


def test_header_is_plain_c_and_links_from_a_c_program(lib, tmp_path):
    """The boundary is a C ABI: the header compiles as C99 and a C program linked against the
    library can call it (host-only entry points here; nothing touches a GPU)."""
    import shutil
    import subprocess
    import paper_2403_02775_amd as eqg
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_abi.c"
    src.write_text(r"""
#include <stdio.h>
#include "easyquant.h"
int main(void) {
  eq_params p;
  eq_default_params(&p);
  eq_qmatrix q = {0};
  int rc = eq_quantize_matrix(NULL, 8, 12, 16, &p, &q, NULL, 0, NULL);   /* cols not a multiple of 8 */
  printf("%d %d %lld %d %s\n", p.bits, p.iters, (long long)eq_code_words_per_row(4096, 3), rc, eq_strerror(rc));
  return 0;
}
""")
    exe = tmp_path / "use_abi"
    libdir = os.path.dirname(eqg.lib_path())
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-leasyquant", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split(None, 4)
    assert out[:4] == ["4", "100", "384", "-2"] and "rows" in out[4]
