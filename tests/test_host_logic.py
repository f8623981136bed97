"""Host-side logic of the library that can be checked without a GPU."""
import ctypes
import math
import os
from fractions import Fraction

import numpy as np
import pytest


@pytest.fixture(scope="module")
def lib():
    import paper_2403_02775_amd as eqg
    if not os.path.exists(eqg.lib_path()):
        from paper_2403_02775_amd.build import build
        build()
    return eqg.lib()


def test_division_by_known_reciprocal_is_the_ieee_quotient(lib):
    """The multiply-add sequence the kernels use for m / (1 - beta^t), v / (1 - beta^t), 2e / D and
    r / D must return the correctly rounded quotient.  Checked against exact rational arithmetic
    (Fraction -> float is correctly rounded) and against the hardware division."""
    rng = np.random.default_rng(0)
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    divisors = [7.0, 15.0, 3.0, 1.0, 127.0, 255.0]
    p1 = p2 = 1.0
    for _ in range(500):
        p1 *= b1
        p2 *= b2
        divisors += [1.0 - p1, 1.0 - p2]
    n = 0
    for b in divisors:
        for a in np.concatenate([rng.standard_normal(40) * 10.0 ** rng.integers(-12, 6, 40), [0.0, -0.0, 1e-300, 3e280]]):
            a = float(a)
            got = lib.eq_test_div_f64(a, b)
            want = a / b
            assert got == want or (math.isnan(got) and math.isnan(want)), (a, b, got, want)
            if a != 0 and abs(a) < 1e200 and abs(a) > 1e-200:
                assert got == float(Fraction(a) / Fraction(b))
            n += 1
    assert n > 40000
    for b in (7.0, 15.0, 3.0, 1.0, 127.0, 255.0):
        a32 = (rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 3, 20000)).astype(np.float32)
        for a in a32[:3000]:
            got = lib.eq_test_div_f32(ctypes.c_float(float(a)), ctypes.c_float(b))
            assert np.float32(got) == np.float32(a) / np.float32(b), (a, b)


def test_work_split_override_does_not_change_workspace_contract(lib):
    import paper_2403_02775_amd as eqg
    p = eqg.Params(group_size=128)
    a = eqg.eq_workspace_bytes([4096], [4096], [100000], p)
    with eqg.override(eqg.OVR_UNITS_PER_ITEM, 100000):
        b = eqg.eq_workspace_bytes([4096], [4096], [100000], p)
    with eqg.override(eqg.OVR_UNITS_PER_ITEM, 256):
        c = eqg.eq_workspace_bytes([4096], [4096], [100000], p)
    assert a > 0 and b > 0 and c >= a
    assert eqg.eq_workspace_bytes([4096], [4096], [100000], p) == a      # the override is gone


def test_plan_items_cover_every_row_exactly_once(lib):
    """Host side of the batch call: the work items of the launch plan tile the rows of every
    matrix that a lane kernel serves, in order, without gaps or overlaps."""
    import paper_2403_02775_amd as eqg
    shapes = [(8192, 8192), (22016, 8192), (8192, 22016), (100, 4096), (7, 1024), (0, 4096), (33, 256)]
    rows, cols = [s[0] for s in shapes], [s[1] for s in shapes]
    for p in (eqg.Params(group_size=128, iters=100), eqg.Params(group_size=128, iters=0), eqg.Params(group_size=0, iters=10)):
        items = eqg.plan_items(rows, cols, [1000] * len(shapes), p)
        covered = {m: np.zeros(r, np.int32) for m, r in enumerate(rows)}
        launches = {}
        for m, r0, nr, stride, step, launch in items:
            assert nr > 0 and 0 <= r0 and r0 + nr <= rows[m], (m, r0, nr)
            if stride == 0:
                covered[m][r0:r0 + nr] += 1
            else:
                assert step > 0 and stride % step == 0 and r0 + nr == rows[m]
                for a in range(r0, rows[m], stride):
                    covered[m][a:a + step] += 1
            launches.setdefault(launch, set()).add(cols[m])
        for launch, cs in launches.items():
            assert len(cs) == 1                                        # one row length per launch
        for m, (r, c) in enumerate(shapes):
            served_by_lanes = r > 0 and ((p.group_size == 128) or (c % 128 == 0 and 2048 <= c <= 32768))
            assert (covered[m] == (1 if served_by_lanes else 0)).all(), (m, r, c, p.group_size)


def test_sorted_evaluation_chunks_cover_their_rows_and_fit_the_record_region(lib):
    """Host side of the sorted evaluation of per-channel rows: the segments of all chunks tile the rows of
    every eligible matrix once, a chunk holds one row length, its records lie back to back inside the
    region the workspace reserves, and the groups of 4 rows are counted per segment."""
    import paper_2403_02775_amd as eqg
    shapes = [(8192, 8192), (22016, 8192), (8192, 22016), (100, 4096), (7, 1024), (0, 4096), (33, 2048), (5, 8192)]
    rows, cols = [s[0] for s in shapes], [s[1] for s in shapes]
    caps = [1000] * len(shapes)

    def record_bytes(c):
        return 64 + 32 * (c // 8)                        # header, then 32 bytes per chunk of 8 values

    for chunk_rows in (0, 1000, 6):
        eqg.set_override(eqg.OVR_SORT_CHUNK_ROWS, chunk_rows)
        try:
            p = eqg.Params(group_size=0, iters=400, bits=4)
            segs, region = eqg.plan_sort_segments(rows, cols, caps, p)
            with_region = eqg.eq_workspace_bytes(rows, cols, caps, p)
            eqg.set_override(eqg.OVR_SORTED_ROWS, 1)
            without = eqg.eq_workspace_bytes(rows, cols, caps, p)
            assert eqg.plan_sort_segments(rows, cols, caps, p)[0] == []
            eqg.set_override(eqg.OVR_SORTED_ROWS, 0)
        finally:
            eqg.set_override(eqg.OVR_SORT_CHUNK_ROWS, 0)
            eqg.set_override(eqg.OVR_SORTED_ROWS, 0)
        assert with_region > region > 0 and with_region > without      # (the two plans also differ in their work items)
        covered = {m: np.zeros(r, np.int32) for m, r in enumerate(rows)}
        by_chunk = {}
        for chunk, m, r0, nr, g0, first_row, off in segs:
            assert nr > 0 and 0 <= r0 and r0 + nr <= rows[m]
            covered[m][r0:r0 + nr] += 1
            by_chunk.setdefault(chunk, []).append((m, nr, g0, first_row, off))
        for m, (r, c) in enumerate(shapes):
            eligible = r > 0 and c % 128 == 0 and 2048 <= c <= 32768
            assert (covered[m] == (1 if eligible else 0)).all(), (m, r, c)
        limit = chunk_rows if chunk_rows else (2 << 30) // record_bytes(8192)
        for chunk, lst in by_chunk.items():
            assert len({cols[m] for m, *_ in lst}) == 1                 # one row length per chunk
            rb = record_bytes(cols[lst[0][0]])
            nrows = ngroups = 0
            for m, nr, g0, first_row, off in lst:
                assert first_row == nrows and g0 == ngroups and off == nrows * rb
                nrows += nr
                ngroups += (nr + 3) // 4
            assert nrows * rb <= region
            assert nrows <= max(4, limit // 4 * 4)
    # rows of 22016 from 60 steps on, rows of 8192 from 65, rows of 4096 from 75, rows of 2048 from 108; bf16 1.4 times as many
    def sorted_cols(**kw):
        return {cols[m] for _, m, *_ in eqg.plan_sort_segments(rows, cols, caps, eqg.Params(group_size=0, **kw))[0]}
    assert sorted_cols(iters=59) == set() and sorted_cols(iters=60) == {22016} and sorted_cols(iters=64) == {22016}
    assert sorted_cols(iters=65) == {8192, 22016} and sorted_cols(iters=74) == {8192, 22016}
    assert sorted_cols(iters=75) == {4096, 8192, 22016} and sorted_cols(iters=107) == {4096, 8192, 22016}
    assert sorted_cols(iters=108) == {2048, 4096, 8192, 22016}
    assert sorted_cols(iters=83, dtype=eqg.EQ_BF16) == set() and sorted_cols(iters=91, dtype=eqg.EQ_BF16) == {8192, 22016}
    # few steps, wide codes or short rows: no sorted evaluation
    for p in (eqg.Params(group_size=0, iters=10), eqg.Params(group_size=0, iters=100, bits=8), eqg.Params(group_size=128, iters=100)):
        assert eqg.plan_sort_segments(rows, cols, caps, p)[0] == []


def test_benchmark_refuses_more_than_one_gpu():
    # every box has one GPU; the benchmark says so instead of pretending to scale
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert res.returncode != 0
    assert "one GPU only" in (res.stderr + res.stdout)


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """The product path has no CPU route: without the built library every entry point raises."""
    import paper_2403_02775_amd as eqg
    from paper_2403_02775_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "lib_path", lambda: str(tmp_path / "libeasyquant.so"))
    with pytest.raises(ImportError, match="no CPU fallback"):
        eqg.eq_workspace_bytes([8], [128], [16], eqg.Params(group_size=128))
    with pytest.raises(ImportError):
        eqg.eq_code_words_per_row(128, 4)


def test_only_tests_smoke_and_the_cpu_baseline_touch_the_oracle():
    """The oracle is test infrastructure: the package, the C sources, the header and the input
    generator never mention it; bench.py imports it inside the functions of its cpu_baseline leg
    only, and __graft_entry__ inside smoke() only.  Nor does the oracle know the HIP path."""
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    product = [os.path.join(root, "eq_inputs.py")]
    for d in ("paper_2403_02775_amd", os.path.join("paper_2403_02775_amd", "csrc"), "include"):
        product += [os.path.join(root, d, f) for f in os.listdir(os.path.join(root, d))
                    if f.endswith((".py", ".h", ".hip"))]
    imp = re.compile(r"^\s*(from\s+oracle\b|import\s+oracle\b)", re.M)
    for path in product:
        text = open(path).read()
        assert not imp.search(text) and "easyquant_oracle" not in text, path
    for name, scope in (("bench.py", "def cpu_baseline"), ("__graft_entry__.py", "def smoke")):
        text = open(os.path.join(root, name)).read()
        hits = [m.start() for m in imp.finditer(text)]
        assert 1 <= len(hits) <= 2, name
        for h in hits:
            before = text[:h]
            last_def = before.rfind("\ndef ")
            assert before[last_def + 1:].startswith(scope), (name, before[last_def + 1:last_def + 40])
    for f in ("easyquant_oracle.py", "rowpool.py"):
        oracle = open(os.path.join(root, "oracle", f)).read()
        assert "paper_2403_02775_amd" not in oracle and "ctypes" not in oracle and "import torch" not in oracle, f
