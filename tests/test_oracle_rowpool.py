"""The row pool (oracle/rowpool.py) only dispatches whole rows to worker processes: its result
must be the oracle's own, bit for bit, for every field, whatever the block size."""
import numpy as np
import pytest

import eq_inputs
from oracle import easyquant_oracle as eqo
from oracle import rowpool

pytestmark = pytest.mark.oracle_pool


@pytest.mark.parametrize("p", [eqo.Params(bits=4, group_size=128, iters=7),
                               eqo.Params(bits=3, group_size=0, iters=5, mode=eqo.ASYMMETRIC),
                               eqo.Params(dtype=eqo.BF16, bits=4, group_size=64, iters=0, stat_scope=eqo.STAT_GROUP)])
def test_row_blocks_stitch_to_the_whole_matrix(oracle_pool, p):
    rec = eq_inputs.with_dtype(eq_inputs.RECIPES["c2"], "bf16" if p.dtype == eqo.BF16 else "f16")
    W = eq_inputs.gen_matrix(45, 512, rec, seed=11, device="cpu")
    raw = W.view(__import__("torch").int16).numpy().view(np.uint16)
    want = eqo.quantize_matrix(raw, p)
    for rows_per_block in (1, 7, 16, 100):
        got = oracle_pool.quantize_matrix(raw, p, rows_per_block)
        for k in ("codes", "scales", "zero_points", "out_row_ptr", "out_col", "out_val", "mask", "u"):
            assert got[k].dtype == want[k].dtype and np.array_equal(got[k], want[k]), (k, rows_per_block)
    assert int(want["out_row_ptr"][-1]) > 0


def test_row_pool_refuses_whole_matrix_statistics(oracle_pool):
    raw = np.zeros((4, 64), np.uint16)
    with pytest.raises(ValueError):
        oracle_pool.quantize_matrix(raw, eqo.Params(stat_scope=eqo.STAT_MATRIX))
    assert rowpool.stitch([eqo.quantize_matrix(raw, eqo.Params(iters=0))])["out_row_ptr"].tolist() == [0] * 5
