"""Seeded synthetic weight generators shared by the tests, the benchmark and the smoke check.

This module holds NO arithmetic of the quantization method: it only draws
matrices.  Both the CPU oracle's tests and the HIP path's tests take their
inputs from here, so that the two sides are compared on identical bytes.

The matrices stand in for the LLM weights the paper quantizes (OPT / BLOOM /
LLaMA linear layers; Section 5, "Experiment Setup"), which are not available
offline.  Shapes are LLaMA-7B / LLaMA-65B linear layers laid out
``out_features x in_features`` (row = output channel).

Recipe for one matrix (all draws from one ``torch.Generator`` seeded per matrix):

* ``sigma_r ~ U[sigma_lo, sigma_hi]`` per row;
* base ``Z``: standard normal, or Student-t with 4 degrees of freedom divided
  by sqrt(2) (unit variance);
* element ``sigma_r * Z``;
* an i.i.d. Bernoulli(p_r) subset of the entries is REPLACED by
  ``+/- U[out_lo, out_hi] * sigma_r`` (sign equiprobable); ``p_r = p`` except on
  a Bernoulli(hot_row_frac) subset of rows where it is ``hot_mult * p``;
* round-to-nearest cast to fp16 / bf16.

The fraction of 3-sigma outliers this produces (0.5-0.8 %) sits in the range the
paper reports for BLOOM-7B (Tables 8 and 9: 0.29-0.86 %).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Iterator, List, Tuple

import torch

_MASK64 = (1 << 64) - 1


def mix_seed(base_seed: int, layer: int, name_id: int) -> int:
    """Fixed 64-bit mixing of (base_seed, layer, name_id) into a per-matrix seed."""
    z = (base_seed * 0x9E3779B97F4A7C15 + layer * 0xBF58476D1CE4E5B9 + name_id * 0x94D049BB133111EB + 0x2545F4914F6CDD1D) & _MASK64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & _MASK64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & _MASK64
    z ^= z >> 31
    return z & ((1 << 63) - 1)


@dataclass(frozen=True)
class Recipe:
    sigma_lo: float
    sigma_hi: float
    p: float            # outlier replacement probability
    out_lo: float       # outlier magnitude, in units of sigma_r
    out_hi: float
    base: str = "gauss"  # "gauss" | "t4"
    hot_row_frac: float = 0.0
    hot_mult: float = 3.0
    dtype: str = "f16"   # "f16" | "bf16"


# One recipe per benchmark configuration (index = position in the config list).
RECIPES = {
    "c1": Recipe(0.01, 0.05, 0.005, 8.0, 20.0),
    "c2": Recipe(0.01, 0.05, 0.005, 8.0, 20.0, hot_row_frac=0.01),
    "c3": Recipe(0.005, 0.03, 0.003, 10.0, 30.0, base="t4"),
    "c4": Recipe(0.01, 0.05, 0.005, 8.0, 20.0, hot_row_frac=0.01, dtype="bf16"),
    "c5": Recipe(0.005, 0.03, 0.005, 8.0, 20.0),
}

LAYER_NAMES = ("q", "k", "v", "o", "gate", "up", "down")


def llama_layer_shapes(hidden: int, ffn: int) -> List[Tuple[str, int, int]]:
    """(name, rows=out_features, cols=in_features) of the seven linear layers of a block."""
    return [("q", hidden, hidden), ("k", hidden, hidden), ("v", hidden, hidden), ("o", hidden, hidden),
            ("gate", ffn, hidden), ("up", ffn, hidden), ("down", hidden, ffn)]


def model_shapes(which: str) -> Tuple[int, List[Tuple[str, int, int]]]:
    """(number of layers, per-layer shapes) of the two whole-model workloads."""
    if which == "llama7b":
        return 32, llama_layer_shapes(4096, 11008)
    if which == "llama65b":
        return 80, llama_layer_shapes(8192, 22016)
    raise ValueError(which)


def torch_dtype(name: str) -> torch.dtype:
    return {"f16": torch.float16, "bf16": torch.bfloat16}[name]


def gen_matrix(rows: int, cols: int, recipe: Recipe, seed: int, device: str = "cpu",
               row_block: int = 0) -> torch.Tensor:
    """Draw one ``rows x cols`` matrix in the recipe's 16-bit dtype on ``device``.

    Rows are produced in blocks so that fp32 temporaries stay bounded; the block
    size is part of the stream definition only through the order of draws, which
    is row-block-major.  ``row_block=0`` picks a block of about 32 Mi elements.
    """
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    out = torch.empty((rows, cols), dtype=torch_dtype(recipe.dtype), device=device)
    if rows == 0 or cols == 0:
        return out
    if row_block <= 0:
        row_block = max(1, (32 << 20) // cols)
    sig = torch.empty(rows, device=device, dtype=torch.float32).uniform_(recipe.sigma_lo, recipe.sigma_hi, generator=g)
    if recipe.hot_row_frac > 0:
        hot = torch.rand(rows, device=device, generator=g) < recipe.hot_row_frac
        p_row = torch.where(hot, torch.tensor(recipe.p * recipe.hot_mult, device=device), torch.tensor(recipe.p, device=device))
    else:
        p_row = torch.full((rows,), recipe.p, device=device, dtype=torch.float32)
    for r0 in range(0, rows, row_block):
        r1 = min(rows, r0 + row_block)
        n = r1 - r0
        z = torch.randn((n, cols), device=device, generator=g)
        if recipe.base == "t4":
            chi = torch.zeros((n, cols), device=device)
            for _ in range(4):
                w = torch.randn((n, cols), device=device, generator=g)
                chi.addcmul_(w, w)
            z = z / torch.sqrt(chi / 4.0) * (0.5 ** 0.5)
            del chi, w
        elif recipe.base != "gauss":
            raise ValueError(recipe.base)
        s = sig[r0:r1, None]
        z *= s
        sel = torch.rand((n, cols), device=device, generator=g) < p_row[r0:r1, None]
        mag = torch.empty((n, cols), device=device).uniform_(recipe.out_lo, recipe.out_hi, generator=g)
        sign = (torch.rand((n, cols), device=device, generator=g) < 0.5).to(torch.float32) * 2.0 - 1.0
        z = torch.where(sel, sign * mag * s, z)
        out[r0:r1] = z.to(out.dtype)
        del z, sel, mag, sign
    return out


def gen_config_small(which: str, device: str = "cpu") -> List[Tuple[str, torch.Tensor]]:
    """The single-matrix configurations (``c1``: 256x256, ``c2``: 4096x4096)."""
    if which == "c1":
        return [("w", gen_matrix(256, 256, RECIPES["c1"], seed=0, device=device))]
    if which == "c2":
        return [("attn", gen_matrix(4096, 4096, RECIPES["c2"], seed=0, device=device))]
    raise ValueError(which)


def mlp_set_shapes() -> List[Tuple[str, int, int]]:
    """LLaMA-7B MLP set (configuration ``c3``)."""
    return [("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]


def iter_model(which: str, recipe: Recipe, device: str, base_seed: int = 0, layers: int = -1,
               scale_rows: int = 1) -> Iterator[Tuple[int, str, torch.Tensor]]:
    """Yield (layer, name, matrix) for a whole-model workload.

    ``layers`` limits the number of layers (-1 = all); ``scale_rows`` > 1 divides
    every matrix's row count (used only by small parity cases that keep the real
    row length and group structure but fewer rows).
    """
    n_layers, shapes = model_shapes(which)
    if layers >= 0:
        n_layers = min(n_layers, layers)
    for layer in range(n_layers):
        for name_id, (name, rows, cols) in enumerate(shapes):
            yield layer, name, gen_matrix(max(1, rows // scale_rows), cols, recipe,
                                          mix_seed(base_seed, layer, name_id), device=device)


def with_dtype(recipe: Recipe, dtype: str) -> Recipe:
    return replace(recipe, dtype=dtype)
