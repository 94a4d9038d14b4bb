"""Evaluation arithmetic shared by the benchmark and the tests (no GPU, no oracle).

``recovery`` is the paper's "fraction of the FP4-FP16 gap closed" (Table 1 caption):
(score - score_fp4) / (score_fp16 - score_fp4).  On synthetic inputs the score is an output
error against exact attention (lower is better), which the same ratio handles.
"""
from __future__ import annotations

import math


def recovery(value_fp16: float, value_fp4: float, value_method: float) -> float:
    gap = value_fp16 - value_fp4
    if gap == 0:
        return float("nan")
    return (value_method - value_fp4) / gap


def causal_tiles(N: int, Bq: int, Bk: int) -> int:
    """Number of (query block, key block) tiles with at least one unmasked pair."""
    return sum(min(N // Bk, ((i + 1) * Bq - 1) // Bk + 1) for i in range(N // Bq))


def attention_flops(N: int, D: int, heads: int, causal: bool) -> float:
    """4*D flops per unmasked (query, key) pair: Q.K^T plus P.V; masked pairs are not counted."""
    pairs = N * (N + 1) / 2 if causal else float(N) * N
    return 4.0 * D * pairs * heads


def blended_peak(frac16: float, peak16: float, peak4: float) -> float:
    """Peak of a tile mix: a fraction frac16 of the tiles at the 16-bit rate, the rest at the
    4-bit rate (the cost model of Sec. 4.4: an FP4 tile costs a quarter of an FP16 tile)."""
    return 1.0 / (frac16 / peak16 + (1.0 - frac16) / peak4)


def rel_fro(x, ref) -> float:
    import numpy as np

    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(math.sqrt(((x - ref) ** 2).sum()) / math.sqrt((ref ** 2).sum()))
