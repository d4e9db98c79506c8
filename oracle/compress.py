"""TEST INFRASTRUCTURE: fp64 oracle of the compressed-cache construction (the step just before the
verification path).  Only tests, the smoke check and the benchmark may import it; it shares nothing with
the HIP library.

The compression branch aggregates the committed tokens into blocks of length l taken every d tokens
(Section 2.2); the aggregation used throughout this build is the plain mean of the block's K (V) rows.
Block c covers slots [c*d, c*d + l); a block exists only when all its slots hold COMMITTED tokens, so
speculative draft tokens never enter the compressed cache before they are accepted (the compressed-cache
invariant the paper's runtime keeps, Sections 3.1 and 6): N_cmp(L) = 0 for L < l, else (L - l) // d + 1.
"""
from __future__ import annotations

import numpy as np


def n_cmp_rows(L: int, l: int, d: int) -> int:
    """Number of complete compression blocks over L committed tokens."""
    return 0 if L < l else (L - l) // d + 1


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 values once to the storage type (bf16: 8 significant bits, ties to even; f32: IEEE single),
    returned as fp64."""
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    m, e = np.frexp(x)                      # x = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # np.rint rounds halves to even


def compress(rows: np.ndarray, committed_before: int, committed_after: int, l: int, d: int, dtype: str):
    """Compressed rows that become complete when the committed length grows from committed_before to
    committed_after.  rows: fp64 [S, D], the raw K (or V) rows of one (sequence, KV head), slot = row.
    Returns (first_row, values[n_new, D] rounded to the storage type, unrounded means[n_new, D])."""
    c_lo, c_hi = n_cmp_rows(committed_before, l, d), n_cmp_rows(committed_after, l, d)
    n_new = max(0, c_hi - c_lo)
    mean = np.zeros((n_new, rows.shape[1]), np.float64)
    for j in range(n_new):
        c = c_lo + j
        mean[j] = rows[c * d:c * d + l].sum(axis=0) / l
    return c_lo, round_to_storage(mean, dtype), mean
