"""Oracle: latent-space neighbourhoods B_k(x) (Sec. 2.2; reused in Sec. 4).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

For every code x the k most similar codes, nearest first, x itself in slot 0.
Similarity is the inner product of the (caller-normalised) codebook rows, i.e.
cosine similarity.  The similarity of a pair is evaluated in float64 from the
float32 inputs, adding the D products one after the other in index order; ties
go to the lower index.
"""
from typing import Optional, Sequence

import numpy as np


def similarity_keys(E: np.ndarray, rows: Sequence[int]) -> np.ndarray:
    """key[r, j] = sum_t E[rows[r], t] * E[j, t], float64, t ascending."""
    E64 = np.asarray(E, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    key = np.zeros((len(rows), E64.shape[0]), dtype=np.float64)
    for t in range(E64.shape[1]):
        key = key + np.outer(E64[rows, t], E64[:, t])
    return key


def build_neighbours(E: np.ndarray, k: int, rows: Optional[Sequence[int]] = None,
                     block: int = 512) -> np.ndarray:
    """int32 [len(rows), k]; row r lists B_k(rows[r]), nearest first, self first."""
    V = E.shape[0]
    if not (1 <= k <= V):
        raise ValueError("k must be in [1, V]")
    rows = np.arange(V) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), k), dtype=np.int32)
    for s in range(0, len(rows), block):
        blk = rows[s:s + block]
        key = similarity_keys(E, blk)
        for n, i in enumerate(blk):
            order = np.argsort(-key[n], kind="stable")     # descending, ties -> lower index
            order = order[order != i]
            out[s + n, 0] = i
            out[s + n, 1:] = order[:k - 1]
    return out
