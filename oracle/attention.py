"""Oracle: tree-masked attention of the flattened draft tree (Sec. 2.1; App. A.2).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

The flattened tree (row 0 = root, rows 1..N = drafted nodes) is verified in one
pass: row i attends to the whole cached prefix and to those tree rows that are
its ancestors or itself; every other tree row is masked out.  Plain softmax
attention, float64, scale 1/sqrt(Dh) unless given.
"""
from typing import Optional

import numpy as np


def ancestor_mask(parent: np.ndarray) -> np.ndarray:
    """bool [M, M]; mask[i, t] is True iff t == i or t is an ancestor of i."""
    M = len(parent)
    mask = np.zeros((M, M), dtype=bool)
    for i in range(M):
        t = i
        while t >= 0:
            mask[i, t] = True
            t = int(parent[t])
    return mask


def tree_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                   k_tree: np.ndarray, v_tree: np.ndarray, parent: np.ndarray,
                   seq_len: Optional[np.ndarray] = None,
                   scale: Optional[float] = None) -> np.ndarray:
    """q [B,H,M,Dh]; k_tree,v_tree [B,Hkv,M,Dh]; k_cache,v_cache [B,Hkv,S,Dh] -> out [B,H,M,Dh] (float64).

    ``seq_len[b]`` (default S) = number of valid cached positions of item b.
    ``Hkv`` divides ``H``: query head h reads key/value head h // (H // Hkv) (grouped-query
    attention; Hkv == H is the plain multi-head case the paper's models use).
    """
    q = np.asarray(q, dtype=np.float64)
    B, H, M, Dh = q.shape
    S = k_cache.shape[2]
    Hkv = k_tree.shape[1]
    assert H % Hkv == 0 and k_cache.shape[1] == Hkv and v_cache.shape[1] == Hkv and v_tree.shape[1] == Hkv
    group = H // Hkv
    scale = 1.0 / np.sqrt(Dh) if not scale else float(scale)
    vis = ancestor_mask(parent)
    out = np.zeros((B, H, M, Dh), dtype=np.float64)
    for b in range(B):
        Sb = S if seq_len is None else int(seq_len[b])
        for h in range(H):
            g = h // group
            K = np.concatenate([np.asarray(k_cache[b, g, :Sb], dtype=np.float64),
                                np.asarray(k_tree[b, g], dtype=np.float64)], axis=0)
            Vv = np.concatenate([np.asarray(v_cache[b, g, :Sb], dtype=np.float64),
                                 np.asarray(v_tree[b, g], dtype=np.float64)], axis=0)
            s = (q[b, h] @ K.T) * scale                      # [M, Sb+M]
            s[:, Sb:][~vis] = -np.inf
            s = s - s.max(axis=1, keepdims=True)
            w = np.exp(s)
            w = w / w.sum(axis=1, keepdims=True)
            out[b, h] = w @ Vv
    return out
