"""Oracle: committing the accepted path to the KV cache (App. A.2 "Tree drafting and decoding":
accepted tokens are kept and appended, everything after the first rejection is discarded).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

After the walk, the tree rows that stay are the root (row 0, the last committed token, whose K/V
were not in the cache yet) and the accepted path.  Their K/V rows are appended to the cache of the
item in path order; the cache length grows by 1 + accept_len.  Rows that would land at or past
the capacity S are dropped and the new length is capped at S.
"""
from typing import Tuple

import numpy as np


def commit_kv(k_cache: np.ndarray, v_cache: np.ndarray, k_tree: np.ndarray, v_tree: np.ndarray,
              path: np.ndarray, accept_len: np.ndarray, seq_len: np.ndarray
              ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """k_cache,v_cache [B,H,S,Dh]; k_tree,v_tree [B,H,M,Dh]; path [B,depth]; accept_len,seq_len [B].
    Returns copies (k_cache', v_cache', new_len)."""
    kc, vc = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    B, H, S, Dh = kc.shape
    new_len = np.zeros(B, dtype=np.int32)
    for b in range(B):
        rows = [0] + [int(path[b, i]) for i in range(int(accept_len[b]))]
        pos = int(seq_len[b])
        for r in rows:
            if pos < S:
                kc[b, :, pos] = k_tree[b, :, r]
                vc[b, :, pos] = v_tree[b, :, r]
            pos += 1
        new_len[b] = min(pos, S)
    return kc, vc, new_len
