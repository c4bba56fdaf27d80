"""Oracle: the sampling configuration in front of the target softmax (App. B "Models":
classifier-free guidance scale 3.0, temperature 1.0, top-k sampling with k = 2000).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

The paper names the configuration, not the formulas; the standard ones are taken:

  guided logit   l(x) = u(x) + s * (c(x) - u(x))      c: text-conditioned, u: null-conditioned row
  top-k          keep the tokens whose guided logit is >= the k-th largest one of the row
                 (ties with the k-th are kept), every other token gets -inf
  temperature    1: nothing to do

Which tokens survive is an integer decision taken by floating point, so it is taken here in the
precision the kernel computes in: float32, the difference, the product and the sum each rounded
once (no fused multiply-add).  A token whose conditioned logit is -inf stays -inf.  Only the image
slice [vocab_offset, vocab_offset + V) of a row takes part; everything outside is -inf.
"""
import numpy as np


def guided_logits(cond: np.ndarray, uncond: np.ndarray, scale: float) -> np.ndarray:
    c = np.asarray(cond, dtype=np.float32)
    u = np.asarray(uncond, dtype=np.float32)
    s = np.float32(scale)
    with np.errstate(invalid="ignore"):
        g = (c - u).astype(np.float32)
        l = (u + (s * g).astype(np.float32)).astype(np.float32)
    return np.where(np.isneginf(c), np.float32(-np.inf), l).astype(np.float32)


def top_k_filter(row: np.ndarray, k: int) -> np.ndarray:
    """row: 1-D float32; returns a copy with everything below the k-th largest value set to -inf."""
    row = np.asarray(row, dtype=np.float32)
    if k <= 0 or k >= row.size:
        return row.copy()
    kth = np.sort(row)[::-1][k - 1]
    return np.where(row >= kth, row, np.float32(-np.inf)).astype(np.float32)


def sampling_frontend(cond: np.ndarray, uncond: np.ndarray, scale: float, top_k: int,
                      vocab_offset: int, V: int) -> np.ndarray:
    """cond, uncond [B,M,ldv] float32 -> target logits [B,M,ldv] float32 as the verify step sees them."""
    B, M, ldv = cond.shape
    out = np.full((B, M, ldv), -np.inf, dtype=np.float32)
    sl = slice(vocab_offset, vocab_offset + V)
    g = guided_logits(cond[:, :, sl], uncond[:, :, sl], scale)
    for b in range(B):
        for m in range(M):
            out[b, m, sl] = top_k_filter(g[b, m], top_k)
    return out
