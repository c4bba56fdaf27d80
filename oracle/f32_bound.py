"""Oracle side-car: how far a float32 evaluation of the relaxed acceptance may sit from the
float64 values of ``relaxed_verify`` (Sec. 4; Sec. 2.2; App. A.2 Eq. 2).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

This is not part of the method; it is a first-order rounding analysis that the GPU parity
tests add to their relative tolerance, kept apart from ``relaxed_verify`` so that the
definition there stays plain.  Why it is needed: Eq. 2 subtracts p from the adjusted target.
Where the two nearly cancel (a sibling that repeats a token whose adjusted target mass is
close to p) the difference keeps the absolute rounding of both operands, and the division by
the normaliser Z blows that up relative to what is left.  Away from such cancellations the
bound is a few float32 roundings (about 2e-7 relative).

Model, with eps = 2^-22 (a few float32 roundings per stored value) as the unit:
  start      err r(x) = eps r(x),  err p(x) = eps p(x)
  child      err mass = err r(x^) + sum_{A} err r;  err q_tok = err r(x^);  err p_tok = err p(x^)
  residual   d(x) = r'(x) - p(x):  err d = err r' + err p + eps (r' + p)
             an entry counts if it is positive or could be (|d| <= err d)
             err Z = sum of err d over the entries that count
             r <- [d]_+ / Z:  err r = err d / Z + r err Z / Z + eps r
  distinct siblings   p <- p / (1 - p(x^)) with p(x^) <- 0: quotient rule plus eps p
The bound is pinned by tests/test_oracle_f32_bound.py against a float32 replay.
"""
from typing import Dict

import numpy as np

from .verify import _children, aggregate_set, softmax64

EPS = 2.0 ** -22


def float32_error_bound(parent: np.ndarray, target_logits: np.ndarray, drafter_logits: np.ndarray,
                        vocab_offset: int, V: int, tokens: np.ndarray, neigh: np.ndarray, k: int, lam: float,
                        bound: str = "multiplicative", rule: str = "prefix",
                        siblings: str = "with_replacement") -> Dict[str, np.ndarray]:
    """Per node [B,M]: mass_err, q_tok_err, p_tok_err (absolute).  Same arguments as
    ``relaxed_verify`` (the uniforms play no part)."""
    parent = np.asarray(parent)
    B, M = tokens.shape
    kids = _children(parent)
    off = int(vocab_offset)
    lam = float(lam)
    mass_err = np.zeros((B, M)); q_tok_err = np.zeros((B, M)); p_tok_err = np.zeros((B, M))
    for b in range(B):
        for P in range(M):
            if not kids[P]:
                continue
            r = softmax64(target_logits[b, P])[off:off + V]
            p = softmax64(drafter_logits[b, P])[off:off + V]
            r_err = EPS * r
            p_err = EPS * p
            for c in kids[P]:
                t = int(tokens[b, c])
                cap = lam * r[t] if bound == "multiplicative" else lam
                _, cum, members, _ = aggregate_set(r, neigh[t], t, k, cap, rule)
                mass_err[b, c] = r_err[t] + r_err[members].sum()
                q_tok_err[b, c] = r_err[t]
                p_tok_err[b, c] = p_err[t]
                r2 = r.copy(); r2[members] = 0.0; r2[t] = cum
                e2 = r_err.copy(); e2[members] = 0.0; e2[t] = mass_err[b, c]
                d = r2 - p
                d_err = e2 + p_err + EPS * (r2 + p)
                live = (d > 0) | (np.abs(d) <= d_err)
                res = np.maximum(d, 0.0)
                Z = res.sum()
                if Z > 0:
                    z_err = d_err[live].sum()
                    r = res / Z
                    r_err = np.where(live, d_err, 0.0) / Z + r * (z_err / Z) + EPS * r
                if siblings == "without_replacement":
                    left = 1.0 - p[t]
                    left_err = p_err[t] + EPS
                    p = p.copy(); p[t] = 0.0
                    if left > 0:
                        p = p / left
                        p_err = p_err / left + p * (left_err / left) + EPS * p
                        p_err[t] = 0.0
                    else:
                        p = np.zeros_like(p); p_err = np.zeros_like(p)
    return {"mass_err": mass_err, "q_tok_err": q_tok_err, "p_tok_err": p_tok_err}
