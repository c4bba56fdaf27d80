"""Oracle: relaxed acceptance over a static draft tree (Sec. 2.2, Sec. 4, App. A.2).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

Per tree row P (root or drafted node) with children c_1, c_2, ... in index order:

  q = softmax(target logits of P), p = softmax(drafter logits of P)   (Sec. 2, T = 1)
  r <- q
  for each child c with drafted token x^:
      A   = longest nearest-first prefix of B_k(x^) with  sum_{x in A} r(x) < lambda * r(x^),
            x^ always a member                                         (Sec. 4, the bound)
      m   = sum_{x in A} r(x);  accept iff u < min(1, m / p(x^))       (Sec. 4, accept prob.)
      on rejection: r' = r with A's mass moved onto x^;
                    r  <- normalise([r' - p]_+)                        (Sec. 2.2 "adjusted", Eq. 2)
  if every child is rejected a replacement is drawn from r; at a leaf a bonus
  token is drawn from q.

Every row is evaluated for the outcome "all earlier siblings were rejected",
which depends on no uniform; the walk from the root then only follows the
recorded decisions (App. A.2: accepted tokens are kept, the rest is discarded).
All arithmetic in float64.
"""
from typing import Dict, List

import numpy as np


def softmax64(logits: np.ndarray) -> np.ndarray:
    x = np.asarray(logits, dtype=np.float64)
    w = np.exp(x - x.max())
    return w / w.sum()


def inverse_cdf(d: np.ndarray, u: float) -> int:
    """Smallest x with cumsum(d)[x] > u * sum(d) (token order ascending)."""
    C = np.cumsum(d)
    x = int(np.searchsorted(C, float(u) * C[-1], side="right"))
    if x >= len(d):                      # only if u*sum rounds up to the total
        x = int(np.flatnonzero(d > 0)[-1])
    return x


def _children(parent: np.ndarray) -> List[List[int]]:
    kids: List[List[int]] = [[] for _ in range(len(parent))]
    for i in range(1, len(parent)):
        kids[int(parent[i])].append(i)
    return kids


def aggregate_set(r: np.ndarray, nb: np.ndarray, t: int, k: int, cap: float, rule: str):
    """The set A inside B_k(x^) (Sec. 4) for the current r.  ``nb`` = B_k(x^) nearest first with
    x^ itself in slot 0.  Returns (|A|, sum_A r, members of A other than x^, the sums that were
    compared with the cap)."""
    vals = r[np.asarray(nb[:k], dtype=np.int64)]
    vals[0] = r[t]                           # x^ itself is always a member
    if rule == "prefix":
        C = np.cumsum(vals)                  # nearest-first prefix sums
        bad = np.flatnonzero(~(C[1:] < cap)) # strict '<' of the bound
        j = 1 + (int(bad[0]) if bad.size else k - 1)
        return j, C[j - 1], np.asarray(nb[1:j], dtype=np.int64), C[1:min(j + 1, k)]
    cum = vals[0]
    taken, tried = [], []
    for i in range(1, k):                    # nearest first; a violator is passed over
        tried.append(cum + vals[i])
        if cum + vals[i] < cap:
            cum = cum + vals[i]
            taken.append(int(nb[i]))
    return 1 + len(taken), cum, np.asarray(taken, dtype=np.int64), np.asarray(tried)


def relaxed_verify(parent: np.ndarray, target_logits: np.ndarray, drafter_logits: np.ndarray,
                   vocab_offset: int, V: int, tokens: np.ndarray, neigh: np.ndarray,
                   k: int, lam: float, u_accept: np.ndarray, u_final: np.ndarray,
                   keep_final_cdf: bool = False, bound: str = "multiplicative",
                   rule: str = "prefix", siblings: str = "with_replacement") -> Dict[str, np.ndarray]:
    """target/drafter logits [B,M,ldv]; tokens,u_* [B,M]; neigh [V,>=k] -> dict of outputs.

    Outputs (all [B,M] unless noted): decision (uint8), ratio, mass, n_agg,
    q_tok, p_tok, final_tok_all; accept_len [B], path [B,depth] (-1 padded),
    final_token [B].  Diagnostics: bound_margin = min_j |cum_j - lam*r(x^)| /
    (lam*r(x^)) over the prefix sums that were compared (inf if none);
    final_cdf [B,M,V] (cumulative, unnormalised) if requested.

    ``bound``: "multiplicative" (Sec. 4, LANTERN++: sum_A r < lam * r(x^)) or "additive" (the
    earlier LANTERN bound as Sec. 4 prints it: sum_A r < delta, with ``lam`` holding delta).  In
    both the sum runs over A including x^, and x^ is a member whatever the bound says.

    ``rule``: how A is picked inside B_k(x^), which Sec. 4 leaves to its constraint.  "prefix":
    the longest nearest-first prefix that keeps the sum below the cap.  "skip": neighbours are
    visited nearest first, one that would lift the sum to the cap or above is left out and the
    visit goes on (a maximal set for that order; a superset of the prefix).

    ``siblings``: how the children of one row were drafted (Sec. 2.1 says only that several
    tokens are sampled from p).  "with_replacement": i.i.d. draws, p is the same for every
    child.  "without_replacement": the children are distinct tokens drawn one after the other
    from p with the earlier ones removed; a rejected child's token is therefore taken out of p
    (p(x^) <- 0, the rest divided by 1 - p(x^)) before the next child is tried.  Both keep the
    output law equal to the target when A = {x^}.
    """
    if bound not in ("multiplicative", "additive"):
        raise ValueError("bound must be 'multiplicative' or 'additive'")
    if rule not in ("prefix", "skip"):
        raise ValueError("rule must be 'prefix' or 'skip'")
    if siblings not in ("with_replacement", "without_replacement"):
        raise ValueError("siblings must be 'with_replacement' or 'without_replacement'")
    parent = np.asarray(parent)
    B, M = tokens.shape
    kids = _children(parent)
    depth = np.zeros(M, dtype=np.int64)
    for i in range(1, M):
        depth[i] = depth[parent[i]] + 1
    max_depth = int(depth.max()) if M > 1 else 0
    off = int(vocab_offset)
    lam = float(lam)

    decision = np.zeros((B, M), dtype=np.uint8)
    ratio = np.zeros((B, M)); mass = np.zeros((B, M))
    q_tok = np.zeros((B, M)); p_tok = np.zeros((B, M))
    n_agg = np.zeros((B, M), dtype=np.int32)
    margin = np.full((B, M), np.inf)
    final_all = np.zeros((B, M), dtype=np.int32)
    accept_len = np.zeros(B, dtype=np.int32)
    path = np.full((B, max(max_depth, 1)), -1, dtype=np.int32)
    final_token = np.zeros(B, dtype=np.int32)
    final_cdf = np.zeros((B, M, V)) if keep_final_cdf else None

    for b in range(B):
        for P in range(M):
            full = softmax64(target_logits[b, P])
            q = full[off:off + V]
            assert full[:off].sum() == 0.0 and full[off + V:].sum() == 0.0, "mass outside the image slice"
            r = q.copy()
            if kids[P]:
                p = softmax64(drafter_logits[b, P])[off:off + V]
                for c in kids[P]:
                    t = int(tokens[b, c])
                    nb = neigh[t]
                    cap = lam * r[t] if bound == "multiplicative" else lam
                    j, cum, members, seen = aggregate_set(r, nb, t, k, cap, rule)
                    if cap > 0 and seen.size:
                        margin[b, c] = np.min(np.abs(seen - cap)) / cap
                    mass[b, c] = cum
                    n_agg[b, c] = j
                    q_tok[b, c] = r[t]
                    p_tok[b, c] = p[t]
                    with np.errstate(divide="ignore", invalid="ignore"):
                        ratio[b, c] = np.float64(cum) / np.float64(p[t])
                    decision[b, c] = 1 if float(u_accept[b, c]) * p[t] < cum else 0
                    # outcome "c rejected": move A's mass onto x^, take the positive residual
                    r2 = r.copy()
                    r2[members] = 0.0
                    r2[t] = cum
                    res = np.maximum(r2 - p, 0.0)
                    Z = res.sum()
                    if Z > 0:
                        r = res / Z                      # else r stays (r' == p: c is accepted with probability 1)
                    if siblings == "without_replacement":
                        left = 1.0 - p[t]                # what the other tokens hold of p
                        p = p.copy()
                        p[t] = 0.0
                        p = p / left if left > 0 else np.zeros_like(p)
            final_all[b, P] = inverse_cdf(r, float(u_final[b, P]))
            if keep_final_cdf:
                final_cdf[b, P] = np.cumsum(r)
        cur, n = 0, 0
        while True:
            nxt = next((c for c in kids[cur] if decision[b, c]), None)
            if nxt is None:
                break
            path[b, n] = nxt
            n += 1
            cur = nxt
        accept_len[b] = n
        final_token[b] = final_all[b, cur]

    out = {"decision": decision, "ratio": ratio, "mass": mass, "n_agg": n_agg,
           "q_tok": q_tok, "p_tok": p_tok, "final_tok_all": final_all,
           "accept_len": accept_len, "path": path, "final_token": final_token,
           "bound_margin": margin}
    if keep_final_cdf:
        out["final_cdf"] = final_cdf
    return out
