"""Pins of oracle.float32_error_bound (the allowance the GPU parity tests add, capped, to the
1e-4 relative rule where Eq. 2's subtraction cancels; Sec. 4, App. A.2 Eq. 2).

The bound is compared with what a float32 evaluation really loses: the same rows are replayed
below in numpy float32, every operation rounded once (exponentials, sums, products, the
difference of Eq. 2, the reciprocal of the normaliser), which is how a float32 implementation
works.  The replay is written here, from the formulas, and shares nothing with the oracle but
the inputs.  Two things are asserted: the replay never leaves ``1e-4 relative + bound`` (the
rule of the GPU tests), and wherever the bound is actually needed it is within a stated
factor of the observed error, so that it cannot be a blanket excuse.
"""
import numpy as np
import pytest

from oracle import float32_error_bound, relaxed_verify
from workloads import CONFIGS, children_lists, make_codebook, make_verify_inputs, static_tree
from oracle import build_neighbours

F = np.float32


def replay_float32(parent, target, drafter, off, V, tokens, neigh, k, lam):
    """mass, q_tok, p_tok, n_agg per node from float32 arithmetic (prefix rule, multiplicative bound,
    i.i.d. siblings).  r is kept unnormalised with a running scale rs, as a float32 kernel would."""
    kids = children_lists(parent)
    B, M = tokens.shape
    mass = np.zeros((B, M), F); q_tok = np.zeros((B, M), F); p_tok = np.zeros((B, M), F)
    n_agg = np.zeros((B, M), np.int32)
    for b in range(B):
        for P in range(M):
            if not kids[P]:
                continue
            x = target[b, P, off:off + V].astype(F)
            y = drafter[b, P, off:off + V].astype(F)
            r = np.exp(x - x.max(), dtype=F)
            rs = F(1) / r.sum(dtype=F)
            e = np.exp(y - y.max(), dtype=F)
            p = e * (F(1) / e.sum(dtype=F))
            for c in kids[P]:
                t = int(tokens[b, c])
                cap = F(lam) * r[t]
                cum, j = r[t], 1
                for i in range(1, k):
                    nxt = F(cum + r[neigh[t, i]])
                    if not nxt < cap:
                        break
                    cum, j = nxt, j + 1
                mass[b, c] = F(cum * rs); q_tok[b, c] = F(r[t] * rs); p_tok[b, c] = p[t]; n_agg[b, c] = j
                r2 = r.copy(); r2[neigh[t, 1:j]] = 0; r2[t] = cum
                res = np.maximum(F(1) * (r2 * rs) - p, F(0)).astype(F)     # product and difference rounded separately
                z = res.sum(dtype=F)
                if z > 0:
                    r, rs = res, F(1) / z
    return {"mass": mass, "q_tok": q_tok, "p_tok": p_tok, "n_agg": n_agg}


def _check(parent, x, neigh, V, off, k, lam, rel=1e-4, factor=50.0):
    want = relaxed_verify(parent, x["target_logits"], x["drafter_logits"], off, V, x["tokens"], neigh, k, lam,
                          x["u_accept"], x["u_final"])
    bnd = float32_error_bound(parent, x["target_logits"], x["drafter_logits"], off, V, x["tokens"], neigh, k, lam)
    got = replay_float32(parent, x["target_logits"], x["drafter_logits"], off, V, x["tokens"], neigh, k, lam)
    kids = children_lists(parent)
    stats = dict(nodes=0, needed=0, tightest=np.inf, max_rel=0.0)
    B, M = x["tokens"].shape
    for b in range(B):
        for P in range(M):
            for c in kids[P]:
                if got["n_agg"][b, c] != want["n_agg"][b, c]:
                    assert want["bound_margin"][b, c] < 1e-4       # a float32-level tie at the stopping sum
                    break                                            # later siblings are not comparable
                stats["nodes"] += 1
                for name in ("mass", "q_tok", "p_tok"):
                    g, w, e = float(got[name][b, c]), float(want[name][b, c]), float(bnd[name + "_err"][b, c])
                    d = abs(g - w)
                    assert d <= rel * abs(w) + e, f"{name} b={b} c={c}: float32 off by {d}, bound {e}, value {w}"
                    stats["max_rel"] = max(stats["max_rel"], d / max(abs(w), 1e-300))
                    if d > rel * abs(w):                              # the bound was needed here
                        stats["needed"] += 1
                        stats["tightest"] = min(stats["tightest"], e / d)
                        assert e <= factor * d, f"{name} b={b} c={c}: bound {e} is {e / d:.0f}x the error {d}"
    return stats


def test_bound_on_the_repeated_token_case():
    # tiny vocabulary, drafter close to the target, two children per row: siblings often repeat a
    # token, and after the first rejection the adjusted target at that token is close to p
    cfg = CONFIGS[1].scaled(V=64, ldv=64, k=4, N=3, branching=(2, 1), B=1500)
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=0.9)
    neigh = build_neighbours(make_codebook(cfg), cfg.k)
    st = _check(parent, x, neigh, cfg.V, 0, cfg.k, cfg.lam)
    print(st)
    assert st["nodes"] > 4000
    assert st["needed"] >= 1, "no node of this input needs the allowance: the case no longer exercises it"
    assert st["tightest"] <= 50.0


@pytest.mark.parametrize("idx,rho", [(1, 0.0), (1, 0.8), (2, 0.8)])
def test_bound_on_workload_rows(idx, rho):
    cfg = CONFIGS[idx]
    cfg = cfg.scaled(B=4) if idx == 1 else cfg.scaled(V=2048, ldv=2048, k=64)
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=rho)
    neigh = build_neighbours(make_codebook(cfg), cfg.k)
    st = _check(parent, x, neigh, cfg.V, cfg.vocab_offset, cfg.k, cfg.lam)
    print(st)
    assert st["nodes"] >= 20
    # ordinary nodes: float32 is far inside the relative rule and the bound is a few roundings
    bnd = float32_error_bound(parent, x["target_logits"], x["drafter_logits"], cfg.vocab_offset, cfg.V, x["tokens"],
                              neigh, cfg.k, cfg.lam)
    want = relaxed_verify(parent, x["target_logits"], x["drafter_logits"], cfg.vocab_offset, cfg.V, x["tokens"], neigh,
                          cfg.k, cfg.lam, x["u_accept"], x["u_final"])
    first = [c[0] for c in children_lists(parent) if c]              # first children: nothing has been subtracted yet
    assert np.all(bnd["mass_err"][:, first] <= 2.0 ** -21 * want["mass"][:, first])
    assert np.all(bnd["q_tok_err"][:, first] == 2.0 ** -22 * want["q_tok"][:, first])


def test_bound_grows_where_the_subtraction_cancels():
    # One row, two children with the same token x^ = 0 and no neighbours (k = 1).  After the first
    # rejection r(0) = gap / Z with gap = q(0) - p(0) and Z = gap + 0.3 (token 2 holds the rest of the
    # residual).  The numerator keeps the rounding of q(0) and p(0) and of their difference,
    # 2 eps (q(0) + p(0)), so the relative bound on the second child's q_tok must be that over the gap,
    # plus a few eps from the normaliser: it grows as the gap closes.
    V, eps = 8, 2.0 ** -22
    parent = np.array([-1, 0, 0], dtype=np.int32)
    neigh = np.arange(V, dtype=np.int32)[:, None].copy()
    rels = []
    for gap in (1e-6, 1e-4, 1e-2):
        q = np.array([0.3, 0.1, 0.5, 0.02, 0.02, 0.02, 0.02, 0.02])
        p = q.copy()
        p[0] -= gap; p[2] -= 0.3; p[1] += gap + 0.3
        tl = np.log(q)[None, None, :].repeat(3, axis=1)
        dl = np.log(p)[None, None, :].repeat(3, axis=1)
        tok = np.zeros((1, 3), dtype=np.int32)
        bnd = float32_error_bound(parent, tl, dl, 0, V, tok, neigh, 1, 2.0)
        want = relaxed_verify(parent, tl, dl, 0, V, tok, neigh, 1, 2.0, np.zeros((1, 3)), np.zeros((1, 3)))
        assert want["q_tok"][0, 1] == pytest.approx(0.3, rel=1e-12)
        assert want["q_tok"][0, 2] == pytest.approx(gap / (gap + 0.3), rel=1e-6)
        assert bnd["q_tok_err"][0, 1] == pytest.approx(eps * 0.3, rel=1e-12)            # first child: one unit
        rels.append(bnd["q_tok_err"][0, 2] / want["q_tok"][0, 2])
        lead = 2.0 * eps * (q[0] + p[0]) / gap
        assert lead <= rels[-1] <= lead + 15.0 * eps
    assert rels[0] > 90 * rels[1] > 90 * 90 * rels[2] * 0.9
