"""Pins for oracle.relaxed_verify (no GPU).

The oracle is checked against things other than itself: a hand-derived example
(Sec. 4 / Eq. 2), an independently written plain speculative sampler (Eq. 1-2),
exact enumeration and Monte Carlo of the output distribution (faithfulness
statement after Eq. 2), the bound invariants of Sec. 4, and brute force over
all prefixes on tiny vocabularies.
"""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import relaxed_verify, build_neighbours, inverse_cdf
from workloads import CONFIGS, static_tree, make_codebook, make_verify_inputs, children_lists

GOLD = os.path.join(os.path.dirname(__file__), "golden", "relaxed_accept_hand_example.json")


def _logits(prob):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(prob, dtype=np.float64))


def _call(parent, q_rows, p_rows, tokens, neigh, k, lam, ua, uf, **kw):
    """q_rows/p_rows: [M,V] probabilities -> one batch item."""
    M, V = np.shape(q_rows)
    return relaxed_verify(np.asarray(parent), _logits(q_rows)[None], _logits(p_rows)[None], 0, V,
                          np.asarray(tokens, dtype=np.int32)[None], np.asarray(neigh), k, lam,
                          np.asarray(ua, dtype=np.float64)[None], np.asarray(uf, dtype=np.float64)[None], **kw)


# ---------------------------------------------------------------- hand example
def test_hand_example():
    g = json.load(open(GOLD))
    q, p = np.array(g["q"]), np.array(g["p"])
    neigh = np.array([g["neigh_row_of_token0"], [1, 0, 2, 3], [2, 1, 3, 0], [3, 2, 1, 0]])
    parent = [-1, 0]
    Q, Pm = np.stack([q, q]), np.stack([p, p])
    for case in g["cases"]:
        for u, want in case["accept_for_u"].items():
            o = _call(parent, Q, Pm, [0, 0], neigh, 4, case["lambda"], [0, float(u)], [0.5, 0.5],
                      keep_final_cdf=True)
            assert o["decision"][0, 1] == want
            assert o["mass"][0, 1] == pytest.approx(case["mass"], rel=1e-12)
            assert o["n_agg"][0, 1] == case["n_agg"]
            assert o["ratio"][0, 1] == pytest.approx(case["ratio"], rel=1e-12)
            cdf = o["final_cdf"][0, 0]
            res = np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
            assert np.allclose(res, case["residual"], atol=1e-12)
            assert o["accept_len"][0] == want
        for u, tok in case["final_for_u"].items():
            # child rejected (u_accept = 0.999) -> final token is the residual draw at the root
            o = _call(parent, Q, Pm, [0, 0], neigh, 4, case["lambda"], [0, 0.999], [float(u), 0.5])
            assert o["decision"][0, 1] == 0 and o["accept_len"][0] == 0
            assert o["final_token"][0] == tok and o["final_tok_all"][0, 0] == tok


# ------------------------------------------- independent plain speculative sampler
def _plain_sps_row(q, p, toks, us):
    """Eq. 1 + Eq. 2 applied sibling after sibling; written without the oracle."""
    r = q.copy()
    rows = []
    for t, u in zip(toks, us):
        a = min(1.0, r[t] / p[t]) if p[t] > 0 else 1.0
        rows.append((r[t], p[t], r[t] / p[t], 1 if u < a else 0))
        d = np.where(r > p, r - p, 0.0)
        if d.sum() > 0:
            r = d / d.sum()
    return rows, r


@pytest.mark.parametrize("mode", ["k1", "lam1", "lam_half"])
def test_reduces_to_plain_speculative_sampling(mode):
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    kids = children_lists(parent)
    E = make_codebook(cfg)
    neigh = build_neighbours(E, 16)
    x = make_verify_inputs(cfg, parent, rho=0.8)
    k, lam = {"k1": (1, 2.0), "lam1": (16, 1.0), "lam_half": (16, 0.5)}[mode]
    o = relaxed_verify(parent, x["target_logits"], x["drafter_logits"], 0, cfg.V, x["tokens"],
                       neigh, k, lam, x["u_accept"], x["u_final"], keep_final_cdf=True)
    sm = lambda l: (lambda w: w / w.sum())(np.exp(l.astype(np.float64) - l.astype(np.float64).max()))
    n_acc = 0
    for P in range(cfg.M):
        q = sm(x["target_logits"][0, P]); p = sm(x["drafter_logits"][0, P])
        if not kids[P]:
            assert o["final_tok_all"][0, P] == inverse_cdf(q, x["u_final"][0, P])
            continue
        rows, r = _plain_sps_row(q, p, x["tokens"][0, kids[P]], x["u_accept"][0, kids[P]])
        for c, (qt, pt, ratio, dec) in zip(kids[P], rows):
            assert o["n_agg"][0, c] == 1
            assert o["q_tok"][0, c] == pytest.approx(qt, rel=1e-12)
            assert o["mass"][0, c] == pytest.approx(qt, rel=1e-12)
            assert o["p_tok"][0, c] == pytest.approx(pt, rel=1e-12)
            assert o["ratio"][0, c] == pytest.approx(ratio, rel=1e-12)
            assert o["decision"][0, c] == dec
            n_acc += dec
        cdf = o["final_cdf"][0, P]
        assert np.allclose(np.diff(np.concatenate([[0.0], cdf])) / cdf[-1], r, rtol=1e-10, atol=1e-15)
    assert n_acc > 0


# ----------------------------------------------------------- exact enumeration
def _first_token_distribution(q, p, n_sib, neigh, k, lam):
    """Exact law of the first emitted token at a root with n_sib i.i.d. drafts."""
    V = len(q)
    parent = [-1] + [0] * n_sib
    out = np.zeros(V)
    Q = np.stack([q] * (n_sib + 1)); Pm = np.stack([p] * (n_sib + 1))
    for toks in itertools.product(range(V), repeat=n_sib):
        w = np.prod([p[t] for t in toks])
        if w == 0:
            continue
        o = _call(parent, Q, Pm, [0] + list(toks), neigh, k, lam, [0.5] * (n_sib + 1),
                  [0.5] * (n_sib + 1), keep_final_cdf=True)
        stay = 1.0
        for i, t in enumerate(toks):
            a = min(1.0, o["ratio"][0, i + 1])
            out[t] += w * stay * a
            stay *= 1.0 - a
        cdf = o["final_cdf"][0, 0]
        out += w * stay * np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
    return out


@pytest.mark.parametrize("n_sib", [1, 2, 3])
def test_unrelaxed_output_distribution_is_target(n_sib):
    g = np.random.default_rng(7 + n_sib)
    V = 5
    q = g.dirichlet(np.ones(V)); p = g.dirichlet(np.ones(V))
    neigh = np.array([np.roll(np.arange(V), -i) for i in range(V)])
    d = _first_token_distribution(q, p, n_sib, neigh, 1, 3.0)
    assert np.max(np.abs(d - q)) < 1e-12
    d = _first_token_distribution(q, p, n_sib, neigh, V, 1.0)     # bound admits no neighbour
    assert np.max(np.abs(d - q)) < 1e-12


def test_relaxed_output_distribution_closed_form():
    """One draft: law = sum_x p(x) [a_x delta_x + (1-a_x) norm([q'_x - p]_+)], q'_x = q with A(x) merged."""
    g = np.random.default_rng(11)
    V, k, lam = 6, 4, 2.5
    q = g.dirichlet(np.ones(V) * 20); p = g.dirichlet(np.ones(V) * 5)   # flat: neighbours are admitted
    neigh = np.array([[i] + [j for j in g.permutation(V) if j != i] for i in range(V)])
    want = np.zeros(V)
    for x in range(V):
        members = [x]
        tot = q[x]
        for j in neigh[x][1:k]:                      # brute force: longest admissible prefix
            if tot + q[j] < lam * q[x]:
                tot += q[j]; members.append(j)
            else:
                break
        a = min(1.0, tot / p[x])
        qp = q.copy(); qp[members] = 0; qp[x] = tot
        res = np.clip(qp - p, 0, None)
        want[x] += p[x] * a
        if res.sum() > 0:
            want += p[x] * (1 - a) * res / res.sum()
    got = _first_token_distribution(q, p, 1, neigh, k, lam)
    assert np.max(np.abs(got - want)) < 1e-12
    assert abs(got.sum() - 1) < 1e-12
    assert np.max(np.abs(got - q)) > 1e-3            # relaxation does move the law


def test_depth2_walk_and_bonus_enumeration():
    """Root -> 2 siblings -> 1 child each: first token ~ q0; given acceptance, second ~ q1(.|first)."""
    g = np.random.default_rng(3)
    V = 3
    q0 = g.dirichlet(np.ones(V)); p0 = g.dirichlet(np.ones(V))
    q1 = g.dirichlet(np.ones(V), size=V); p1 = g.dirichlet(np.ones(V), size=V)   # rows indexed by token
    q2 = g.dirichlet(np.ones(V), size=V)
    parent = [-1, 0, 0, 1, 2]
    neigh = np.arange(V)[:, None]
    first = np.zeros(V); pair = np.zeros((V, V)); triple_bonus = np.zeros(V)
    for t1, t2, t3, t4 in itertools.product(range(V), repeat=4):
        w = p0[t1] * p0[t2] * p1[t1][t3] * p1[t2][t4]
        Q = np.stack([q0, q1[t1], q1[t2], q2[t3], q2[t4]])
        Pm = np.stack([p0, p1[t1], p1[t2], p0, p0])
        # integrate the uniforms exactly: enumerate the accept/reject pattern by choosing u
        base = _call(parent, Q, Pm, [0, t1, t2, t3, t4], neigh, 1, 2.0, [0.5] * 5, [0.5] * 5, keep_final_cdf=True)
        a = np.minimum(1.0, base["ratio"][0])
        dist = lambda row: np.diff(np.concatenate([[0.0], base["final_cdf"][0, row]])) / base["final_cdf"][0, row][-1]
        for first_node, pw in ((1, a[1]), (2, (1 - a[1]) * a[2])):
            tok = [0, t1, t2][first_node]
            first[tok] += w * pw
            child = 3 if first_node == 1 else 4
            ctok = t3 if first_node == 1 else t4
            pair[tok, ctok] += w * pw * a[child]
            pair[tok] += w * pw * (1 - a[child]) * dist(first_node)
            triple_bonus += w * pw * a[child] * dist(child) if tok == 0 and ctok == 0 else 0
        first += w * (1 - a[1]) * (1 - a[2]) * dist(0)
        # the walk must agree with the decisions for concrete uniforms
        for ua in ([0, 0.0, 0.0, 0.0, 0.0], [0, 0.999999, 0.0, 0.0, 0.0], [0, 0.999999, 0.999999, 0, 0]):
            o = _call(parent, Q, Pm, [0, t1, t2, t3, t4], neigh, 1, 2.0, ua, [0.5] * 5)
            d = o["decision"][0]
            cur, n = 0, 0
            for lvl_kids in ([1, 2],):
                nxt = next((c for c in lvl_kids if d[c]), None)
                if nxt is not None:
                    cur, n = nxt, 1
                    ch = 3 if nxt == 1 else 4
                    if d[ch]:
                        cur, n = ch, 2
            assert o["accept_len"][0] == n
            assert o["final_token"][0] == o["final_tok_all"][0, cur]
            assert list(o["path"][0][:n]) == ([cur] if n == 1 else ([parent[cur], cur] if n == 2 else []))
    assert np.max(np.abs(first - q0)) < 1e-12
    # P(first = x, second = y, first was an accepted draft) = P(first = x, accepted) * q1[x][y]
    acc_first = pair.sum(axis=1)
    assert np.max(np.abs(pair - acc_first[:, None] * q1)) < 1e-12
    # bonus token after the fully accepted path (0, 0) follows q2[0]
    assert np.max(np.abs(triple_bonus / triple_bonus.sum() - q2[0])) < 1e-12


# ------------------------------------------------------------------ Monte Carlo
def _monte_carlo_chunk(args):
    """First emitted tokens of n seeded runs of the oracle at a root with two drafted children
    (a worker of the test below: tokens from p, uniforms, then the oracle's own decisions and walk)."""
    seed, n, q, p = args
    g = np.random.default_rng(seed)
    V = len(q)
    parent = np.array([-1, 0, 0])
    toks = np.concatenate([np.zeros((n, 1), int), g.choice(V, size=(n, 2), p=p)], axis=1).astype(np.int32)
    tl = np.broadcast_to(_logits(q), (n, 3, V)); dl = np.broadcast_to(_logits(p), (n, 3, V))
    neigh = np.array([np.roll(np.arange(V), -i) for i in range(V)])
    o = relaxed_verify(parent, tl, dl, 0, V, toks, neigh, 1, 2.0, g.random((n, 3)), g.random((n, 3)))
    first = np.where(o["accept_len"] > 0, toks[np.arange(n), np.maximum(o["path"][:, 0], 0)], o["final_token"])
    return np.bincount(first, minlength=V)


def test_monte_carlo_unrelaxed_matches_target():
    # 10^6 seeded runs (eight chunks with seeds of their own, a few worker processes): with A = {x^}
    # the first emitted token follows the target exactly (App. A.2, Eq. 1-2)
    from concurrent.futures import ProcessPoolExecutor
    g = np.random.default_rng(2025)
    V, n_chunks, per = 6, 8, 125000
    n = n_chunks * per
    q = g.dirichlet(np.ones(V) * 0.7); p = g.dirichlet(np.ones(V) * 0.7)
    jobs = [(2025_000 + i, per, q, p) for i in range(n_chunks)]
    with ProcessPoolExecutor(max_workers=4) as pool:
        counts = sum(pool.map(_monte_carlo_chunk, jobs))
    assert counts.sum() == n >= 10 ** 6
    freq = counts / n
    assert np.all(np.abs(freq - q) < 4 * np.sqrt(q * (1 - q) / n) + 1e-9)
    chi2 = (n * (freq - q) ** 2 / q).sum()
    assert chi2 < 25.7                                 # chi^2_{5}, p = 1e-4
    # and a deliberately wrong target is rejected by the same statistic
    assert (n * (freq - p) ** 2 / p).sum() > 25.7
    # ... and so is a target that is off by one percent of its mass (the resolution 10^6 runs buy)
    q_off = q.copy(); q_off[0] += 0.01 * (1 - q[0]); q_off[1:] *= 0.99
    assert (n * (freq - q_off) ** 2 / q_off).sum() > 25.7


# ------------------------------------------------------- bound invariants (Sec. 4)
@pytest.mark.parametrize("rho", [0.0, 0.8])
def test_bound_invariants_and_monotonicity(rho):
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    kids = children_lists(parent)
    E = make_codebook(cfg)
    neigh = build_neighbours(E, 64)
    x = make_verify_inputs(cfg, parent, rho=rho)
    first_kids = [c[0] for c in kids if c]
    prev_mass = None
    for k, lam in [(1, 2.0), (4, 2.0), (16, 2.0), (64, 2.0), (64, 3.0), (64, 8.0)]:
        o = relaxed_verify(parent, x["target_logits"], x["drafter_logits"], 0, cfg.V, x["tokens"],
                           neigh, k, lam, x["u_accept"], x["u_final"])
        for c in range(1, cfg.M):
            qt, m, na = o["q_tok"][0, c], o["mass"][0, c], o["n_agg"][0, c]
            assert 1 <= na <= k
            assert qt <= m * (1 + 1e-15)
            assert m < lam * qt or na == 1
            assert o["ratio"][0, c] <= lam * qt / o["p_tok"][0, c] * (1 + 1e-12)
            assert o["ratio"][0, c] >= qt / o["p_tok"][0, c] * (1 - 1e-12)
        if prev_mass is not None:                      # first siblings see r = q: monotone in k and lambda
            assert np.all(o["mass"][0, first_kids] >= prev_mass - 1e-18)
        prev_mass = o["mass"][0, first_kids].copy()
    assert np.any(o["n_agg"][0, 1:] > 1)


def test_prefix_choice_brute_force():
    """|A| = the largest j whose prefix sum is below the cap (all prefixes enumerated)."""
    g = np.random.default_rng(5)
    V = 8
    for trial in range(40):
        q = g.dirichlet(np.ones(V) * 0.5); p = g.dirichlet(np.ones(V))
        lam = float(g.uniform(1.05, 6.0)); k = int(g.integers(1, V + 1))
        t = int(g.integers(V))
        neigh = np.array([[i] + [j for j in g.permutation(V) if j != i] for i in range(V)])
        o = _call([-1, 0], np.stack([q, q]), np.stack([p, p]), [0, t], neigh, k, lam, [0, 0.3], [0.1, 0.1])
        sums = [q[neigh[t][:j]].sum() for j in range(1, k + 1)]
        ok = [j for j in range(1, k + 1) if all(s < lam * q[t] for s in sums[1:j])]
        assert o["n_agg"][0, 1] == max(ok)
        assert o["mass"][0, 1] == pytest.approx(sums[max(ok) - 1], rel=1e-12)
        assert o["decision"][0, 1] == (1 if 0.3 < min(1.0, sums[max(ok) - 1] / p[t]) else 0)


def test_zero_probability_tokens():
    q = np.array([0.0, 0.5, 0.5, 0.0]); p = np.array([0.25, 0.25, 0.25, 0.25])
    neigh = np.array([[0, 1, 2, 3], [1, 0, 2, 3], [2, 3, 0, 1], [3, 2, 1, 0]])
    o = _call([-1, 0], np.stack([q, q]), np.stack([p, p]), [0, 0], neigh, 4, 3.0, [0, 0.0], [0.999999, 0.0])
    assert o["n_agg"][0, 1] == 1 and o["mass"][0, 1] == 0 and o["decision"][0, 1] == 0
    assert o["final_tok_all"][0, 0] in (1, 2) and o["final_tok_all"][0, 1] == 1


# ------------------------------------------------- additive (LANTERN) bound variant
def test_additive_bound_brute_force_and_reduction():
    """sum_A r < delta (Sec. 4, the LANTERN form), x^ always a member: |A| by enumerating all
    prefixes; delta <= q(x^) leaves A = {x^}, i.e. Eq. 1; and on a single child the additive bound
    with delta = lambda * q(x^) is the multiplicative one."""
    g = np.random.default_rng(11)
    V = 8
    grew = 0
    for trial in range(60):
        q = g.dirichlet(np.ones(V) * 0.5); p = g.dirichlet(np.ones(V))
        k = int(g.integers(1, V + 1)); t = int(g.integers(V))
        delta = float(g.uniform(0.02, 0.9))
        neigh = np.array([[i] + [j for j in g.permutation(V) if j != i] for i in range(V)])
        args = ([-1, 0], np.stack([q, q]), np.stack([p, p]), [0, t], neigh, k)
        o = _call(*args, delta, [0, 0.3], [0.1, 0.1], bound="additive")
        sums = [q[neigh[t][:j]].sum() for j in range(1, k + 1)]
        ok = [j for j in range(1, k + 1) if all(s < delta for s in sums[1:j])]
        assert o["n_agg"][0, 1] == max(ok)
        assert o["mass"][0, 1] == pytest.approx(sums[max(ok) - 1], rel=1e-12)
        assert o["mass"][0, 1] < delta or o["n_agg"][0, 1] == 1
        assert o["decision"][0, 1] == (1 if 0.3 < min(1.0, sums[max(ok) - 1] / p[t]) else 0)
        grew += int(o["n_agg"][0, 1] > 1)
        # no room under the bound: plain speculative sampling
        o0 = _call(*args, 0.999 * q[t], [0, 0.3], [0.1, 0.1], bound="additive")
        assert o0["n_agg"][0, 1] == 1 and o0["ratio"][0, 1] == pytest.approx(q[t] / p[t], rel=1e-12)
        # the same cap, written both ways
        lam = float(g.uniform(1.05, 6.0))
        om = _call(*args, lam, [0, 0.3], [0.1, 0.9], bound="multiplicative")
        oa = _call(*args, lam * np.float64(q[t]), [0, 0.3], [0.1, 0.9], bound="additive")
        for name in ("n_agg", "mass", "ratio", "decision", "final_tok_all"):
            assert np.array_equal(om[name], oa[name]), name
    assert grew > 10


def test_additive_bound_on_workload_rows():
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    E = make_codebook(cfg)
    neigh = build_neighbours(E, 64)
    x = make_verify_inputs(cfg, parent, rho=0.8)
    prev = None
    for delta in (1e-4, 0.01, 0.05, 0.3):
        o = relaxed_verify(parent, x["target_logits"], x["drafter_logits"], 0, cfg.V, x["tokens"],
                           neigh, 64, delta, x["u_accept"], x["u_final"], bound="additive")
        for c in range(1, cfg.M):
            qt, m, na = o["q_tok"][0, c], o["mass"][0, c], o["n_agg"][0, c]
            assert qt <= m * (1 + 1e-15) and (m < delta or na == 1)
        first = [c[0] for c in children_lists(parent) if c]
        if prev is not None:
            assert np.all(o["mass"][0, first] >= prev - 1e-18)      # monotone in delta where r = q
        prev = o["mass"][0, first].copy()
    assert np.any(o["n_agg"][0, 1:] > 1)
    with pytest.raises(ValueError):
        relaxed_verify(parent, x["target_logits"], x["drafter_logits"], 0, cfg.V, x["tokens"],
                       neigh, 64, 0.1, x["u_accept"], x["u_final"], bound="other")


# ------------------------------------------------- "skip violators" choice of A
def test_skip_rule_hand_example_and_prefix_comparison():
    """Worked by hand (Sec. 4 bound, lambda = 3, r(x^) = 0.1 -> cap 0.3), neighbours nearest first
    with r = 0.15, 0.3, 0.04, 0.2, 0.005:  0.1 + 0.15 = 0.25 fits; + 0.3 does not (skipped);
    + 0.04 = 0.29 fits; + 0.2 does not; + 0.005 = 0.295 fits.  A = {x^, n1, n3, n5}, mass 0.295;
    the prefix rule stops at the first violator: A = {x^, n1}, mass 0.25."""
    q = np.array([0.1, 0.15, 0.3, 0.04, 0.2, 0.005, 0.205])
    p = np.array([0.5, 0.1, 0.1, 0.1, 0.1, 0.05, 0.05])
    neigh = np.array([[0, 1, 2, 3, 4, 5, 6]] + [[i] + [j for j in range(7) if j != i] for i in range(1, 7)])
    kw = dict(keep_final_cdf=True)
    o = _call([-1, 0], np.stack([q, q]), np.stack([p, p]), [0, 0], neigh, 6, 3.0, [0, 0.55], [0.5, 0.5], rule="skip", **kw)
    assert o["n_agg"][0, 1] == 4 and o["mass"][0, 1] == pytest.approx(0.295, rel=1e-12)
    assert o["ratio"][0, 1] == pytest.approx(0.59, rel=1e-12) and o["decision"][0, 1] == 1
    # residual after a rejection: members n1, n3, n5 hold nothing, x^ holds 0.295
    adj = np.array([0.295, 0.0, 0.3, 0.0, 0.2, 0.0, 0.205])
    res = np.clip(adj - p, 0, None)
    cdf = o["final_cdf"][0, 0]
    assert np.allclose(np.diff(np.concatenate([[0.0], cdf])) / cdf[-1], res / res.sum(), atol=1e-12)
    o2 = _call([-1, 0], np.stack([q, q]), np.stack([p, p]), [0, 0], neigh, 6, 3.0, [0, 0.55], [0.5, 0.5])
    assert o2["n_agg"][0, 1] == 2 and o2["mass"][0, 1] == pytest.approx(0.25, rel=1e-12) and o2["decision"][0, 1] == 0


def test_skip_rule_maximal_superset_of_prefix_and_reductions():
    g = np.random.default_rng(21)
    V = 9
    hits = 0
    for trial in range(60):
        q = g.dirichlet(np.ones(V) * 0.7); p = g.dirichlet(np.ones(V))
        lam = float(g.uniform(0.5, 5.0)); k = int(g.integers(1, V + 1))
        t = int(g.integers(V))
        neigh = np.array([[i] + [j for j in g.permutation(V) if j != i] for i in range(V)])
        args = ([-1, 0], np.stack([q, q]), np.stack([p, p]), [0, t], neigh, k, lam, [0, 0.3], [0.1, 0.1])
        s = _call(*args, rule="skip", keep_final_cdf=True)
        f = _call(*args)
        cap = lam * q[t]
        cdf = s["final_cdf"][0, 0]
        if lam <= 1 or k == 1:
            assert s["n_agg"][0, 1] == 1 and s["mass"][0, 1] == pytest.approx(q[t], rel=1e-12)   # Eq. 1
        assert s["n_agg"][0, 1] >= f["n_agg"][0, 1] and s["mass"][0, 1] >= f["mass"][0, 1] - 1e-15
        assert s["mass"][0, 1] < cap or s["n_agg"][0, 1] == 1                # the bound of Sec. 4
        # independent replay: walk the list, a neighbour is out iff adding it to what is in breaks the bound
        inside, tot = [t], q[t]
        for j in neigh[t][1:k]:
            if not (tot + q[j] < cap):
                continue
            inside.append(int(j)); tot += q[j]
        assert s["n_agg"][0, 1] == len(inside) and s["mass"][0, 1] == pytest.approx(tot, rel=1e-12)
        for j in neigh[t][1:k]:                                               # maximal: nothing left out fits at the end
            if int(j) not in inside:
                assert s["mass"][0, 1] + q[j] >= cap * (1 - 1e-12)
        # the members' mass sits on x^ and nowhere else: the residual's support avoids them
        resid = np.diff(np.concatenate([[0.0], cdf]))
        assert all(resid[j] == 0 for j in inside[1:])
        hits += int(s["n_agg"][0, 1] > f["n_agg"][0, 1])
    assert hits > 5                                                           # the two rules do differ


# ------------------------------------------------- siblings drawn without replacement
def _first_token_distribution_without_replacement(q, p, n_sib, neigh, k, lam):
    """Exact law of the first emitted token at a root whose n_sib drafts are distinct tokens,
    drawn one after the other from p with the earlier draws removed."""
    V = len(q)
    parent = [-1] + [0] * n_sib
    out = np.zeros(V)
    Q = np.stack([q] * (n_sib + 1)); Pm = np.stack([p] * (n_sib + 1))
    for toks in itertools.permutations(range(V), n_sib):
        w, left = 1.0, 1.0
        for t in toks:                      # probability of drawing this ordered tuple
            w *= p[t] / left
            left -= p[t]
        if w == 0:
            continue
        o = _call(parent, Q, Pm, [0] + list(toks), neigh, k, lam, [0.5] * (n_sib + 1),
                  [0.5] * (n_sib + 1), keep_final_cdf=True, siblings="without_replacement")
        stay = 1.0
        for i, t in enumerate(toks):
            a = min(1.0, o["ratio"][0, i + 1])
            out[t] += w * stay * a
            stay *= 1.0 - a
        cdf = o["final_cdf"][0, 0]
        out += w * stay * np.diff(np.concatenate([[0.0], cdf])) / cdf[-1]
    return out


@pytest.mark.parametrize("n_sib", [1, 2, 3])
def test_without_replacement_output_distribution_is_target(n_sib):
    """Faithfulness (statement after Eq. 2) carries over to distinct drafts when A = {x^}."""
    g = np.random.default_rng(17 + n_sib)
    V = 5
    q = g.dirichlet(np.ones(V)); p = g.dirichlet(np.ones(V))
    neigh = np.array([np.roll(np.arange(V), -i) for i in range(V)])
    d = _first_token_distribution_without_replacement(q, p, n_sib, neigh, 1, 3.0)
    assert abs(d.sum() - 1) < 1e-12 and np.max(np.abs(d - q)) < 1e-12
    d = _first_token_distribution_without_replacement(q, p, n_sib, neigh, V, 0.9)
    assert np.max(np.abs(d - q)) < 1e-12


def test_without_replacement_drafter_probabilities_and_first_child():
    g = np.random.default_rng(3)
    V = 6
    q = g.dirichlet(np.ones(V)); p = g.dirichlet(np.ones(V))
    neigh = np.array([[i] + [j for j in range(V) if j != i] for i in range(V)])
    toks = [0, 4, 1, 3]
    args = ([-1, 0, 0, 0], np.stack([q] * 4), np.stack([p] * 4), toks, neigh, 3, 2.0, [0, .3, .3, .3], [.2] * 4)
    a = _call(*args, siblings="without_replacement")
    b = _call(*args)
    for f in ("mass", "ratio", "p_tok", "q_tok", "n_agg", "decision"):
        assert a[f][0, 1] == b[f][0, 1]                                       # the first child sees p itself
    assert a["p_tok"][0, 2] == pytest.approx(p[1] / (1 - p[4]), rel=1e-12)
    assert a["p_tok"][0, 3] == pytest.approx(p[3] / (1 - p[4] - p[1]), rel=1e-12)
    # a token that was already tried has no drafter mass left: certain acceptance if it has any target mass
    dup = _call([-1, 0, 0], np.stack([q] * 3), np.stack([p] * 3), [0, 2, 2], neigh, 1, 2.0, [0, .99, .99], [.2] * 3,
                siblings="without_replacement")
    assert dup["p_tok"][0, 2] == 0.0 and dup["decision"][0, 2] == 1
