"""GPU parity: lpp_relaxed_verify_opts (the other choice of A, distinct siblings, and their
combinations with both bounds) against the float64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from workloads import CONFIGS, static_tree, make_codebook, make_verify_inputs
from gpu_common import run_verify, compare_verify, sparse_neighbour_table

pytestmark = pytest.mark.gpu


def _case(cfg, rho, skip=False, distinct=False, k=None, lam=None, additive=False, topk=0, salt=0, dup=False):
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=rho, topk_filter=topk, salt=salt)
    if dup:                                     # a token handed in twice under one parent
        x["tokens"][:, 2] = x["tokens"][:, 1]
    E = make_codebook(cfg)
    k = cfg.k if k is None else k
    lam = cfg.lam if lam is None else lam
    neigh = sparse_neighbour_table(E, k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    opts = dict(rule=lpp.LPP_RULE_SKIP if skip else lpp.LPP_RULE_PREFIX,
                siblings=lpp.LPP_SIBLINGS_DISTINCT if distinct else lpp.LPP_SIBLINGS_IID)
    got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, lam, additive=additive, opts=opts)
    rep = compare_verify(parent, x, neigh, cfg.V, cfg.vocab_offset, k, lam, got, additive=additive,
                         rule="skip" if skip else "prefix",
                         siblings="without_replacement" if distinct else "with_replacement")
    print(f"cfg{cfg.idx} rho={rho} skip={skip} distinct={distinct} k={k} lam={lam}: {rep} "
          f"mean n_agg={got['n_agg'][:, 1:].mean():.1f} accept_len={got['accept_len'].mean():.2f}", flush=True)
    return rep, got, (tree, x, neigh, k, lam)


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
@pytest.mark.parametrize("skip,distinct", [(True, False), (False, True), (True, True)])
def test_opts_parity_configs(idx, skip, distinct):
    rep, got, _ = _case(CONFIGS[idx], 0.8, skip=skip, distinct=distinct)
    assert rep["nodes"] > 0 and rep["near_tie_decisions"] <= 2
    assert rep["nagg_ties"] <= (6 if skip else 2)


def test_opts_defaults_equal_the_plain_entry_points():
    cfg = CONFIGS[3]
    rep, got, (tree, x, neigh, k, lam) = _case(cfg, 0.8)
    plain = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, lam)
    for n in got:
        assert np.array_equal(got[n], plain[n]), n
    add = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, 0.05, additive=True)
    add2 = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, 0.05, additive=True,
                      opts=dict(rule=lpp.LPP_RULE_PREFIX, siblings=lpp.LPP_SIBLINGS_IID))
    for n in add:
        assert np.array_equal(add[n], add2[n]), n


def test_opts_skip_rule_differs_from_prefix_and_contains_it():
    cfg = CONFIGS[3]
    _, sk, (tree, x, neigh, k, lam) = _case(cfg, 0.8, skip=True)
    pre = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, lam)
    assert np.all(sk["n_agg"] >= pre["n_agg"]) and np.any(sk["n_agg"] > pre["n_agg"])
    # first children see the same r under both rules: their mass can only grow (up to float32 rounding order)
    parent = static_tree(cfg.branching, cfg.N)
    first = [c for c in range(1, cfg.M) if c == 1 or parent[c] != parent[c - 1]]
    assert np.all(sk["mass"][:, first] >= pre["mass"][:, first] * (1 - 1e-5))


@pytest.mark.parametrize("additive,lam", [(False, 3.0), (True, 0.02)])
def test_opts_skip_rule_stress_full_batch_and_filtered_targets(additive, lam):
    rep, got, _ = _case(CONFIGS[5], 0.8, skip=True, distinct=True, additive=additive, lam=lam)
    assert rep["nodes"] + rep["skipped_after_tie"] == 16 * 128        # (nodes counts the tied ones too)
    rep, _, _ = _case(CONFIGS[3].scaled(B=2), 0.8, skip=True, additive=additive, lam=lam, topk=2000)
    assert rep["nodes"] > 0


@pytest.mark.parametrize("k,lam", [(1, 3.0), (1000, 1.0), (1000, 0.5), (7, 50.0), (1000, 1e9), (4096, 1.5)])
def test_opts_special_cases(k, lam):
    cfg = CONFIGS[3].scaled(B=1)
    _case(cfg, 0.8, skip=True, distinct=True, k=k, lam=lam)


def test_opts_distinct_siblings_repeated_token_and_ragged_vocab():
    rep, got, _ = _case(CONFIGS[2], 0.8, distinct=True, dup=True)
    assert got["p_tok"][0, 2] == 0.0                       # the second copy has no drafter mass left
    cfg = CONFIGS[2].scaled(V=5003, ldv=5100, vocab_offset=3, k=37, N=26)
    _case(cfg, 0.8, skip=True, distinct=True)
    cfg = CONFIGS[1].scaled(V=33, ldv=40, vocab_offset=1, k=33)
    _case(cfg, 0.5, skip=True, distinct=True, lam=4.0)


def test_opts_argument_errors():
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=0.5)
    neigh = sparse_neighbour_table(make_codebook(cfg), cfg.k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    for bad in (dict(rule=2), dict(siblings=-1), dict(rule=0, siblings=7)):
        with pytest.raises(lpp.LppError) as e:
            run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam, opts=bad)
        assert e.value.status == lpp.LPP_EINVAL


@pytest.mark.parametrize("additive,lam", [(False, 3.0), (True, 0.05)])
def test_opts_everything_at_once_front_end_skip_rule_distinct_siblings(additive, lam):
    """Guidance + top-k in front, the skip rule and distinct siblings behind, either bound: the oracle
    pipeline is sampling_frontend -> relaxed_verify with the same options."""
    from oracle import sampling_frontend
    from gpu_common import DEV, dev
    cfg = CONFIGS[3].scaled(B=2)
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    x = make_verify_inputs(cfg, parent, rho=0.8, salt=3)
    y = make_verify_inputs(cfg, parent, rho=0.0, salt=103)
    V, off, k = cfg.V, cfg.vocab_offset, cfg.k
    B, M = x["tokens"].shape
    neigh = sparse_neighbour_table(make_codebook(cfg), k, x["tokens"][:, 1:], V)
    out = {"accept_len": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "path": torch.full((B, max(tree.depth, 1)), -7, dtype=torch.int32, device=DEV),
           "final_token": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "decision": torch.full((B, M), 9, dtype=torch.uint8, device=DEV),
           "ratio": torch.zeros((B, M), device=DEV), "mass": torch.zeros((B, M), device=DEV),
           "n_agg": torch.zeros((B, M), dtype=torch.int32, device=DEV),
           "q_tok": torch.zeros((B, M), device=DEV), "p_tok": torch.zeros((B, M), device=DEV),
           "final_tok_all": torch.full((B, M), -7, dtype=torch.int32, device=DEV)}
    ws = torch.empty(lpp.lpp_relaxed_verify_workspace(tree, B, V, k), dtype=torch.uint8, device=DEV)
    lpp.lpp_relaxed_verify_opts(tree, dev(x["target_logits"]), dev(x["drafter_logits"]), cfg.ldv, off, V, B,
                                dev(x["tokens"]), dev(neigh), neigh.shape[1], k, dev(x["u_accept"]), dev(x["u_final"]),
                                out, ws, bound=lpp.LPP_BOUND_ADDITIVE if additive else lpp.LPP_BOUND_MULTIPLICATIVE,
                                bound_value=lam, rule=lpp.LPP_RULE_SKIP, siblings=lpp.LPP_SIBLINGS_DISTINCT,
                                uncond_logits=dev(y["target_logits"]), cfg_scale=3.0, top_k=2000)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in out.items()}
    filt = sampling_frontend(x["target_logits"], y["target_logits"], 3.0, 2000, off, V)
    rep = compare_verify(parent, dict(x, target_logits=filt), neigh, V, off, k, lam, got, additive=additive,
                         rule="skip", siblings="without_replacement")
    print(f"front end + skip + distinct, additive={additive}: {rep}", flush=True)
    assert rep["nodes"] > 0 and rep["near_tie_decisions"] <= 2
