"""GPU parity: lpp_relaxed_verify against the float64 oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from workloads import CONFIGS, static_tree, make_codebook, make_verify_inputs
from gpu_common import run_verify, compare_verify, sparse_neighbour_table

pytestmark = pytest.mark.gpu


def _case(cfg, rho, k=None, lam=None, items=None, topk=0, salt=0, additive=False):
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=rho, items=items, topk_filter=topk, salt=salt)
    E = make_codebook(cfg)
    k = cfg.k if k is None else k
    lam = cfg.lam if lam is None else lam
    neigh = sparse_neighbour_table(E, k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, lam, additive=additive)
    rep = compare_verify(parent, x, neigh, cfg.V, cfg.vocab_offset, k, lam, got, additive=additive)
    print(f"cfg{cfg.idx} rho={rho} k={k} lam={lam}: {rep} mean accept_len={got['accept_len'].mean():.2f}", flush=True)
    return rep, got


@pytest.mark.parametrize("rho", [0.0, 0.8])
@pytest.mark.parametrize("idx", [1, 2, 3])
def test_verify_parity_configs(idx, rho):
    rep, got = _case(CONFIGS[idx], rho)
    assert rep["nodes"] > 0 and rep["near_tie_decisions"] <= 2 and rep["nagg_ties"] <= 2


def test_verify_parity_lumina_like_strided_rows():
    rep, _ = _case(CONFIGS[4], 0.8)
    assert rep["nodes"] == 60


def test_verify_parity_stress_full_batch():
    rep, got = _case(CONFIGS[5], 0.8)
    assert rep["nodes"] + rep["skipped_after_tie"] == 16 * 128        # (nodes counts the tied ones too)
    assert got["accept_len"].max() >= 2


@pytest.mark.parametrize("k,lam", [(1, 3.0), (1000, 1.0), (1000, 0.5), (7, 50.0), (1000, 1e9)])
def test_verify_special_cases(k, lam):
    cfg = CONFIGS[3].scaled(B=1)
    rep, got = _case(cfg, 0.8, k=k, lam=lam)
    if k == 1 or lam <= 1:
        pass  # reduces to plain speculative sampling; the oracle pins that case


@pytest.mark.parametrize("idx,delta", [(1, 0.05), (3, 0.01), (3, 0.2), (4, 0.05)])
def test_verify_additive_bound_parity(idx, delta):
    """The LANTERN form of the bound (sum over A below delta), same kernel, other cap."""
    cfg = CONFIGS[idx]
    rep, got = _case(cfg, 0.8, lam=delta, additive=True)
    assert rep["nodes"] > 0 and rep["near_tie_decisions"] <= 2 and rep["nagg_ties"] <= 2
    # and it really is another rule than the multiplicative one with the same number
    _, mult = _case(cfg, 0.8, lam=delta)
    assert not np.array_equal(got["n_agg"], mult["n_agg"])


def test_verify_topk_filtered_targets_long_prefixes():
    cfg = CONFIGS[3].scaled(B=2)
    rep, got = _case(cfg, 0.8, topk=2000)
    assert rep["nodes"] > 0


def test_verify_ragged_vocab_and_unaligned_offset():
    # V not a multiple of 4, odd offset: exercises the scalar-load path and the zero tail
    cfg = CONFIGS[2].scaled(V=5003, ldv=5100, vocab_offset=3, k=37, N=26)
    rep, _ = _case(cfg, 0.8)
    assert rep["nodes"] == 26
    cfg = CONFIGS[1].scaled(V=33, ldv=40, vocab_offset=1, k=33)
    rep, _ = _case(cfg, 0.5, lam=4.0)


def test_verify_single_row_tree_and_minimal_outputs():
    cfg = CONFIGS[1]
    parent = np.array([-1], dtype=np.int32)
    tree = lpp.Tree(parent)
    x = make_verify_inputs(cfg, parent)
    neigh = np.arange(cfg.V, dtype=np.int32)[:, None].copy()
    got = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, 1, 2.0, want_all=False)
    from oracle import relaxed_verify
    want = relaxed_verify(parent, x["target_logits"], x["drafter_logits"], 0, cfg.V, x["tokens"], neigh, 1, 2.0,
                          x["u_accept"], x["u_final"])
    assert got["accept_len"][0] == 0 and got["path"][0, 0] == -1
    assert got["final_token"][0] == want["final_token"][0]


def test_verify_identical_drafter_and_target():
    # p == q and no relaxation: every node is accepted (ratio exactly 1), residual stays r
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=1.0)
    assert np.array_equal(x["target_logits"], x["drafter_logits"])
    E = make_codebook(cfg)
    neigh = sparse_neighbour_table(E, 16, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    got = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, 1, 2.0)
    assert np.all(got["decision"][0, 1:] == 1) and np.all(got["ratio"][0, 1:] == 1.0)
    assert got["accept_len"][0] == 4
    compare_verify(parent, x, neigh, cfg.V, 0, 1, 2.0, got)


def test_verify_deterministic_run_to_run():
    cfg = CONFIGS[3].scaled(B=2)
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=0.8)
    neigh = sparse_neighbour_table(make_codebook(cfg), cfg.k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    a = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, cfg.k, cfg.lam)
    b = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, cfg.k, cfg.lam)
    for n in a:
        assert np.array_equal(a[n], b[n]), n


def test_verify_argument_errors_on_device():
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    x = make_verify_inputs(cfg, parent)
    neigh = np.zeros((cfg.V, 4), dtype=np.int32)
    with pytest.raises(lpp.LppError) as e:
        run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, 5, 2.0)       # k > kstride
    assert e.value.status == lpp.LPP_EINVAL
    with pytest.raises(lpp.LppError) as e:
        run_verify(tree, x, neigh, cfg.V, 8, cfg.ldv, 4, 2.0)       # slice leaves the row
    assert e.value.status == lpp.LPP_EINVAL


def test_verify_walk_by_a_row_other_than_the_root_and_repeated_calls():
    # The row with the most children is not row 0 here: with the whole grid resident its block is
    # the one that collects the other rows' results and walks.  Several calls on one handle, with
    # different inputs, each against the oracle: what a call leaves behind must not reach the next.
    cfg = CONFIGS[1]
    parent = np.array([-1, 0, 1, 1, 1, 1, 0, 6, 2, 2], dtype=np.int32)
    tree = lpp.Tree(parent)
    E = make_codebook(cfg)
    for salt, rho in ((0, 0.0), (1, 0.8), (2, 0.5), (3, 1.0)):
        x = make_verify_inputs(cfg, parent, rho=rho, salt=salt)
        neigh = sparse_neighbour_table(E, cfg.k, x["tokens"][:, 1:], cfg.V)
        got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam)
        rep = compare_verify(parent, x, neigh, cfg.V, cfg.vocab_offset, cfg.k, cfg.lam, got)
        assert rep["nodes"] > 0


def test_verify_walk_that_gives_up_is_loud_and_harms_no_later_call():
    # The bounded wait of the walking block is made to run out from the host (no kernel hangs or
    # faults: the block just does not look at the results).  The call must say so in its outputs
    # and the handle must count it; the rows' results of that call, which nobody took, must not be
    # taken for the next call's: the next calls, with other inputs, match the oracle with no reset.
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    E = make_codebook(cfg)
    tree = lpp.Tree(parent)
    assert tree.walk_gave_up() == 0

    def good_call(salt):
        x = make_verify_inputs(cfg, parent, rho=0.8, salt=salt)
        neigh = sparse_neighbour_table(E, cfg.k, x["tokens"][:, 1:], cfg.V)
        got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam)
        compare_verify(parent, x, neigh, cfg.V, cfg.vocab_offset, cfg.k, cfg.lam, got)

    good_call(0)
    for round_ in range(2):
        x = make_verify_inputs(cfg, parent, rho=0.8, salt=10 + round_)
        neigh = sparse_neighbour_table(E, cfg.k, x["tokens"][:, 1:], cfg.V)
        tree.set_walk_patience(-1)
        got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam, want_all=False)
        assert np.all(got["accept_len"] == -1) and np.all(got["final_token"] == -1) and np.all(got["path"] == -1)
        assert tree.walk_gave_up() == (round_ + 1) * cfg.B
        tree.set_walk_patience(1 << 19)
        good_call(20 + round_)      # other inputs: a stale word taken for this call's would show
        good_call(30 + round_)
    tree.walk_reset()
    torch.cuda.synchronize()
    assert tree.walk_gave_up() == 0
    good_call(40)
    with pytest.raises(lpp.LppError):
        tree.set_walk_patience(-2)


def test_verify_many_calls_on_one_handle_tags_wrap():
    # The call number inside the rows' words wraps after 512 calls: 600 calls on one handle, the
    # last ones checked (inputs alternate, so a word of the call before would be a wrong one).
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    E = make_codebook(cfg)
    tree = lpp.Tree(parent)
    xs = [make_verify_inputs(cfg, parent, rho=0.8, salt=s) for s in (0, 1)]
    neigh = sparse_neighbour_table(E, cfg.k, np.concatenate([x["tokens"][:, 1:].ravel() for x in xs]), cfg.V)
    for i in range(600):
        x = xs[i % 2]
        got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam, want_all=False)
        if i in (0, 1, 510, 511, 512, 513, 598, 599):
            got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam)
            compare_verify(parent, x, neigh, cfg.V, cfg.vocab_offset, cfg.k, cfg.lam, got)
    assert tree.walk_gave_up() == 0


@pytest.mark.parametrize("B,parent", [(120, [-1, 0]), (85, [-1, 0, 0]), (64, [-1, 0, 1, 2])])
def test_verify_many_items_with_the_whole_grid_resident(B, parent):
    # Many items of a tiny tree: every item has its own walking block and its own stretch of the
    # handle's words; B * M stays within one block per compute unit.
    cfg = CONFIGS[1].scaled(B=B, V=256, ldv=256, k=8)
    parent = np.array(parent, dtype=np.int32)
    x = make_verify_inputs(cfg, parent, rho=0.7)
    neigh = sparse_neighbour_table(make_codebook(cfg), cfg.k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    for _ in range(2):
        got = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, cfg.k, cfg.lam)
        rep = compare_verify(parent, x, neigh, cfg.V, 0, cfg.k, cfg.lam, got)
    assert rep["walks_compared"] >= B - 2


@pytest.mark.parametrize("salt", [0, 1, 2, 3])
@pytest.mark.parametrize("V,k,lam", [(64, 8, 2.0), (48, 48, 6.0), (300, 32, 1.5)])
def test_verify_resident_grid_siblings_that_repeat_tokens_and_join_later_sets(V, k, lam, salt):
    # Tiny vocabularies, a drafter close to the target, four siblings under the root and two under each
    # of them: drafted tokens repeat among siblings, a token that carries an earlier sibling's
    # mass turns up inside a later sibling's neighbourhood, whole neighbourhoods fit under the bound
    # (k = V with a wide bound).  B * M = 247 rows: the whole grid is resident at once.
    cfg = CONFIGS[1].scaled(V=V, ldv=V + 4, vocab_offset=4, k=k, N=12, branching=(4, 2), B=19)
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=0.9, salt=salt)
    neigh = sparse_neighbour_table(make_codebook(cfg), k, x["tokens"][:, 1:], V)
    tree = lpp.Tree(parent)
    got = run_verify(tree, x, neigh, V, cfg.vocab_offset, cfg.ldv, k, lam)
    rep = compare_verify(parent, x, neigh, V, cfg.vocab_offset, k, lam, got, max_slack_used=12)
    print(f"V={V} k={k} lam={lam} salt={salt}: {rep}", flush=True)
    assert rep["nodes"] + rep["skipped_after_tie"] == 19 * 12
    toks = x["tokens"]
    kids = [[c for c in range(len(parent)) if parent[c] == P] for P in range(len(parent))]
    repeats = sum(len(set(toks[b, c])) < len(c) for b in range(19) for c in kids if len(c) > 1)
    assert repeats > 0 or V > 100, "no sibling repeats a token: the case no longer exercises that path"


@pytest.mark.parametrize("k,lam", [(1, 2.0), (8, 0.9), (8, 3.0)])
def test_verify_identical_drafter_and_target_with_repeated_tokens(k, lam):
    # p == q on a tiny vocabulary with four siblings: without relaxation (k = 1, or a bound that
    # admits nobody) every level after a child is empty and r stays as it was, also for a token
    # that is drafted twice; with relaxation the residual sits on the drafted token alone.
    V = 32
    cfg = CONFIGS[1].scaled(V=V, ldv=V, k=k, N=12, branching=(4, 2), B=19)
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=1.0)
    assert np.array_equal(x["target_logits"], x["drafter_logits"])
    neigh = sparse_neighbour_table(make_codebook(cfg), k, x["tokens"][:, 1:], V)
    got = run_verify(lpp.Tree(parent), x, neigh, V, 0, cfg.ldv, k, lam)
    if k == 1 or lam <= 1:
        assert np.all(got["decision"][:, 1:] == 1) and np.all(got["ratio"][:, 1:] == 1.0)
    rep = compare_verify(parent, x, neigh, V, 0, k, lam, got, max_slack_used=12)
    print(f"k={k} lam={lam}: {rep}", flush=True)
