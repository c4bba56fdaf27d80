"""GPU parity at the limits the header states: widest vocabulary (the 1024-lane rows), most rows,
a row with many children, more batch items than fused-walk counters, longest neighbour lists;
attention with the most rows, long caches and the float32 length limit; the largest codebook."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from oracle import tree_attention, build_neighbours
from workloads import CONFIGS, static_tree, make_codebook, make_verify_inputs, make_attention_inputs
from gpu_common import (run_verify, compare_verify, sparse_neighbour_table, run_attention, attention_error,
                        run_knn)

pytestmark = pytest.mark.gpu


def _verify_case(cfg, rho=0.8, k=None, lam=None, opts=None, **okw):
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=rho)
    k = cfg.k if k is None else k
    lam = cfg.lam if lam is None else lam
    neigh = sparse_neighbour_table(make_codebook(cfg), k, x["tokens"][:, 1:], cfg.V)
    got = run_verify(lpp.Tree(parent), x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, k, lam, opts=opts)
    rep = compare_verify(parent, x, neigh, cfg.V, cfg.vocab_offset, k, lam, got, **okw)
    print(f"V={cfg.V} M={cfg.M} B={cfg.B} k={k}: {rep}", flush=True)
    return rep


@pytest.mark.parametrize("V,ldv,off", [(32768, 32768, 0), (20001, 20100, 3), (16388, 16400, 4)])
def test_verify_widest_vocabulary(V, ldv, off):
    cfg = CONFIGS[2].scaled(V=V, ldv=ldv, vocab_offset=off, k=1000, B=2)
    rep = _verify_case(cfg)
    assert rep["nodes"] == 2 * 26
    opts = dict(rule=lpp.LPP_RULE_SKIP, siblings=lpp.LPP_SIBLINGS_DISTINCT)
    _verify_case(cfg, opts=opts, rule="skip", siblings="without_replacement")


def test_verify_most_rows_and_a_row_with_many_children():
    cfg = CONFIGS[2].scaled(V=4096, ldv=4096, k=64, N=255, branching=(15, 16), B=2)      # M = 256
    rep = _verify_case(cfg)
    assert rep["nodes"] + rep["skipped_after_tie"] == 2 * 255
    cfg = CONFIGS[2].scaled(V=2048, ldv=2048, k=40, N=40, branching=(40,), B=3)          # 40 children of the root
    rep = _verify_case(cfg)
    assert rep["nodes"] + rep["skipped_after_tie"] == 3 * 40
    opts = dict(rule=lpp.LPP_RULE_SKIP, siblings=lpp.LPP_SIBLINGS_DISTINCT)
    _verify_case(cfg, opts=opts, rule="skip", siblings="without_replacement")


@pytest.mark.parametrize("B", [1, 3])
def test_verify_row_with_more_children_than_a_wave_has_lanes(B):
    # 100 children of the root, two more below the first of them: the per-child results of such
    # a row are kept and written out by more than one wave.  B = 1: the whole grid is resident
    # (103 blocks; the root's block walks, its second wave owning children 64..99 as well);
    # B = 3: more blocks than compute units, the walk by tickets.
    cfg = CONFIGS[1].scaled(V=1024, ldv=1024, k=16, B=B)
    parent = np.array([-1] + [0] * 100 + [1, 1], dtype=np.int32)
    x = make_verify_inputs(cfg, parent, rho=0.3)
    neigh = sparse_neighbour_table(make_codebook(cfg), cfg.k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    got = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, cfg.k, cfg.lam)
    rep = compare_verify(parent, x, neigh, cfg.V, 0, cfg.k, cfg.lam, got)
    print(f"100 children, B={B}: {rep}", flush=True)
    assert rep["nodes"] + rep["skipped_after_tie"] == B * 102
    opts = dict(rule=lpp.LPP_RULE_SKIP, siblings=lpp.LPP_SIBLINGS_DISTINCT)
    got = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, cfg.k, cfg.lam, opts=opts)
    compare_verify(parent, x, neigh, cfg.V, 0, cfg.k, cfg.lam, got, rule="skip", siblings="without_replacement")


def test_verify_two_rows_with_more_children_than_a_wave_has_lanes():
    # 70 children of the root and 70 of its first child (141 blocks, the whole grid resident): the
    # root's block walks; row 1 does not, and its second wave sends children 64..69 on their way to
    # the walking block itself.  Twice on one handle, with other inputs.
    cfg = CONFIGS[1].scaled(V=1024, ldv=1024, k=16, B=1)
    parent = np.array([-1] + [0] * 70 + [1] * 70, dtype=np.int32)
    tree = lpp.Tree(parent)
    E = make_codebook(cfg)
    for salt in (0, 1):
        x = make_verify_inputs(cfg, parent, rho=0.3, salt=salt)
        neigh = sparse_neighbour_table(E, cfg.k, x["tokens"][:, 1:], cfg.V)
        got = run_verify(tree, x, neigh, cfg.V, 0, cfg.ldv, cfg.k, cfg.lam)
        rep = compare_verify(parent, x, neigh, cfg.V, 0, cfg.k, cfg.lam, got)
        assert rep["nodes"] + rep["skipped_after_tie"] == 140
    assert tree.walk_gave_up() == 0


def test_verify_more_items_than_walk_counters():
    cfg = CONFIGS[1].scaled(V=64, ldv=64, k=4, N=3, branching=(2, 1), B=4100)
    # (tiny vocabulary, drafter close to the target: siblings often repeat a token, the input on which
    #  Eq. 2's cancellation shows -- up to 0.2 % of the values may need the float32 allowance here)
    rep = _verify_case(cfg, rho=0.9, max_slack_used=24)
    assert rep["walks_compared"] > 4000 and rep["max_slack_rel"] < 5e-3


def test_verify_longest_neighbour_lists():
    cfg = CONFIGS[3].scaled(B=1, N=12, branching=(3, 3))
    rep = _verify_case(cfg, k=4096, lam=40.0)
    assert rep["nodes"] == 12
    with pytest.raises(lpp.LppError) as e:
        _verify_case(cfg, k=4097, lam=40.0)
    assert e.value.status == lpp.LPP_EUNSUPPORTED


@pytest.mark.parametrize("Dh", [64, 128])
def test_attention_most_rows(Dh):
    cfg = CONFIGS[2].scaled(N=255, branching=(15, 16), H=3, S=333, Dh=Dh, B=2)
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    seq_len = np.array([333, 100], dtype=np.int32)
    got = run_attention(lpp.Tree(parent), att, cfg, seq_len=seq_len)
    want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent, seq_len=seq_len)
    err = attention_error(got, want)
    print(f"M=256 Dh={Dh}: err={err:.3e}", flush=True)
    assert err <= 2e-2


def test_attention_long_cache_and_float32_length_limit():
    cfg = CONFIGS[3].scaled(H=1, S=70000, B=1)
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    got = run_attention(lpp.Tree(parent), att, cfg)
    want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent)
    assert attention_error(got, want) <= 2e-2
    cfg = CONFIGS[1].scaled(H=1, S=36864 - 16, B=1)                     # S + M = the float32 limit
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    tree = lpp.Tree(parent)
    got = run_attention(tree, att, cfg)
    want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent)
    assert attention_error(got, want) <= 1e-4
    att1 = make_attention_inputs(cfg.scaled(S=cfg.S + 1))
    with pytest.raises(lpp.LppError) as e:
        run_attention(tree, att1, cfg.scaled(S=cfg.S + 1))
    assert e.value.status == lpp.LPP_EUNSUPPORTED


def test_knn_largest_codebook_and_longest_lists():
    g = np.random.default_rng(4)
    E = g.standard_normal((65536, 8))
    E = (E / np.linalg.norm(E, axis=1, keepdims=True)).astype(np.float32)
    got = run_knn(E, 4096)
    rows = np.concatenate([[0, 65535], g.choice(65536, size=12, replace=False)])
    want = build_neighbours(E, 4096, rows=rows)
    assert np.array_equal(got[rows], want)
    E = g.standard_normal((4096, 256))
    E = (E / np.linalg.norm(E, axis=1, keepdims=True)).astype(np.float32)
    got = run_knn(E, 4096)                                              # k = V: every row a permutation
    rows = np.arange(0, 4096, 257)
    assert np.array_equal(got[rows], build_neighbours(E, 4096, rows=rows))
    assert np.array_equal(np.sort(got, axis=1), np.broadcast_to(np.arange(4096, dtype=np.int32), got.shape))
