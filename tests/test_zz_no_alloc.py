"""GPU: lpp_relaxed_verify_static (the entry point that allocates nothing: its walk words live in
a static device array of the library) against lpp_relaxed_verify, through the C ABI.

Same kernels, so every output must agree bit for bit.  Two calls in a row, the second with a
smaller input (the array keeps the first call's words), then a shape whose whole grid is
resident at once, then the size limit."""
import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from workloads import CONFIGS, static_tree, make_codebook, make_verify_inputs
from gpu_common import DEV, dev, run_verify, sparse_neighbour_table

pytestmark = pytest.mark.gpu

NAMES = ("accept_len", "path", "final_token", "decision", "ratio", "mass", "n_agg", "q_tok", "p_tok", "final_tok_all")


def _run_static(tree, x, neigh, cfg):
    B, M = x["tokens"].shape
    depth = max(tree.depth, 1)
    d = {n: dev(x[n]) for n in ("target_logits", "drafter_logits", "tokens", "u_accept", "u_final")}
    out = {"accept_len": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "path": torch.full((B, depth), -7, dtype=torch.int32, device=DEV),
           "final_token": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "decision": torch.full((B, M), 9, dtype=torch.uint8, device=DEV),
           "ratio": torch.zeros((B, M), device=DEV), "mass": torch.zeros((B, M), device=DEV),
           "n_agg": torch.zeros((B, M), dtype=torch.int32, device=DEV),
           "q_tok": torch.zeros((B, M), device=DEV), "p_tok": torch.zeros((B, M), device=DEV),
           "final_tok_all": torch.full((B, M), -7, dtype=torch.int32, device=DEV)}
    dn = dev(neigh)
    torch.cuda.synchronize()
    lpp.lpp_relaxed_verify_static(tree, d["target_logits"], d["drafter_logits"], cfg.ldv, cfg.vocab_offset, cfg.V, B,
                                  d["tokens"], dn, neigh.shape[1], cfg.k, cfg.lam, d["u_accept"], d["u_final"], out)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy() for n, t in out.items()}


def _both(cfg, rho=0.8):
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent, rho=rho)
    neigh = sparse_neighbour_table(make_codebook(cfg), cfg.k, x["tokens"][:, 1:], cfg.V)
    tree = lpp.Tree(parent)
    want = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam)
    got = _run_static(tree, x, neigh, cfg)
    for n in NAMES:
        assert np.array_equal(got[n], want[n], equal_nan=True) if got[n].dtype.kind == "f" else np.array_equal(got[n], want[n]), n
    assert np.all(got["accept_len"] >= 0)
    return got


def test_static_entry_point_matches_workspace_entry_point_twice_then_smaller():
    big = CONFIGS[3].scaled(B=8)                 # 488 rows: more blocks than compute units, walk by tickets through the array
    small = CONFIGS[2].scaled(B=12)              # 324 rows, another tree, fewer words
    print("static verify: B=8 config-3 rows", flush=True)
    a = _both(big)
    print("static verify: B=12 config-2 rows (smaller)", flush=True)
    b = _both(small)
    print("static verify: B=8 again", flush=True)
    c = _both(big)
    for n in NAMES:
        assert np.array_equal(a[n], c[n], equal_nan=True) if a[n].dtype.kind == "f" else np.array_equal(a[n], c[n]), n
    assert a["accept_len"].max() >= 1 and b["accept_len"].shape == (12,)


def test_static_entry_point_whole_grid_resident_and_size_limit():
    print("static verify: config 3 as it is (grid resident at once)", flush=True)
    _both(CONFIGS[3])
    # the array holds LPP_STATIC_MAX_NODES rows: one more is refused before anything is enqueued
    parent = np.array([-1, 0], dtype=np.int32)
    tree = lpp.Tree(parent)
    B = 65536 // 2 + 1
    one = torch.zeros(1, device=DEV)
    with pytest.raises(lpp.LppError) as e:
        lpp.lpp_relaxed_verify_static(tree, one, one, 64, 0, 64, B, one, one, 4, 4, 2.0, one, one,
                                      {"accept_len": one, "path": one, "final_token": one})
    assert e.value.status == lpp.LPP_EUNSUPPORTED
