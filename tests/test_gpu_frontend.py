"""GPU parity: lpp_relaxed_verify_sampled (guidance + top-k fused into the target load) against the
oracle pipeline sampling_frontend -> relaxed_verify, through the C ABI.  Which tokens survive the
top-k is an integer decision: the kernel's probabilities must be zero exactly where the oracle's
filtered logits are -inf (checked through q_tok of drafted tokens and the final draws)."""
import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from oracle import sampling_frontend
from workloads import CONFIGS, static_tree, make_codebook, make_verify_inputs
from gpu_common import DEV, dev, compare_verify, sparse_neighbour_table

pytestmark = pytest.mark.gpu


def _run(cfg, scale, top_k, guide=True, salt=0):
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    x = make_verify_inputs(cfg, parent, rho=0.8, salt=salt)
    y = make_verify_inputs(cfg, parent, rho=0.0, salt=salt + 100)      # an unrelated row set: the null-conditioned rows
    cond, uncond = x["target_logits"], y["target_logits"]
    B, M = x["tokens"].shape
    V, off, k = cfg.V, cfg.vocab_offset, cfg.k
    neigh = sparse_neighbour_table(make_codebook(cfg), k, x["tokens"][:, 1:], V)
    depth = max(tree.depth, 1)
    out = {"accept_len": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "path": torch.full((B, depth), -7, dtype=torch.int32, device=DEV),
           "final_token": torch.full((B,), -7, dtype=torch.int32, device=DEV),
           "decision": torch.full((B, M), 9, dtype=torch.uint8, device=DEV),
           "ratio": torch.zeros((B, M), device=DEV), "mass": torch.zeros((B, M), device=DEV),
           "n_agg": torch.zeros((B, M), dtype=torch.int32, device=DEV),
           "q_tok": torch.zeros((B, M), device=DEV), "p_tok": torch.zeros((B, M), device=DEV),
           "final_tok_all": torch.full((B, M), -7, dtype=torch.int32, device=DEV)}
    ws = torch.empty(lpp.lpp_relaxed_verify_workspace(tree, B, V, k), dtype=torch.uint8, device=DEV)
    lpp.lpp_relaxed_verify_sampled(tree, dev(cond), dev(uncond) if guide else None, scale, top_k,
                                   dev(x["drafter_logits"]), cfg.ldv, off, V, B, dev(x["tokens"]), dev(neigh),
                                   neigh.shape[1], k, cfg.lam, dev(x["u_accept"]), dev(x["u_final"]), out, ws)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in out.items()}
    filt = sampling_frontend(cond, uncond if guide else cond, scale if guide else 0.0, top_k, off, V)
    if not guide:
        assert np.array_equal(sampling_frontend(cond, cond, 3.0, 0, off, V)[:, :, off:off + V], cond[:, :, off:off + V])
    xx = dict(x, target_logits=filt)
    rep = compare_verify(parent, xx, neigh, V, off, k, cfg.lam, got)
    # survivors: drafted tokens the filter removed have q = 0 exactly, the others do not
    tok_logit = np.take_along_axis(filt[:, :, off:off + V][:, [int(p) if p >= 0 else 0 for p in parent]],
                                   x["tokens"][:, :, None].astype(np.int64), axis=2)[:, :, 0]
    first = np.zeros((B, M), dtype=bool)
    seen = set()
    for c in range(1, M):
        if int(parent[c]) not in seen:
            first[:, c] = True
            seen.add(int(parent[c]))
    removed = np.isneginf(tok_logit) & first
    assert np.array_equal(got["q_tok"][first] == 0, removed[first])
    # no final draw lands on a filtered token of its row
    fin = got["final_tok_all"]
    assert np.all(np.isfinite(np.take_along_axis(filt[:, :, off:off + V], fin[:, :, None].astype(np.int64), axis=2)))
    print(f"cfg{cfg.idx} scale={scale} top_k={top_k} guide={guide}: {rep}; removed first-children {int(removed.sum())}", flush=True)
    return rep, got


@pytest.mark.parametrize("idx,top_k", [(1, 100), (3, 2000), (3, 300), (4, 2000)])
def test_sampled_verify_parity(idx, top_k):
    cfg = CONFIGS[idx] if idx != 3 else CONFIGS[3].scaled(B=2)
    rep, got = _run(cfg, 3.0, top_k)
    assert rep["nodes"] > 0 and rep["near_tie_decisions"] <= 2 and rep["nagg_ties"] <= 2


def test_sampled_verify_switches():
    cfg = CONFIGS[3].scaled(B=1)
    _run(cfg, 3.0, 0)                    # guidance only
    _run(cfg, 0.0, 2000, guide=False)    # top-k only
    rep, got = _run(cfg, 1.5, cfg.V)     # top_k >= V: no filter
    assert rep["nodes"] > 0


def test_sampled_verify_argument_errors():
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    z = torch.zeros(4096, dtype=torch.float32, device=DEV)
    zi = torch.zeros(4096, dtype=torch.int32, device=DEV)
    out = {"accept_len": zi, "path": zi, "final_token": zi}
    for scale, tk in ((float("nan"), 10), (3.0, -1)):
        with pytest.raises(lpp.LppError) as e:
            lpp.lpp_relaxed_verify_sampled(tree, z, z, scale, tk, z, 1024, 0, 1024, 1, zi, zi, 16, 16, 2.0, z, z, out,
                                           torch.empty(4096, dtype=torch.uint8, device=DEV))
        assert e.value.status == lpp.LPP_EINVAL
