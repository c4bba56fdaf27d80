"""GPU: a captured HIP graph of one verification step (attention + relaxed verify) replays to the
same results as eager launches, on every replay, with eager work in between (the library's
"last block" counters must be back at zero after every call for that to hold)."""
import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from workloads import CONFIGS, static_tree, make_codebook, make_attention_inputs, make_verify_inputs
from gpu_common import DEV, bf16_dev, dev, sparse_neighbour_table

pytestmark = pytest.mark.gpu


def test_step_graph_replays_match_eager():
    cfg = CONFIGS[3].scaled(B=2, H=4, S=200)
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    B, H, M, S, Dh, V, k = cfg.B, cfg.H, cfg.M, cfg.S, cfg.Dh, cfg.V, cfg.k
    depth = max(tree.depth, 1)
    att = make_attention_inputs(cfg)
    sets = []
    for salt in (0, 1):
        x = make_verify_inputs(cfg, parent, rho=0.8, salt=salt)
        sets.append({n: dev(x[n]) for n in ("target_logits", "drafter_logits", "tokens", "u_accept", "u_final")})
    E = make_codebook(cfg)
    toks = np.concatenate([s["tokens"].cpu().numpy()[:, 1:].ravel() for s in sets])
    neigh = dev(sparse_neighbour_table(E, k, toks, V))
    t = {n: bf16_dev(att[n + "_bits"]) for n in ("q", "kc", "vc", "kt", "vt")}
    cur = {n: torch.empty_like(v) for n, v in sets[0].items()}      # the buffers the graph reads

    def outputs():
        return {"o": torch.full((B, H, M, Dh), float("nan"), device=DEV),
                "accept_len": torch.full((B,), -7, dtype=torch.int32, device=DEV),
                "path": torch.full((B, depth), -7, dtype=torch.int32, device=DEV),
                "final_token": torch.full((B,), -7, dtype=torch.int32, device=DEV),
                "decision": torch.full((B, M), 9, dtype=torch.uint8, device=DEV),
                "ratio": torch.zeros((B, M), device=DEV),
                "final_tok_all": torch.full((B, M), -7, dtype=torch.int32, device=DEV)}

    aws = torch.empty(max(lpp.lpp_tree_attention_workspace(tree, B, H, S, Dh), 256), dtype=torch.uint8, device=DEV)
    vws = torch.empty(lpp.lpp_relaxed_verify_workspace(tree, B, V, k), dtype=torch.uint8, device=DEV)

    def step(out, stream):
        lpp.lpp_tree_attention(tree, lpp.LPP_BF16, t["q"], t["kc"], t["vc"], t["kt"], t["vt"], None,
                               B, H, S, Dh, 0.0, out["o"], aws, stream)
        vo = {n: out[n] for n in out if n != "o"}
        lpp.lpp_relaxed_verify(tree, cur["target_logits"], cur["drafter_logits"], cfg.ldv, cfg.vocab_offset, V, B,
                               cur["tokens"], neigh, k, k, cfg.lam, cur["u_accept"], cur["u_final"], vo, vws, stream)

    def load(i):
        for n in cur:
            cur[n].copy_(sets[i][n])

    eager = []
    for i in (0, 1):
        load(i)
        out = outputs()
        step(out, torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager.append({n: v.clone() for n, v in out.items()})

    gout = outputs()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(gout, side)
    torch.cuda.synchronize()
    for rep, i in enumerate((0, 1, 1, 0, 1)):
        load(i)
        for v in gout.values():
            v.fill_(0)
        scratch = outputs()
        step(scratch, torch.cuda.current_stream())      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n in gout:
            assert torch.equal(gout[n], eager[i][n]), f"replay {rep}: {n} differs from the eager result"


def test_layers_and_static_verify_graph_replays_match_eager():
    """Three layers of attention in one launch (lpp_tree_attention_layers) and the verify entry
    point that brings no workspace (lpp_relaxed_verify_static), captured together."""
    cfg = CONFIGS[3].scaled(B=2, H=4, S=333)
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    B, H, M, S, Dh, V, k = cfg.B, cfg.H, cfg.M, cfg.S, cfg.Dh, cfg.V, cfg.k
    depth = max(tree.depth, 1)
    L = 3
    names = {"q": "q", "kc": "k_cache", "vc": "v_cache", "kt": "k_tree", "vt": "v_tree"}
    layer_sets = []
    for i in (0, 1):
        layer_sets.append([{names[n]: bf16_dev(make_attention_inputs(cfg, salt=100 * i + 7 * l)[n + "_bits"])
                            for n in names} for l in range(L)])
    sets = []
    for salt in (0, 1):
        x = make_verify_inputs(cfg, parent, rho=0.8, salt=salt)
        sets.append({n: dev(x[n]) for n in ("target_logits", "drafter_logits", "tokens", "u_accept", "u_final")})
    E = make_codebook(cfg)
    toks = np.concatenate([s["tokens"].cpu().numpy()[:, 1:].ravel() for s in sets])
    neigh = dev(sparse_neighbour_table(E, k, toks, V))
    cur = {n: torch.empty_like(v) for n, v in sets[0].items()}
    cur_layers = [{n: torch.empty_like(v) for n, v in y.items()} for y in layer_sets[0]]

    def outputs():
        out = {"accept_len": torch.full((B,), -7, dtype=torch.int32, device=DEV),
               "path": torch.full((B, depth), -7, dtype=torch.int32, device=DEV),
               "final_token": torch.full((B,), -7, dtype=torch.int32, device=DEV),
               "decision": torch.full((B, M), 9, dtype=torch.uint8, device=DEV),
               "final_tok_all": torch.full((B, M), -7, dtype=torch.int32, device=DEV)}
        for l in range(L):
            out[f"o{l}"] = torch.full((B, H, M, Dh), float("nan"), device=DEV)
        return out

    aws = torch.empty(max(lpp.lpp_tree_attention_layers_workspace(tree, L, B, H, S, Dh), 256), dtype=torch.uint8,
                      device=DEV)

    def step(out, stream):
        layers = [dict(cur_layers[l], out=out[f"o{l}"]) for l in range(L)]
        lpp.lpp_tree_attention_layers(tree, lpp.LPP_BF16, lpp.LPP_F32, layers, None, B, H, H, S, Dh, 0.0, aws, stream)
        vo = {n: v for n, v in out.items() if not n.startswith("o")}
        lpp.lpp_relaxed_verify_static(tree, cur["target_logits"], cur["drafter_logits"], cfg.ldv, cfg.vocab_offset, V,
                                      B, cur["tokens"], neigh, k, k, cfg.lam, cur["u_accept"], cur["u_final"], vo,
                                      stream)

    def load(i):
        for n in cur:
            cur[n].copy_(sets[i][n])
        for l in range(L):
            for n in cur_layers[l]:
                cur_layers[l][n].copy_(layer_sets[i][l][n])

    eager = []
    for i in (0, 1):        # also the static entry point's first call on this device, outside the capture
        load(i)
        out = outputs()
        step(out, torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager.append({n: v.clone() for n, v in out.items()})
    for l in range(L):
        assert not torch.equal(eager[0][f"o{l}"], eager[1][f"o{l}"])

    gout = outputs()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(gout, side)
    torch.cuda.synchronize()
    for rep, i in enumerate((1, 0, 0, 1)):
        load(i)
        for v in gout.values():
            v.fill_(0)
        scratch = outputs()
        step(scratch, torch.cuda.current_stream())
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n in gout:
            assert torch.equal(gout[n], eager[i][n]), f"replay {rep}: {n} differs from the eager result"
