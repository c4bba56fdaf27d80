"""GPU parity: lpp_tree_attention_layers (several layers of one step in one launch; Sec. 2.1,
App. A.2) against the float64 oracle, layer by layer, through the C ABI.  Every layer has its own
queries, keys and values (seeded apart), so a block that reads another layer's tensors, partials
or counters shows up as an error."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from oracle import tree_attention
from workloads import CONFIGS, static_tree, make_attention_inputs
from gpu_common import DEV, dev, bf16_dev, attention_error

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _layer_inputs(cfg, Hkv, layer):
    att = make_attention_inputs(cfg, salt=10 * layer)
    if Hkv != cfg.H:
        kv = make_attention_inputs(dataclasses.replace(cfg, H=Hkv), salt=10 * layer + 1)
        for n in ("kc", "vc", "kt", "vt"):
            att[n] = kv[n]
            if n + "_bits" in kv:
                att[n + "_bits"] = kv[n + "_bits"]
    return att


def _run_layers(tree, atts, cfg, Hkv, out_dtype=lpp.LPP_F32, seq_len=None):
    B, H, M, Dh = atts[0]["q"].shape
    S = atts[0]["kc"].shape[2]
    bf = cfg.kv_dtype == "bf16"
    names = {"q": "q", "kc": "k_cache", "vc": "v_cache", "kt": "k_tree", "vt": "v_tree"}
    layers, outs = [], []
    for att in atts:
        y = {names[n]: (bf16_dev(att[n + "_bits"]) if bf else dev(att[n])) for n in names}
        y["out"] = torch.full((B, H, M, Dh), float("nan"),
                              dtype=torch.bfloat16 if out_dtype == lpp.LPP_BF16 else torch.float32, device=DEV)
        layers.append(y)
        outs.append(y["out"])
    sl = None if seq_len is None else dev(np.asarray(seq_len, dtype=np.int32))
    L = len(layers)
    ws = torch.empty(max(lpp.lpp_tree_attention_layers_workspace(tree, L, B, H, S, Dh), 256), dtype=torch.uint8, device=DEV)
    lpp.lpp_tree_attention_layers(tree, lpp.LPP_BF16 if bf else lpp.LPP_F32, out_dtype, layers, sl, B, H, Hkv, S, Dh, 0.0, ws)
    torch.cuda.synchronize()
    return [o.float().cpu().numpy() for o in outs]


@pytest.mark.parametrize("idx,L,Hkv", [(1, 3, 4), (2, 3, 16), (3, 3, 24), (4, 3, 32), (2, 19, 16), (3, 2, 8),
                                       (4, 5, 8)])
def test_layers_parity(idx, L, Hkv):
    # cfg 2 and 4 at L = 3 split the keys of a head over several blocks (partials and counters per
    # layer); L = 19 takes two launches; cfg 3 with 8 key/value heads shares them among query heads.
    # Launches with more blocks than compute units run blocks of 4 waves: cfg 3 at L = 2 and 3
    # (head size 64), cfg 4 at L = 5 (head size 128, 8 key/value heads).
    cfg = CONFIGS[idx]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    atts = [_layer_inputs(cfg, Hkv, l) for l in range(L)]
    got = _run_layers(tree, atts, cfg, Hkv)
    worst = 0.0
    for l in range(L):
        want = tree_attention(atts[l]["q"], atts[l]["kc"], atts[l]["vc"], atts[l]["kt"], atts[l]["vt"], parent)
        err = attention_error(got[l], want)
        worst = max(worst, err)
        assert np.all(np.isfinite(got[l])) and err <= TOL[cfg.kv_dtype], f"layer {l}: err {err}"
    print(f"cfg{idx} L={L} Hkv={Hkv}: worst err {worst:.3e}", flush=True)


def test_layers_equal_the_single_layer_call_and_repeat():
    # the same layers through lpp_tree_attention one by one: identical bits; twice on one handle
    cfg = CONFIGS[2]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    atts = [_layer_inputs(cfg, cfg.H, l) for l in range(4)]
    a = _run_layers(tree, atts, cfg, cfg.H)
    b = _run_layers(tree, atts, cfg, cfg.H)
    from gpu_common import run_attention
    for l in range(4):
        one = run_attention(tree, atts[l], cfg)
        assert np.array_equal(a[l], b[l])
        err = attention_error(a[l], one)
        assert err <= 1e-5, f"layer {l} differs from the single-layer call by {err}"   # (other key splits: other rounding)


def test_layers_ragged_lengths_bf16_out_and_errors():
    cfg = CONFIGS[3].scaled(B=3)
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    atts = [_layer_inputs(cfg, 8, l) for l in range(2)]
    seq = [0, 517, cfg.S]
    got = _run_layers(tree, atts, cfg, 8, out_dtype=lpp.LPP_BF16, seq_len=seq)
    for l in range(2):
        for b, n in enumerate(seq):
            want = tree_attention(atts[l]["q"][b:b + 1], atts[l]["kc"][b:b + 1, :, :n], atts[l]["vc"][b:b + 1, :, :n],
                                  atts[l]["kt"][b:b + 1], atts[l]["vt"][b:b + 1], parent)
            assert attention_error(got[l][b:b + 1], want) <= 2e-2
    one = torch.zeros(16, device=DEV)
    with pytest.raises(lpp.LppError) as e:
        lpp.lpp_tree_attention_layers(tree, lpp.LPP_BF16, lpp.LPP_F32, [], None, 1, 4, 4, 64, 64, 0.0, one)
    assert e.value.status == lpp.LPP_EINVAL
    with pytest.raises(lpp.LppError) as e:
        lpp.lpp_tree_attention_layers(tree, lpp.LPP_BF16, lpp.LPP_F32, [dict(q=one, k_cache=one, v_cache=one, k_tree=one,
                                                                             v_tree=None, out=one)],
                                      None, 1, 4, 4, 64, 64, 0.0, one)
    assert e.value.status == lpp.LPP_EINVAL
