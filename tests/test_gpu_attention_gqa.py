"""GPU parity: lpp_tree_attention_gqa (shared key/value heads, float32 or bf16 output) against the
float64 oracle, through the C ABI.  Same tolerance as the multi-head call; a bf16 output adds its
own rounding (2^-9 relative), which the bf16 bound covers and the fp32 bound is widened for."""
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


def _inputs(cfg, Hkv, salt=0):
    """q from a config with H heads; keys and values from the same recipe with Hkv heads."""
    att = make_attention_inputs(cfg, salt=salt)
    kv = make_attention_inputs(dataclasses.replace(cfg, H=Hkv), salt=salt + 1)
    for n in ("kc", "vc", "kt", "vt"):
        att[n] = kv[n]
        if n + "_bits" in kv:
            att[n + "_bits"] = kv[n + "_bits"]
    return att


def _run(tree, att, cfg, Hkv, out_dtype, seq_len=None):
    B, H, M, Dh = att["q"].shape
    S = att["kc"].shape[2]
    if cfg.kv_dtype == "bf16":
        t = {n: bf16_dev(att[n + "_bits"]) for n in ("q", "kc", "vc", "kt", "vt")}
        dtype = lpp.LPP_BF16
    else:
        t = {n: dev(att[n]) for n in ("q", "kc", "vc", "kt", "vt")}
        dtype = lpp.LPP_F32
    sl = None if seq_len is None else dev(np.asarray(seq_len, dtype=np.int32))
    tdt = torch.bfloat16 if out_dtype == lpp.LPP_BF16 else torch.float32
    out = torch.full((B, H, M, Dh), float("nan"), dtype=tdt, device=DEV)
    ws = torch.empty(max(lpp.lpp_tree_attention_workspace(tree, B, H, S, Dh), 256), dtype=torch.uint8, device=DEV)
    lpp.lpp_tree_attention_gqa(tree, dtype, out_dtype, t["q"], t["kc"] if S > 0 else None,
                               t["vc"] if S > 0 else None, t["kt"], t["vt"], sl, B, H, Hkv, S, Dh, 0.0, out, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy()


@pytest.mark.parametrize("idx,Hkv", [(1, 2), (2, 4), (3, 8), (3, 1), (4, 8)])
@pytest.mark.parametrize("out_bf16", [False, True])
def test_gqa_parity_configs(idx, Hkv, out_bf16):
    cfg = CONFIGS[idx]
    parent = static_tree(cfg.branching, cfg.N)
    att = _inputs(cfg, Hkv)
    got = _run(lpp.Tree(parent), att, cfg, Hkv, lpp.LPP_BF16 if out_bf16 else lpp.LPP_F32)
    want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent)
    err = attention_error(got, want)
    tol = TOL[cfg.kv_dtype] if not out_bf16 else max(TOL[cfg.kv_dtype], 4e-3)
    print(f"cfg{idx} H={cfg.H} Hkv={Hkv} out_bf16={out_bf16}: err={err:.3e}", flush=True)
    assert np.all(np.isfinite(got)) and err <= tol


def test_gqa_equals_multi_head_call_on_repeated_heads_and_bf16_is_the_rounded_float():
    cfg = dataclasses.replace(CONFIGS[2], H=12)
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    Hkv = 3
    att = _inputs(cfg, Hkv, salt=5)
    seq_len = [cfg.S - 37]
    a = _run(tree, att, cfg, Hkv, lpp.LPP_F32, seq_len=seq_len)
    rep = {n: np.repeat(att[n], cfg.H // Hkv, axis=1) for n in ("kc", "vc", "kt", "vt")}
    rep.update({n + "_bits": np.repeat(att[n + "_bits"], cfg.H // Hkv, axis=1) for n in ("kc", "vc", "kt", "vt")})
    rep["q"], rep["q_bits"] = att["q"], att["q_bits"]
    b = _run(tree, rep, cfg, cfg.H, lpp.LPP_F32, seq_len=seq_len)
    assert np.array_equal(a, b)                       # same arithmetic, same order
    h = _run(tree, att, cfg, Hkv, lpp.LPP_BF16, seq_len=seq_len)
    assert np.array_equal(h, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_gqa_large_tree_many_row_tiles_sampled_heads():
    cfg = dataclasses.replace(CONFIGS[5], B=2, H=16, S=777)
    parent = static_tree(cfg.branching, cfg.N)
    Hkv = 4
    att = _inputs(cfg, Hkv, salt=9)
    seq_len = np.array([777, 300])
    got = _run(lpp.Tree(parent), att, cfg, Hkv, lpp.LPP_F32, seq_len=seq_len)
    want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent, seq_len=seq_len)
    err = attention_error(got, want)
    print(f"large tree GQA err={err:.3e}", flush=True)
    assert err <= TOL["bf16"]


def test_gqa_argument_errors():
    cfg = CONFIGS[2]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    att = _inputs(cfg, 4)
    for Hkv, out_dtype, code in [(0, lpp.LPP_F32, lpp.LPP_EINVAL), (5, lpp.LPP_F32, lpp.LPP_EINVAL),
                                 (32, lpp.LPP_F32, lpp.LPP_EINVAL), (4, 7, lpp.LPP_EUNSUPPORTED)]:
        with pytest.raises(lpp.LppError) as e:
            _run(tree, att, cfg, Hkv, out_dtype)
        assert e.value.status == code
