"""GPU parity: lpp_tree_attention against the float64 oracle (through the C ABI).

Tolerance (relative to |want| + the row's max |want|): 1e-4 for fp32 inputs,
2e-2 for bf16 inputs (fp32 softmax/accumulation, bf16 probabilities on the
matrix cores)."""
import numpy as np
import pytest

import paper_2502_06352_amd as lpp
from oracle import tree_attention
from workloads import CONFIGS, static_tree, make_attention_inputs
from gpu_common import run_attention, attention_error

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _check(cfg, parent, att, got, seq_len=None, pairs=None):
    B, H = att["q"].shape[:2]
    assert np.all(np.isfinite(got))
    if pairs is None:
        want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent, seq_len=seq_len)
        err = attention_error(got, want)
    else:
        err = 0.0
        for b, h in pairs:
            sl = None if seq_len is None else seq_len[b:b + 1]
            want = tree_attention(att["q"][b:b + 1, h:h + 1], att["kc"][b:b + 1, h:h + 1], att["vc"][b:b + 1, h:h + 1],
                                  att["kt"][b:b + 1, h:h + 1], att["vt"][b:b + 1, h:h + 1], parent, seq_len=sl)
            err = max(err, attention_error(got[b:b + 1, h:h + 1], want))
    print(f"cfg{cfg.idx} B={B} H={H} M={cfg.M} S={att['kc'].shape[2]} Dh={cfg.Dh} {cfg.kv_dtype}: err={err:.3e}", flush=True)
    assert err <= TOL[cfg.kv_dtype]
    return err


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_attention_parity_configs(idx):
    cfg = CONFIGS[idx]
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    got = run_attention(lpp.Tree(parent), att, cfg)
    _check(cfg, parent, att, got)


def test_attention_parity_stress_full_size():
    # config 5 at its full size: every head of three batch items (the first, one in the middle, the
    # last) and one head of every other item
    cfg = CONFIGS[5]
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    got = run_attention(lpp.Tree(parent), att, cfg)
    pairs = [(b, h) for b in (0, 7, cfg.B - 1) for h in range(cfg.H)]
    pairs += [(b, (5 * b + 3) % cfg.H) for b in range(cfg.B) if b not in (0, 7, cfg.B - 1)]
    _check(cfg, parent, att, got, pairs=pairs)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_attention_ragged_lengths_and_odd_shapes(dtype):
    # S not a multiple of 32, per-item lengths (one empty), odd row counts
    for (N, branching, S, H, Dh, lens) in [
        (5, (2, 2, 1), 77, 3, 64, [77, 0, 31, 33]),
        (40, (5, 3, 2, 1), 130, 2, 128, [130, 1, 64, 97]),
        (128, (8, 4, 2, 2, 1, 1, 1, 1), 45, 2, 64, [45, 7, 0, 32]),
        (16, (16,), 100, 1, 128, [100, 99, 3, 50]),
    ]:
        cfg = CONFIGS[2].scaled(N=N, branching=branching, S=S, H=H, Dh=Dh, B=4, kv_dtype=dtype)
        parent = static_tree(cfg.branching, cfg.N)
        att = make_attention_inputs(cfg)
        sl = np.array(lens, dtype=np.int32)
        got = run_attention(lpp.Tree(parent), att, cfg, seq_len=sl)
        _check(cfg, parent, att, got, seq_len=sl)


def test_attention_no_cache_and_single_row():
    cfg = CONFIGS[2].scaled(N=0, branching=(1,), S=64, H=2, B=2)
    parent = np.array([-1], dtype=np.int32)
    att = make_attention_inputs(cfg)
    got = run_attention(lpp.Tree(parent), att, cfg)
    _check(cfg, parent, att, got)
    # S = 0: only the tree keys; a root row then returns its own V row exactly (bf16 value)
    cfg = CONFIGS[2].scaled(N=9, branching=(3, 2), S=0, H=2, B=1)
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    got = run_attention(lpp.Tree(parent), att, cfg, S=0)
    _check(cfg, parent, att, got)
    assert np.array_equal(got[:, :, 0], att["vt"][:, :, 0])


def test_attention_masked_sibling_has_no_influence():
    cfg = CONFIGS[2].scaled(S=96, H=2)
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    tree = lpp.Tree(parent)
    a = run_attention(tree, att, cfg)
    att2 = dict(att)
    from workloads import bf16_bits
    kt = att["kt"].copy(); kt[:, :, 2] *= 50.0
    att2["kt"], att2["kt_bits"] = kt, bf16_bits(kt)
    b = run_attention(tree, att2, cfg)
    from oracle import ancestor_mask
    vis = ancestor_mask(parent)
    for i in range(cfg.M):
        assert np.array_equal(a[:, :, i], b[:, :, i]) == (not vis[i, 2])


def test_attention_deterministic_run_to_run():
    cfg = CONFIGS[3]
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    tree = lpp.Tree(parent)
    assert np.array_equal(run_attention(tree, att, cfg), run_attention(tree, att, cfg))


def test_attention_argument_errors():
    cfg = CONFIGS[1].scaled(Dh=32)
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    with pytest.raises(lpp.LppError) as e:
        run_attention(lpp.Tree(parent), att, cfg)
    assert e.value.status == lpp.LPP_EUNSUPPORTED
