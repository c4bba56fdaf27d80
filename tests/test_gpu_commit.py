"""GPU parity: lpp_commit_kv against the oracle (bit-exact: pure data movement), through the C ABI,
fed by the path / accept_len that lpp_relaxed_verify wrote on the device."""
import numpy as np
import pytest
import torch

import paper_2502_06352_amd as lpp
from oracle import commit_kv
from workloads import CONFIGS, static_tree, make_codebook, make_attention_inputs, make_verify_inputs
from gpu_common import DEV, bf16_dev, dev, run_verify, sparse_neighbour_table

pytestmark = pytest.mark.gpu


def _device_kv(att, cfg):
    if cfg.kv_dtype == "bf16":
        return {n: bf16_dev(att[n + "_bits"]) for n in ("kc", "vc", "kt", "vt")}, lpp.LPP_BF16
    return {n: dev(att[n]) for n in ("kc", "vc", "kt", "vt")}, lpp.LPP_F32


def _host(t, cfg):
    if cfg.kv_dtype == "bf16":
        return (t.view(torch.int16).cpu().numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    return t.cpu().numpy()


@pytest.mark.parametrize("idx,kv", [(3, "bf16"), (4, "bf16"), (1, "f32")])
def test_commit_after_verify_matches_oracle(idx, kv):
    cfg = CONFIGS[idx].scaled(kv_dtype=kv, S=min(CONFIGS[idx].S, 512))
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    B, H, M, S, Dh = cfg.B, cfg.H, cfg.M, cfg.S, cfg.Dh
    att = make_attention_inputs(cfg)
    x = make_verify_inputs(cfg, parent, rho=0.9)
    neigh = sparse_neighbour_table(make_codebook(cfg), cfg.k, x["tokens"][:, 1:], cfg.V)
    got = run_verify(tree, x, neigh, cfg.V, cfg.vocab_offset, cfg.ldv, cfg.k, cfg.lam)
    assert got["accept_len"].max() >= 1
    # lengths: room for everything, no room at all, room for part of the path, empty cache
    seq_len = np.array([S - 10, S, S - 2, 0][:B] + [S // 2] * max(0, B - 4), dtype=np.int32)[:B]
    t, dtype = _device_kv(att, cfg)
    d_path, d_acc, d_seq = dev(got["path"]), dev(got["accept_len"]), dev(seq_len)
    new_len = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lpp.lpp_commit_kv(tree, dtype, t["kt"], t["vt"], d_path, d_acc, d_seq, B, H, S, Dh, t["kc"], t["vc"], new_len)
    torch.cuda.synchronize()
    kc, vc, nl = commit_kv(att["kc"], att["vc"], att["kt"], att["vt"], got["path"], got["accept_len"], seq_len)
    assert np.array_equal(new_len.cpu().numpy(), nl)
    assert np.array_equal(_host(t["kc"], cfg), kc)
    assert np.array_equal(_host(t["vc"], cfg), vc)


def test_commit_after_a_walk_that_gave_up_commits_the_root_only():
    # accept_len = -1 and path = -1 are what lpp_relaxed_verify writes for an item whose walk gave
    # up: the commit must treat it as "nothing accepted" (root only), like the oracle on a length of 0.
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    B, H, M, S, Dh = cfg.B, cfg.H, cfg.M, cfg.S, cfg.Dh
    att = make_attention_inputs(cfg)
    depth = max(tree.depth, 1)
    path = np.full((B, depth), -1, dtype=np.int32)
    acc = np.full((B,), -1, dtype=np.int32)
    seq_len = np.full((B,), S - 5, dtype=np.int32)
    t, dtype = _device_kv(att, cfg)
    new_len = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lpp.lpp_commit_kv(tree, dtype, t["kt"], t["vt"], dev(path), dev(acc), dev(seq_len), B, H, S, Dh, t["kc"], t["vc"],
                      new_len)
    torch.cuda.synchronize()
    kc, vc, nl = commit_kv(att["kc"], att["vc"], att["kt"], att["vt"], np.zeros_like(path), np.zeros_like(acc), seq_len)
    assert np.array_equal(new_len.cpu().numpy(), nl) and np.all(nl == S - 4)
    assert np.array_equal(_host(t["kc"], cfg), kc)
    assert np.array_equal(_host(t["vc"], cfg), vc)


def test_commit_argument_errors():
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    tree = lpp.Tree(parent)
    z = torch.zeros(64, dtype=torch.int32, device=DEV)
    kv = torch.zeros((1, 1, 16, 64), dtype=torch.float32, device=DEV)
    with pytest.raises(lpp.LppError) as e:
        lpp.lpp_commit_kv(tree, lpp.LPP_F32, kv, kv, z, z, z, 1, 1, 16, 64, kv, kv, z)       # new_len aliases seq_len
    assert e.value.status == lpp.LPP_EINVAL
    with pytest.raises(lpp.LppError) as e:
        lpp.lpp_commit_kv(tree, 5, kv, kv, z, z, z, 1, 1, 16, 64, kv, kv, None)
    assert e.value.status == lpp.LPP_EUNSUPPORTED
    with pytest.raises(lpp.LppError) as e:
        lpp.lpp_commit_kv(tree, lpp.LPP_F32, kv, kv, z, z, None, 1, 1, 16, 64, kv, kv, None)
    assert e.value.status == lpp.LPP_EINVAL
