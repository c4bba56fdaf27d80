"""Pins for oracle.commit_kv (no GPU): what the commit must mean for the next step.

App. A.2: the tree mask lets a node see the prefix, its ancestors and itself; accepted tokens are
kept.  So after committing the root and the accepted path, plain (unmasked) attention of the last
accepted node's query over the first new_len cache positions must equal the tree-masked attention
output that node had inside the tree -- computed here directly, not through the oracle's own
attention.  Plus the bookkeeping: untouched positions, capacity, empty path."""
import numpy as np

from oracle import commit_kv, tree_attention
from workloads import CONFIGS, static_tree, make_attention_inputs, children_lists


def _plain_attention(q, K, V):
    s = (K @ q) / np.sqrt(len(q))
    w = np.exp(s - s.max())
    return (w / w.sum()) @ V


def _some_path(parent, rng, length):
    kids = children_lists(parent)
    cur, path = 0, []
    while len(path) < length and kids[cur]:
        cur = int(rng.choice(kids[cur]))
        path.append(cur)
    return path


def test_committed_cache_reproduces_tree_attention_rows():
    cfg = CONFIGS[2].scaled(B=3, H=2, S=96, kv_dtype="f32")
    parent = static_tree(cfg.branching, cfg.N)
    depth = len(cfg.branching)
    att = make_attention_inputs(cfg)
    rng = np.random.default_rng(3)
    seq_len = np.array([40, 0, 77], dtype=np.int32)
    paths = [_some_path(parent, rng, n) for n in (3, 0, depth)]
    path = np.full((cfg.B, depth), -1, dtype=np.int32)
    for b, pth in enumerate(paths):
        path[b, :len(pth)] = pth
    accept_len = np.array([len(p) for p in paths], dtype=np.int32)
    kc, vc, new_len = commit_kv(att["kc"], att["vc"], att["kt"], att["vt"], path, accept_len, seq_len)
    assert new_len.tolist() == [40 + 1 + 3, 1, 77 + 1 + len(paths[2])]
    want = tree_attention(att["q"], att["kc"], att["vc"], att["kt"], att["vt"], parent, seq_len=seq_len)
    for b in range(cfg.B):
        last = paths[b][-1] if paths[b] else 0
        n = int(new_len[b])
        for h in range(cfg.H):
            got = _plain_attention(att["q"][b, h, last].astype(np.float64), kc[b, h, :n].astype(np.float64),
                                   vc[b, h, :n].astype(np.float64))
            assert np.allclose(got, want[b, h, last], rtol=1e-10, atol=1e-12)
        # nothing else moved
        assert np.array_equal(kc[b, :, :seq_len[b]], att["kc"][b, :, :seq_len[b]])
        assert np.array_equal(kc[b, :, n:], att["kc"][b, :, n:])
        assert np.array_equal(vc[b, :, n:], att["vc"][b, :, n:])


def test_commit_respects_capacity():
    cfg = CONFIGS[2].scaled(B=1, H=1, S=8, kv_dtype="f32")
    parent = static_tree(cfg.branching, cfg.N)
    att = make_attention_inputs(cfg)
    path = np.array([[1, 5, -1, -1, -1]], dtype=np.int32)
    kc, vc, new_len = commit_kv(att["kc"], att["vc"], att["kt"], att["vt"], path, np.array([2]), np.array([6]))
    assert new_len.tolist() == [8]                       # root and one node fit; the second is dropped
    assert np.array_equal(kc[0, :, 6], att["kt"][0, :, 0]) and np.array_equal(kc[0, :, 7], att["kt"][0, :, 1])
    assert np.array_equal(vc[0, :, 7], att["vt"][0, :, 1])
