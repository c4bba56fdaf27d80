"""Pins for oracle.tree_attention (no GPU): one masked pass over the flattened
tree must equal verifying every root-to-node path on its own (App. A.2)."""
import numpy as np
import pytest
import torch

from oracle import tree_attention, ancestor_mask
from workloads import static_tree


def _causal_last_row(qrow, K, V, scale):
    """Ordinary attention of one query over all given keys, written out with loops."""
    s = np.array([float(np.dot(qrow, K[j])) * scale for j in range(len(K))])
    w = np.exp(s - s.max())
    w /= w.sum()
    out = np.zeros(V.shape[1])
    for j in range(len(K)):
        out += w[j] * V[j]
    return out


def _inputs(B, H, M, S, Dh, seed):
    g = np.random.default_rng(seed)
    f = lambda *s: g.standard_normal(s)
    return f(B, H, M, Dh), f(B, H, S, Dh), f(B, H, S, Dh), f(B, H, M, Dh), f(B, H, M, Dh)


def test_ancestor_mask_small():
    parent = np.array([-1, 0, 0, 1, 1, 2])
    m = ancestor_mask(parent)
    want = np.array([[1, 0, 0, 0, 0, 0], [1, 1, 0, 0, 0, 0], [1, 0, 1, 0, 0, 0],
                     [1, 1, 0, 1, 0, 0], [1, 1, 0, 0, 1, 0], [1, 0, 1, 0, 0, 1]], dtype=bool)
    assert np.array_equal(m, want)


def test_path_unrolled_equivalence():
    parent = static_tree((4, 2, 1, 1), 15)
    B, H, M, S, Dh = 2, 2, 16, 37, 16
    q, kc, vc, kt, vt = _inputs(B, H, M, S, Dh, 0)
    out = tree_attention(q, kc, vc, kt, vt, parent)
    for b in range(B):
        for h in range(H):
            for i in range(M):
                path = []
                t = i
                while t >= 0:
                    path.append(t); t = parent[t]
                path = path[::-1]
                K = np.concatenate([kc[b, h], kt[b, h, path]])
                V = np.concatenate([vc[b, h], vt[b, h, path]])
                want = _causal_last_row(q[b, h, i], K, V, 1 / np.sqrt(Dh))
                assert np.allclose(out[b, h, i], want, rtol=1e-11, atol=1e-13)


def test_chain_tree_is_causal_attention_and_matches_library():
    M, S, Dh = 9, 20, 8
    parent = np.arange(-1, M - 1)
    q, kc, vc, kt, vt = _inputs(1, 3, M, S, Dh, 1)
    out = tree_attention(q, kc, vc, kt, vt, parent)
    K = torch.from_numpy(np.concatenate([kc, kt], axis=2)); V = torch.from_numpy(np.concatenate([vc, vt], axis=2))
    mask = torch.ones(M, S + M, dtype=torch.bool)
    mask[:, S:] = torch.tril(torch.ones(M, M, dtype=torch.bool))
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q), K, V, attn_mask=mask)
    assert np.allclose(out, ref.numpy(), rtol=1e-10, atol=1e-12)


def test_library_second_opinion_tree_mask_and_scale():
    parent = static_tree((3, 2, 2), 12)
    M, S, Dh = 13, 33, 32
    q, kc, vc, kt, vt = _inputs(2, 2, M, S, Dh, 2)
    out = tree_attention(q, kc, vc, kt, vt, parent, scale=0.3)
    mask = torch.ones(M, S + M, dtype=torch.bool)
    mask[:, S:] = torch.from_numpy(ancestor_mask(parent))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(np.concatenate([kc, kt], 2)),
        torch.from_numpy(np.concatenate([vc, vt], 2)), attn_mask=mask, scale=0.3)
    assert np.allclose(out, ref.numpy(), rtol=1e-10, atol=1e-12)


def test_constant_values_and_seq_len():
    parent = static_tree((2, 2), 6)
    M, S, Dh = 7, 16, 8
    q, kc, vc, kt, vt = _inputs(2, 1, M, S, Dh, 3)
    row = np.arange(Dh, dtype=np.float64)
    out = tree_attention(q, kc, np.broadcast_to(row, vc.shape), kt, np.broadcast_to(row, vt.shape), parent)
    assert np.allclose(out, row)                      # weights sum to one
    sl = np.array([5, 16])
    a = tree_attention(q, kc, vc, kt, vt, parent, seq_len=sl)
    b0 = tree_attention(q[:1], kc[:1, :, :5], vc[:1, :, :5], kt[:1], vt[:1], parent)
    b1 = tree_attention(q[1:], kc[1:], vc[1:], kt[1:], vt[1:], parent)
    assert np.allclose(a[0], b0[0], rtol=1e-12) and np.allclose(a[1], b1[0], rtol=1e-12)
    # a masked sibling's key must have no influence at all
    kt2 = kt.copy(); kt2[:, :, 2] += 100.0
    c = tree_attention(q, kc, vc, kt2, vt, parent)
    d = tree_attention(q, kc, vc, kt, vt, parent)
    vis = ancestor_mask(parent)
    for i in range(M):
        assert np.array_equal(c[:, :, i], d[:, :, i]) == (not vis[i, 2])


def test_grouped_query_heads_equal_repeated_key_value_heads_and_library():
    """Grouped-query attention: query head h reads key/value head h // (H // Hkv).  Repeating every
    key/value head H // Hkv times must give plain multi-head attention (checked against the pinned
    multi-head path and against the library routine on the repeated tensors); a head permutation
    that breaks the grouping must change the result."""
    rng = np.random.default_rng(11)
    parent = static_tree((3, 3, 2), 10)
    B, H, Hkv, M, Dh, S = 2, 6, 2, len(parent), 8, 7
    q = rng.standard_normal((B, H, M, Dh))
    kc, vc = rng.standard_normal((2, B, Hkv, S, Dh))
    kt, vt = rng.standard_normal((2, B, Hkv, M, Dh))
    seq_len = np.array([7, 4])
    out = tree_attention(q, kc, vc, kt, vt, parent, seq_len=seq_len)
    rep = lambda x: np.repeat(x, H // Hkv, axis=1)
    want = tree_attention(q, rep(kc), rep(vc), rep(kt), rep(vt), parent, seq_len=seq_len)
    assert np.array_equal(out, want)
    for b in range(B):
        Sb = int(seq_len[b])
        mask = np.concatenate([np.ones((M, Sb), dtype=bool), ancestor_mask(parent)], axis=1)
        K = np.concatenate([rep(kc)[b:b + 1, :, :Sb], rep(kt)[b:b + 1]], axis=2)
        Vv = np.concatenate([rep(vc)[b:b + 1, :, :Sb], rep(vt)[b:b + 1]], axis=2)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q[b:b + 1]), torch.from_numpy(K), torch.from_numpy(Vv),
            attn_mask=torch.from_numpy(mask))
        assert np.abs(out[b:b + 1] - ref.numpy()).max() < 1e-12
    # interleaved assignment (h % Hkv) is a different function
    til = lambda x: np.tile(x, (1, H // Hkv, 1, 1))
    other = tree_attention(q, til(kc), til(vc), til(kt), til(vt), parent, seq_len=seq_len)
    assert np.abs(other - out).max() > 1e-3
