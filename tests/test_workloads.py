"""Input generators: tree topologies and seeded tensors (no GPU)."""
import numpy as np
import pytest

from workloads import CONFIGS, static_tree, tree_depths, children_lists
from workloads import make_codebook, make_verify_inputs, make_attention_inputs, bf16_round, bf16_bits

# drafted nodes per depth for the five shapes
PER_DEPTH = {1: [3, 4, 4, 4], 2: [4, 6, 7, 5, 4], 3: [5, 9, 11, 12, 12, 11],
             4: [5, 9, 11, 12, 12, 11], 5: [7, 15, 16, 18, 18, 18, 18, 18]}
PARENTS = {1: 12, 2: 20, 3: 49, 4: 49, 5: 107}
MAXKIDS = {1: 3, 2: 4, 3: 5, 4: 5, 5: 7}


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_tree_shape(idx):
    cfg = CONFIGS[idx]
    parent = static_tree(cfg.branching, cfg.N)
    assert len(parent) == cfg.M and parent[0] == -1
    assert all(0 <= parent[i] < i for i in range(1, cfg.M))
    d = tree_depths(parent)
    assert [int((d == j).sum()) for j in range(1, cfg.depth + 1)] == PER_DEPTH[idx]
    kids = children_lists(parent)
    assert sum(1 for c in kids if c) == PARENTS[idx]
    assert max(len(c) for c in kids) == MAXKIDS[idx]
    # BFS order, children of a row consecutive, left-heavy
    assert all(d[i] <= d[i + 1] for i in range(cfg.M - 1))
    for c in kids:
        assert c == list(range(c[0], c[0] + len(c))) if c else True
    for lvl in range(1, cfg.depth):
        rows = [i for i in range(cfg.M) if d[i] == lvl]
        n = [len(kids[i]) for i in rows]
        assert n[0] == max(n)


def test_tree_worked_example():
    parent = static_tree((4, 2, 1, 1), 15)
    assert parent.tolist() == [-1, 0, 0, 0, 1, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11]


def test_bf16_round():
    x = np.array([1.0, 1.00390625, 1.005859375, -3.14159, 0.0, 65504.0], dtype=np.float32)
    r = bf16_round(x)
    assert r[0] == 1.0 and r[1] == 1.0          # tie rounds to even mantissa
    assert r[2] == np.float32(1.0078125)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert bf16_bits(np.array([1.0], np.float32))[0] == 0x3F80


def test_inputs_seeded_and_shaped():
    cfg = CONFIGS[1]
    parent = static_tree(cfg.branching, cfg.N)
    a = make_verify_inputs(cfg, parent, rho=0.8)
    b = make_verify_inputs(cfg, parent, rho=0.8)
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert a["target_logits"].shape == (1, 16, 1024) and a["tokens"].shape == (1, 16)
    assert a["tokens"].min() >= 0 and a["tokens"].max() < cfg.V
    assert 0 <= a["u_accept"].min() and a["u_accept"].max() < 1
    E = make_codebook(cfg)
    assert E.shape == (1024, 8) and np.allclose((E.astype(np.float64) ** 2).sum(1), 1, atol=1e-6)
    att = make_attention_inputs(cfg)
    assert att["kc"].shape == (1, 4, 256, 64) and att["q"].dtype == np.float32
    assert abs(float(a["target_logits"].std()) - 1.5) < 0.02


def test_lumina_like_row_layout():
    cfg = CONFIGS[4].scaled(N=5, branching=(2, 2, 1))
    parent = static_tree(cfg.branching, cfg.N)
    x = make_verify_inputs(cfg, parent)
    t = x["target_logits"]
    assert t.shape == (1, 6, 65536)
    assert np.all(np.isneginf(t[..., :4])) and np.all(np.isneginf(t[..., 4 + 8192:]))
    assert np.all(np.isfinite(t[..., 4:4 + 8192]))
