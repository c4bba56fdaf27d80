"""Pins for oracle.build_neighbours (no GPU): the definition of B_k (Sec. 2.2)."""
from fractions import Fraction
import itertools

import numpy as np

from oracle import build_neighbours, similarity_keys
from workloads import CONFIGS, make_codebook


def test_hand_example_2d():
    # unit vectors at 0, 10, 100, 180, 205 degrees -> angular order fixes the neighbours
    ang = np.deg2rad([0, 10, 100, 180, 205])
    E = np.stack([np.cos(ang), np.sin(ang)], 1).astype(np.float32)
    nb = build_neighbours(E, 5)
    assert nb.tolist() == [[0, 1, 2, 4, 3], [1, 0, 2, 4, 3], [2, 3, 1, 0, 4], [3, 4, 2, 1, 0], [4, 3, 2, 0, 1]]
    assert build_neighbours(E, 2).tolist() == [[0, 1], [1, 0], [2, 3], [3, 4], [4, 3]]
    assert build_neighbours(E, 3, rows=[3, 0]).tolist() == [[3, 4, 2], [0, 1, 2]]


def test_invariants_on_tiny_config():
    cfg = CONFIGS[1]
    E = make_codebook(cfg)
    nb = build_neighbours(E, cfg.k)
    assert nb.shape == (1024, 16) and np.array_equal(nb[:, 0], np.arange(1024))
    key = similarity_keys(E, np.arange(1024))
    assert np.array_equal(key, key.T)                                  # same bits both ways
    ks = np.take_along_axis(key, nb.astype(np.int64), 1)
    assert np.all(ks[:, 1:-1] >= ks[:, 2:])                            # nearest first
    # nothing outside the list beats the last listed neighbour
    for i in range(0, 1024, 37):
        rest = np.setdiff1d(np.arange(1024), nb[i])
        assert key[i, rest].max() <= ks[i, -1]
    full = build_neighbours(E, 1024, rows=[0, 511])
    assert np.array_equal(np.sort(full, 1), np.tile(np.arange(1024), (2, 1)))
    assert np.array_equal(full[:, :16], nb[[0, 511]])                 # prefix property in k


def test_key_is_the_sequential_float64_sum():
    g = np.random.default_rng(0)
    E = g.standard_normal((7, 12)).astype(np.float32)
    key = similarity_keys(E, np.arange(7))
    for i, j in itertools.product(range(7), repeat=2):
        exact = sum(Fraction(float(E[i, t])) * Fraction(float(E[j, t])) for t in range(12))
        assert abs(Fraction(float(key[i, j])) - exact) <= Fraction(12, 2 ** 52) * max(1, abs(exact))
        acc = 0.0
        for t in range(12):
            acc = acc + float(E[i, t]) * float(E[j, t])
        assert acc == key[i, j]


def test_cosine_order_equals_euclidean_order_on_unit_rows_with_ties():
    # exactly-unit rows (+-1/2 in 4-D, +-e_i): many exact ties -> lower index first
    rows = [np.array(s) * 0.5 for s in itertools.product([-1, 1], repeat=4)]
    rows += [s * np.eye(4)[i] for i in range(4) for s in (1, -1)]
    E = np.array(rows, dtype=np.float32)
    V = len(E)
    nb = build_neighbours(E, V)
    E64 = E.astype(np.float64)
    for i in range(V):
        d2 = ((E64[i] - E64) ** 2).sum(1)
        order = sorted((j for j in range(V) if j != i), key=lambda j: (d2[j], j))
        assert nb[i].tolist() == [i] + order


def test_duplicate_code_keeps_self_first():
    E = np.array([[1, 0], [0, 1], [1, 0], [0.6, 0.8]], dtype=np.float32)
    nb = build_neighbours(E, 3)
    assert nb[2].tolist() == [2, 0, 3] and nb[0].tolist() == [0, 2, 3]
