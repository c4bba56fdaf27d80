"""Pins for oracle.sampling_frontend (no GPU): special cases that fix the guidance formula's
orientation and the top-k rule, a library second opinion, brute force on tiny rows."""
import numpy as np
import torch

from oracle import guided_logits, top_k_filter, sampling_frontend, softmax64


def test_guidance_special_cases_and_orientation():
    g = np.random.default_rng(0)
    c = g.normal(0, 2, 64).astype(np.float32); u = g.normal(0, 2, 64).astype(np.float32)
    assert np.array_equal(guided_logits(c, u, 0.0), u)            # scale 0: the null-conditioned row
    assert np.array_equal(guided_logits(c, c, 3.0), c)            # nothing to guide towards
    l1 = guided_logits(c, u, 1.0)
    assert np.allclose(l1, c, rtol=0, atol=4e-7 * np.abs(c).max())   # scale 1: the conditioned row (up to rounding)
    l3 = guided_logits(c, u, 3.0)
    # guidance pushes away from the null-conditioned row, 3x the gap (float64 check of a float32 result)
    want = u.astype(np.float64) + 3.0 * (c.astype(np.float64) - u.astype(np.float64))
    assert np.allclose(l3, want, rtol=0, atol=1e-5)
    assert np.all(np.sign(l3 - u) == np.sign(c - u))
    c2 = c.copy(); c2[5] = -np.inf
    assert np.isneginf(guided_logits(c2, u, 3.0)[5]) and not np.any(np.isnan(guided_logits(c2, u, 3.0)))


def test_top_k_rule_against_library_and_brute_force():
    g = np.random.default_rng(1)
    for n, k in [(16, 1), (16, 5), (16, 16), (16, 40), (2048, 2000), (4096, 100), (33, 0)]:
        row = g.normal(0, 2, n).astype(np.float32)
        out = top_k_filter(row, k)
        if k <= 0 or k >= n:
            assert np.array_equal(out, row)
            continue
        kept = np.flatnonzero(np.isfinite(out))
        assert len(kept) == k                                      # no ties in continuous data
        assert set(kept) == set(torch.topk(torch.from_numpy(row), k).indices.tolist())
        assert np.array_equal(out[kept], row[kept])
        assert out[kept].min() > np.max(np.delete(row, kept), initial=-np.inf)
    # brute force on a tiny row with ties at the threshold: the ties are kept
    row = np.array([1.0, 3.0, 2.0, 2.0, 0.5, 2.0], dtype=np.float32)
    assert np.isfinite(top_k_filter(row, 2)).tolist() == [False, True, True, True, False, True]
    assert np.isfinite(top_k_filter(row, 1)).tolist() == [False, True, False, False, False, False]


def test_frontend_on_strided_rows():
    g = np.random.default_rng(2)
    B, M, ldv, off, V, K = 2, 3, 64, 4, 40, 7
    c = g.normal(0, 2, (B, M, ldv)).astype(np.float32); u = g.normal(0, 2, (B, M, ldv)).astype(np.float32)
    out = sampling_frontend(c, u, 3.0, K, off, V)
    assert np.all(np.isneginf(out[:, :, :off])) and np.all(np.isneginf(out[:, :, off + V:]))
    assert np.all(np.isfinite(out[:, :, off:off + V]).sum(axis=-1) == K)
    q = softmax64(out[0, 0])
    assert abs(q.sum() - 1) < 1e-12 and np.count_nonzero(q) == K
    assert np.array_equal(sampling_frontend(c, u, 3.0, 0, off, V)[:, :, off:off + V],
                          guided_logits(c[:, :, off:off + V], u[:, :, off:off + V], 3.0))
