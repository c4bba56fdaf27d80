"""Seeded input tensors (numpy, CPU).  No arithmetic of the method lives here.

Every array comes from ``numpy.random.Generator(Philox(...))`` keyed by
``seed_for(cfg, stream)`` and a per-kind tag, so one batch item can be
regenerated alone (``stream`` = batch item).  bf16 tensors are returned both as
raw 16-bit patterns (what is uploaded) and as the float32 values those patterns
denote (what a checker reads), so both sides see identical inputs.
"""
from typing import Dict, Optional, Sequence

import numpy as np

from .configs import Config
from .tree import children_lists

_BASE = 20250206 * 100
_KIND = {"codebook": 1, "q": 2, "kt": 3, "vt": 4, "kc": 5, "vc": 6,
         "target": 7, "drafter": 8, "tokens": 9, "u_accept": 10, "u_final": 11}


def seed_for(cfg_idx: int, stream: int = 0) -> int:
    return _BASE + 10 * int(cfg_idx) + int(stream)


def _rng(cfg_idx: int, stream: int, kind: str, salt: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([seed_for(cfg_idx, stream), _KIND[kind], int(salt)])
    return np.random.Generator(np.random.Philox(ss))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> float32 holding the nearest bf16 value."""
    return (bf16_bits(x).astype(np.uint32) << 16).view(np.float32)


def make_codebook(cfg: Config, salt: int = 0) -> np.ndarray:
    """VQ codebook: N(0,1) rows, L2-normalised in float64, stored float32 [V,D]."""
    g = _rng(cfg.idx, 0, "codebook", salt)
    e = g.standard_normal((cfg.V, cfg.D))
    e /= np.sqrt((e * e).sum(axis=1, keepdims=True))
    return e.astype(np.float32)


def _normal(cfg, stream, kind, shape, salt):
    return _rng(cfg.idx, stream, kind, salt).standard_normal(shape, dtype=np.float32)


def make_attention_inputs(cfg: Config, items: Optional[Sequence[int]] = None,
                          salt: int = 0) -> Dict[str, np.ndarray]:
    """Q / tree K,V ``[B,H,M,Dh]`` and cached K,V ``[B,H,S,Dh]``, all N(0,1).

    Returns float32 value arrays under q,kt,vt,kc,vc; for a bf16 config the
    values are bf16-representable and ``<name>_bits`` holds the uint16 patterns.
    ``items`` selects batch items (default ``range(cfg.B)``); item b uses
    seed stream b.
    """
    items = list(range(cfg.B)) if items is None else list(items)
    out: Dict[str, np.ndarray] = {}
    for kind, rows in (("q", cfg.M), ("kt", cfg.M), ("vt", cfg.M), ("kc", cfg.S), ("vc", cfg.S)):
        per = [_normal(cfg, b, kind, (cfg.H, rows, cfg.Dh), salt) for b in items]
        x = np.stack(per, axis=0)
        if cfg.kv_dtype == "bf16":
            bits = bf16_bits(x)
            out[kind + "_bits"] = bits
            x = (bits.astype(np.uint32) << 16).view(np.float32)
        out[kind] = x
    return out


def make_verify_inputs(cfg: Config, parent: np.ndarray, rho: float = 0.0,
                       items: Optional[Sequence[int]] = None, salt: int = 0,
                       topk_filter: int = 0) -> Dict[str, np.ndarray]:
    """Per-row logits, drafted tokens and the uniforms of one verification step.

    target logits ~ N(0, sigma^2); drafter = rho*target + sqrt(1-rho^2)*N(0, sigma^2)
    (marginal N(0, sigma^2) for every rho).  Image token x sits at column
    ``vocab_offset + x`` of a row of ``ldv`` columns; the other columns are -inf.
    The children of row P are i.i.d. draws (with replacement) from the drafter's
    distribution at P, taken by inverse CDF.  ``topk_filter`` > 0 sets all but
    the largest ``topk_filter`` target logits of every row to -inf.
    """
    items = list(range(cfg.B)) if items is None else list(items)
    M, V, off = len(parent), cfg.V, cfg.vocab_offset
    kids = children_lists(parent)
    nb = len(items)
    target = np.full((nb, M, cfg.ldv), -np.inf, dtype=np.float32)
    drafter = np.full((nb, M, cfg.ldv), -np.inf, dtype=np.float32)
    tokens = np.zeros((nb, M), dtype=np.int32)
    u_accept = np.zeros((nb, M), dtype=np.float32)
    u_final = np.zeros((nb, M), dtype=np.float32)
    c = float(np.sqrt(max(0.0, 1.0 - rho * rho)))
    for n, b in enumerate(items):
        t = _normal(cfg, b, "target", (M, V), salt) * np.float32(cfg.sigma)
        z = _normal(cfg, b, "drafter", (M, V), salt) * np.float32(cfg.sigma)
        d = (np.float32(rho) * t + np.float32(c) * z).astype(np.float32)
        if topk_filter and topk_filter < V:
            kth = np.partition(t, V - topk_filter, axis=1)[:, V - topk_filter][:, None]
            t = np.where(t >= kth, t, -np.inf).astype(np.float32)
        target[n, :, off:off + V] = t
        drafter[n, :, off:off + V] = d
        g = _rng(cfg.idx, b, "tokens", salt)
        for P in range(M):
            if not kids[P]:
                continue
            w = np.exp(d[P].astype(np.float64) - float(d[P].max()))
            cdf = np.cumsum(w)
            draws = g.random(len(kids[P])) * cdf[-1]
            tok = np.minimum(np.searchsorted(cdf, draws, side="right"), V - 1)
            tokens[n, kids[P]] = tok.astype(np.int32)
        u_accept[n] = _rng(cfg.idx, b, "u_accept", salt).random(M, dtype=np.float32)
        u_final[n] = _rng(cfg.idx, b, "u_final", salt).random(M, dtype=np.float32)
    return {"target_logits": target, "drafter_logits": drafter, "tokens": tokens,
            "u_accept": u_accept, "u_final": u_final}
