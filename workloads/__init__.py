"""Seeded synthetic inputs for the static-tree relaxed-verification path.

This package only *produces inputs* (shapes, value distributions, tree
topologies).  It holds none of the method's arithmetic and is imported by the
tests, by ``bench.py`` and by ``__graft_entry__.py``; neither ``oracle/`` nor
the HIP path depends on it for anything they compute.
"""
from .configs import CONFIGS, Config, get_config            # noqa: F401
from .tree import static_tree, tree_depths, children_lists  # noqa: F401
from .gen import (                                           # noqa: F401
    make_codebook, make_attention_inputs, make_verify_inputs,
    bf16_round, bf16_bits, seed_for,
)
