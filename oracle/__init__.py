"""CPU oracle for the static-tree relaxed-verification step (LANTERN++).

TEST INFRASTRUCTURE ONLY.  A plain, slow, float64 numpy statement of what the
verification step computes, written from the paper (Sec. 2.1, Sec. 2.2, Sec. 4,
App. A.2 Eq. 1-2).  It shares no code with the HIP library and is imported only
by ``tests/``, by ``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of
``bench.py``.  The product path never routes through it.

Functions and what pins them (see tests/test_oracle_*.py):

  build_neighbours  brute-force definition of B_k(x) (Sec. 2.2).  Pinned by
                    invariants, the Euclidean-order equivalence on unit rows and
                    an independent per-pair re-evaluation.
  tree_attention    masked softmax attention, ancestors-only mask (App. A.2
                    "Tree drafting and decoding").  Pinned by the path-unrolled
                    equivalence with ordinary causal attention and by a library
                    second opinion.
  relaxed_verify    relaxed acceptance under the multiplicative bound (Sec. 4),
                    residual resampling (Eq. 2) and the tree walk.  Pinned by
                    the reduction to plain speculative sampling (Eq. 1-2), exact
                    enumeration of the output distribution on tiny vocabularies,
                    Monte Carlo, and the bound invariants of Sec. 4.

  float32_error_bound   not part of the method: a first-order bound on what a float32
                    evaluation loses where Eq. 2's subtraction cancels; the GPU parity
                    tests add it (capped) to their relative tolerance.  Pinned by a float32
                    replay of the same rows: never exceeded, and within a stated factor of
                    the observed error where it matters.

  commit_kv         appends the K/V rows of the root and of the accepted path to
                    the cache (App. A.2).  Pinned by the next step's view: plain
                    attention over the committed cache equals the tree-masked
                    attention row of the last accepted node.

  sampling_frontend classifier-free guidance + top-k in front of the target softmax
                    (App. B "Models").  Pinned by special cases (scale 0, equal rows),
                    a library top-k, counts and brute force.

Readings the paper does not fix ("parity unpinned": every invariant the paper
states holds under the alternatives too, so the choice below is the definition):
  * A_{k,lambda} is the longest nearest-first prefix of B_k whose cumulative
    target mass stays below lambda*q(x^), the drafted token always included;
  * after a rejection the "adjusted distribution" is the target with A's mass
    moved onto the drafted token, and the resample distribution is the
    normalised positive part of (adjusted - drafter);
  * siblings are i.i.d. drafter samples tried in index order, each against the
    current residual;
  (the other reading of each of these two is available as an option of
  ``relaxed_verify``: ``rule="skip"`` passes over a neighbour that would break the
  bound and goes on down the list; ``siblings="without_replacement"`` takes a
  rejected child's token out of the drafter distribution before the next child --
  pinned by a hand example, a maximality check and exact enumeration of the output law)
  * the tree generator in ``workloads.tree`` (the paper's figure is not text).
"""
from .knn import build_neighbours, similarity_keys            # noqa: F401
from .attention import tree_attention, ancestor_mask          # noqa: F401
from .verify import relaxed_verify, softmax64, inverse_cdf    # noqa: F401
from .f32_bound import float32_error_bound                    # noqa: F401
from .commit import commit_kv                                 # noqa: F401
from .frontend import guided_logits, top_k_filter, sampling_frontend   # noqa: F401
