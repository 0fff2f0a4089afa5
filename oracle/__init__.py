"""CPU checker for the tree-verification path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 NumPy written from the paper's statement of each operation.
Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import it;
the GPU library never does, and nothing here imports the GPU library.

Pin status (see tests/test_oracle_*.py):
  draft_entropy_topk  pinned: closed forms (uniform, one-hot, two-point), hand-summed tiny
                      vocabularies with math.fsum, permutation / shift invariance, K = V.
  tree_prune          pinned: brute-force path products on tiny trees, ancestor-closure,
                      monotonicity in theta, identity when all filters are off.
  tree_attention      pinned: chain tree == dense causal attention, star tree == independent
                      single-query attentions, dense-mask brute force, constant-V, GQA replication.
  verify_accept       pinned: brute-force longest matching path (greedy), planted paths, chain tree
                      == textbook speculative sampling, exact output-distribution enumeration
                      on tiny vocabularies, one-hot target == greedy.
  adaptive_control    pinned: the Section 4.3 formulas worked by hand on the framework figure's
                      example, Eq. 1 on uniform rows (T ln K), brute-force enumeration of the
                      deepest paths, numpy.searchsorted for the bin lookup.
  tree_expand         pinned: hand-worked two-level tree, brute-force ranking by float64 path
                      products, structural invariants, the pipeline's whole-tree builder.
  tree_validate       pinned: hand-made trees with known defects, and validity == every row reaches
                      the root through earlier rows.
  kv_commit           pinned: numpy.concatenate of the accepted rows, and decoding through several
                      commits equals dense causal attention (torch) over the whole sequence; the
                      paged forms (kv_commit_paged, gather_pages) by scatter / gather identity and
                      equality with the dense commit.
"""
from .entropy_topk import draft_entropy_topk
from .tree_prune import tree_prune
from .tree_attention import tree_attention
from .verify_accept import verify_accept
from .adaptive_control import adaptive_control
from .tree_expand import tree_expand
from .kv_commit import kv_commit

__all__ = ["draft_entropy_topk", "tree_prune", "tree_attention", "verify_accept", "adaptive_control", "tree_expand", "kv_commit"]
