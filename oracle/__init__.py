"""CPU oracle for the draft-verify step (TEST INFRASTRUCTURE ONLY).

A plain, slow, obviously-correct numpy implementation of what the GPU library
computes: a decoder-only transformer forward pass over a KV cache (chunked
prefill and k-draft verification) and the lossless acceptance rules.  It exists
to check the HIP kernels and is never on the product path: only the tests, the
smoke check and the CPU-baseline leg of the benchmark may import it.  It shares
no code with the GPU library and imports nothing from it.

Paper anchors (section / table):
  * draft-then-verify, "only correct tokens are accepted and any tokens after
    the first mismatch are discarded"  -- Sec. 3, "NPU-only decoding ..."
  * x = [T, x_1..x_n], predictions y = [y_1..y_{n+1}], accepted prefix
    x_1..x_{e-1}, y_e                       -- Sec. 4.3, empirical analysis
  * reuse of rejected draft tokens: longest run after the rejection on which
    draft and prediction agree              -- Sec. 4.3, Eq. (reuse), Table "cases"
  * "tree-structured drafts" verified in one pass (mechanics: tree.py)
                                            -- Sec. 4, workflow
  * top successors of every prefill position from the prefill logits
                                            -- Sec. 4.2, workflow step "Sample"
  * retrieval drafts: what followed the longest earlier occurrence of the
    text's suffix                           -- Sec. 3, Sec. 5.1
  * fixed-size chunked prefill              -- Sec. 2 / Sec. 4.1
  * "executing the short graph several times equals one long execution"
                                            -- Sec. 4.1 (equivalence insight)

Parity pins (tests/test_oracle_*.py): every public function here is pinned by
invariants, closed forms, brute force on a tiny vocabulary and a library
cross-check; none is "parity unpinned".
"""
from .numfmt import round_bf16
from .transformer import ModelSpec, Weights, KVCache, forward, prefill, verify
from .acceptance import greedy_accept, stochastic_accept, first_token
from .reuse import reuse_segment, ReusePool
from .tree import verify_tree, tree_greedy_accept, tree_stochastic_accept, compact
from .calibration import topk_rows
from .drafter import suffix_match_draft

__all__ = [
    "round_bf16", "ModelSpec", "Weights", "KVCache", "forward", "prefill",
    "verify", "greedy_accept", "stochastic_accept", "first_token", "reuse_segment", "ReusePool",
    "verify_tree", "tree_greedy_accept", "tree_stochastic_accept", "compact", "topk_rows", "suffix_match_draft",
]
