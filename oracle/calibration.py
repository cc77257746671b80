"""Top successors of every prefill position (test infrastructure only).

Sec. 4.2 ("Leverage prefill logits", workflow step "Sample"): after prefill the
method takes, for every context position, the top-probability successor tokens
from that position's next-token logits and builds its calibrated token tree
from them.  The softmax is monotone, so the k most probable successors of a
row are the k largest logits of that row.

`topk_rows` is that definition: per row, ids ordered by falling logit, equal
logits by rising id (the arg-max convention of the acceptance rule), cut at k.
Only the selection is specified here; how the token tree is searched afterwards
is host logic of the drafter and outside this library.
"""
import numpy as np


def topk_rows(z, k):
    """z: logits [n, V] (float32 values); returns (values [n, k] float32, ids [n, k] int32)."""
    z = np.asarray(z, dtype=np.float32)
    n, V = z.shape
    if not 1 <= k <= V:
        raise ValueError("k out of range")
    ids = np.empty((n, k), dtype=np.int32)
    for r in range(n):
        # lexsort: last key is the primary one; ties of -z fall back to the id
        order = np.lexsort((np.arange(V), -z[r].astype(np.float64)))
        ids[r] = order[:k]
    return np.take_along_axis(z, ids.astype(np.int64), axis=1), ids
