"""Verification of tree-structured drafts (test infrastructure only).

The paper verifies "tree-structured drafts" (Sec. 4, workflow) and says no more
about the mechanics; what follows is the plain meaning of verifying a token
tree in one forward pass, as in the tree-attention literature it builds on:

  * rows [T, x_1..x_k] with a parent row for every draft; a node stands at the
    position of its depth and attends to the cache and to its own ancestors
    (`transformer.forward(..., parents=...)`);
  * greedy: walk down from the root; at a node whose prediction (arg-max) equals
    the token of one of its children, move to that child (the lowest row among
    equal tokens); stop otherwise and emit the prediction there.  The accepted
    drafts are the path; the output is the path's tokens and that prediction;
  * stochastic, deterministic drafter (one-hot draft distributions): at a node
    with target distribution p, the children are tried in row order against the
    residual r (r = p at first): child with token x is kept with probability
    r(x) / sum(r); a refused child's token is struck from r.  If no child is
    kept the output token is drawn from r.  For a chain this is the linear rule
    with one-hot draft distributions; for any tree the emitted token at a node
    follows p exactly (pinned by brute force);
  * afterwards the K/V rows of the accepted path move to the rows right after
    the old length, in path order, and the rest is dropped.

Uniforms: u[c - 1] decides node c (as in the linear rule, where u[i] decides
draft i + 1); u[m + i] drives the draw made at node i; m = k + 1 rows.
"""
import numpy as np

from .acceptance import _argmax_rows, inverse_cdf, softmax_t
from .transformer import forward, tree_depths


def verify_tree(spec, w, cache, tokens, parents, dt=np.float64):
    """Tree verify forward: tokens = [T, x_1..x_k], parents[0] = -1.  Returns logits [k+1, V]; the
    cache grows by k+1 rows (row len + r holds node r) until `compact`."""
    return forward(spec, w, cache, tokens, dt, parents=parents)


def children_of(parents, node):
    return [c for c in range(1, len(parents)) if int(parents[c]) == node]


def tree_greedy_accept(z, tokens, parents):
    """Returns (path, out_tokens, y): path = accepted rows starting with 0, out_tokens = tokens of
    path[1:] followed by the prediction at the last node, y = per-row arg-max."""
    tree_depths(parents)
    y = _argmax_rows(z)
    path = [0]
    while True:
        nxt = [c for c in children_of(parents, path[-1]) if int(tokens[c]) == int(y[path[-1]])]
        if not nxt:
            break
        path.append(nxt[0])
    out = [int(tokens[c]) for c in path[1:]] + [int(y[path[-1]])]
    return path, np.asarray(out, dtype=np.int32), y


def tree_stochastic_accept(z, tokens, parents, u, temperature):
    """Sequential rejection along the children, deterministic drafter.  Returns (path, out_tokens, y)."""
    tree_depths(parents)
    m = len(tokens)
    u = np.asarray(u, dtype=np.float32).astype(np.float64)
    y = _argmax_rows(z)
    path = [0]
    while True:
        cur = path[-1]
        r = softmax_t(z[cur], temperature).copy()
        kept = None
        for c in children_of(parents, cur):
            x = int(tokens[c])
            if u[c - 1] * r.sum() < r[x]:
                kept = c
                break
            r[x] = 0.0
        if kept is None:
            if r.sum() == 0.0:
                r = softmax_t(z[cur], temperature)
            out = [int(tokens[c]) for c in path[1:]] + [inverse_cdf(r, u[m + cur])]
            return path, np.asarray(out, dtype=np.int32), y
        path.append(kept)


def compact(cache, p0, path):
    """Moves the K/V rows of the accepted path to rows p0, p0+1, ... and drops everything after."""
    for j, r in enumerate(path):
        cache.k[:, :, p0 + j] = cache.k[:, :, p0 + r]
        cache.v[:, :, p0 + j] = cache.v[:, :, p0 + r]
    n = p0 + len(path)
    cache.k[:, :, n:] = 0
    cache.v[:, :, n:] = 0
    cache.len = n
