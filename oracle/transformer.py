"""Plain decoder-only transformer forward over a KV cache (test infrastructure).

The model is the one the workload configs fix: pre-norm blocks with RMSNorm,
rotary position embedding (rotate-half pairing), grouped-query causal
attention, a SwiGLU feed-forward, and an output head tied to the embedding.
The paper only names the model families it runs (Sec. 5.1, "Models"); the
operator set follows those families.

Everything is written out as its textbook definition, row by row where that is
the clearest form; no blocking, fusion or reordering.  Arithmetic is float64
by default.  In "bf16" mode the values are rounded to bfloat16 at exactly the
points where the GPU path stores or feeds a bfloat16 tensor:
  weights (already bfloat16 values on input), the input of every linear layer
  (normalised activations, attention output, SwiGLU product), q after RoPE,
  and K (after RoPE) and V as they are stored in the cache.
Everything else (residual stream, accumulators, softmax, logits) is unrounded.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from .numfmt import round_bf16


@dataclass
class ModelSpec:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # "bf16" | "f32": where rounding points apply
    rope_theta: float = 10000.0
    rms_eps: float = 1e-6
    qkv_bias: bool = False


@dataclass
class LayerWeights:
    attn_norm: np.ndarray        # [d]
    wq: np.ndarray               # [Hq*hd, d]   (row-major [out, in])
    wk: np.ndarray               # [Hkv*hd, d]
    wv: np.ndarray               # [Hkv*hd, d]
    wo: np.ndarray               # [d, Hq*hd]
    ffn_norm: np.ndarray         # [d]
    w_gate: np.ndarray           # [F, d]
    w_up: np.ndarray             # [F, d]
    w_down: np.ndarray           # [d, F]
    bq: Optional[np.ndarray] = None
    bk: Optional[np.ndarray] = None
    bv: Optional[np.ndarray] = None


@dataclass
class Weights:
    embed: np.ndarray            # [V, d]; also the output head (tied)
    final_norm: np.ndarray       # [d]
    layers: List[LayerWeights] = field(default_factory=list)

    def astype(self, dt):
        """Copy with every array converted to dtype `dt` (values unchanged)."""
        def c(a):
            return None if a is None else np.asarray(a, dtype=dt)
        return Weights(c(self.embed), c(self.final_norm), [
            LayerWeights(**{k: c(v) for k, v in vars(l).items()}) for l in self.layers])


class KVCache:
    """K and V of every layer for positions 0..len-1: arrays [L, Hkv, cap, hd]."""

    def __init__(self, spec: ModelSpec, capacity: int, dt=np.float64):
        shp = (spec.n_layers, spec.n_kv_heads, capacity, spec.head_dim)
        self.k = np.zeros(shp, dtype=dt)
        self.v = np.zeros(shp, dtype=dt)
        self.len = 0
        self.capacity = capacity

    def clone(self):
        c = object.__new__(KVCache)
        c.k, c.v, c.len, c.capacity = self.k.copy(), self.v.copy(), self.len, self.capacity
        return c


def rmsnorm(h, g, eps):
    """RMSNorm(h) = h / sqrt(mean(h^2) + eps) * g, along the last axis."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * g


def rope_tables(positions, head_dim, theta):
    """cos/sin of angle pos * theta^(-2i/hd), i = 0..hd/2-1.

    Computed in float64, then rounded to float32: the angle table is data both
    sides hold in single precision.
    """
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.power(np.float64(theta), -2.0 * i / head_dim)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return (np.cos(ang).astype(np.float32).astype(np.float64),
            np.sin(ang).astype(np.float32).astype(np.float64))


def rope(x, cos, sin):
    """Rotate pairs (i, i + hd/2) of x[n, heads, hd] by the per-position angle."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(a):
    return a / (1.0 + np.exp(-a))


def tree_depths(parents):
    """Depth of every node of a draft tree given as parent row indices: parents[0] = -1 (the root,
    the pending token), 0 <= parents[i] < i for the others."""
    parents = [int(p) for p in parents]
    if not parents or parents[0] != -1 or any(not 0 <= p < i for i, p in enumerate(parents) if i):
        raise ValueError("parents must start with -1 and point to earlier rows")
    depth = [0] * len(parents)
    for i in range(1, len(parents)):
        depth[i] = depth[parents[i]] + 1
    return depth


def forward(spec: ModelSpec, w: Weights, cache: KVCache, tokens, dt=np.float64, parents=None, logit_rows=None):
    """Run `tokens` (ids) at positions cache.len.. through the model.

    Appends their K/V rows to the cache and returns the logits [n, V] (dtype
    `dt`): row r is the model's prediction for the token after position
    cache.len + r.  `w` must already hold arrays of dtype `dt`.

    logit_rows: if given, the output head is applied to these rows only and
    the result is [len(logit_rows), V] (the same values: a row's logits depend
    on no other row of the final hidden state); the layers run on all rows.

    parents (tree-structured drafts, Sec. 4 "tree-structured drafts"): row r is
    a node of a token tree rooted at row 0.  It stands at the position of its
    depth, cache.len + depth[r], sees the whole cache and, of the rows of this
    call, only its ancestors and itself; its K/V go to cache row cache.len + r.
    Row r then predicts the token after the root-to-r path.
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    n = tokens.shape[0]
    p0 = cache.len
    if p0 + n > cache.capacity:
        raise ValueError("KV cache capacity exceeded")
    act = (lambda a: round_bf16(a)) if spec.dtype == "bf16" else (lambda a: a)
    hq, hkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    group = hq // hkv
    if parents is None:
        pos = p0 + np.arange(n)
        # key t is visible to row r iff t <= pos[r]
        visible = np.arange(p0 + n)[None, :] <= pos[:, None]
    else:
        if len(parents) != n:
            raise ValueError("one parent per row")
        pos = p0 + np.asarray(tree_depths(parents))
        visible = np.zeros((n, p0 + n), dtype=bool)
        visible[:, :p0] = True
        for r in range(n):
            a = r
            while a >= 0:
                visible[r, p0 + a] = True
                a = int(parents[a])
    cos, sin = rope_tables(pos, hd, spec.rope_theta)
    cos, sin = cos.astype(dt), sin.astype(dt)
    scale = 1.0 / np.sqrt(np.float64(hd))

    h = w.embed[tokens].astype(dt)
    for l, lw in enumerate(w.layers):
        x = act(rmsnorm(h, lw.attn_norm, spec.rms_eps))
        q = x @ lw.wq.T
        k = x @ lw.wk.T
        v = x @ lw.wv.T
        if spec.qkv_bias:
            q, k, v = q + lw.bq, k + lw.bk, v + lw.bv
        q = act(rope(q.reshape(n, hq, hd), cos, sin))
        k = act(rope(k.reshape(n, hkv, hd), cos, sin))
        v = act(v.reshape(n, hkv, hd))
        cache.k[l, :, p0:p0 + n] = k.transpose(1, 0, 2)
        cache.v[l, :, p0:p0 + n] = v.transpose(1, 0, 2)
        o = np.empty((n, hq, hd), dtype=dt)
        for j in range(hq):
            kk = cache.k[l, j // group, :p0 + n]
            vv = cache.v[l, j // group, :p0 + n]
            s = (q[:, j] @ kk.T) * scale
            s = np.where(visible, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            e = np.exp(s)
            o[:, j] = (e / e.sum(axis=-1, keepdims=True)) @ vv
        o = act(o.reshape(n, hq * hd))
        h = h + o @ lw.wo.T
        x = act(rmsnorm(h, lw.ffn_norm, spec.rms_eps))
        a = act(silu(x @ lw.w_gate.T) * (x @ lw.w_up.T))
        h = h + a @ lw.w_down.T
    cache.len = p0 + n
    if logit_rows is not None:
        h = h[np.asarray(logit_rows, dtype=np.int64)]
    return act(rmsnorm(h, w.final_norm, spec.rms_eps)) @ w.embed.T


def prefill(spec, w, cache, tokens, chunk, dt=np.float64):
    """Chunked prefill (Sec. 2, Sec. 4.1): feed `tokens` in pieces of `chunk`.

    The last piece may be shorter.  Returns the logits of the last row only.
    """
    tokens = np.asarray(tokens)
    z = None
    for s in range(0, len(tokens), chunk):
        piece = tokens[s:s + chunk]
        z = forward(spec, w, cache, piece, dt, logit_rows=[len(piece) - 1])
    return z[-1]


def verify(spec, w, cache, pending, drafts, dt=np.float64):
    """Verify forward (Sec. 4.3): rows [T, x_1..x_k] at positions len..len+k.

    Returns logits z[k+1, V]; z[i] predicts the token after [.., T, x_1..x_i].
    The cache grows by k+1 rows; the caller truncates it after acceptance.
    """
    return forward(spec, w, cache, np.concatenate([[pending], np.asarray(drafts, dtype=np.int64)]), dt)
