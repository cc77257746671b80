"""Seeded generators: weights, contexts, drafts, uniforms, the batched RAG mix.

Master seed 15312.  Config i draws from PCG64(15312*10 + i), split into
independent sub-streams in the fixed order
    weights, context, drafts, gumbel, uniforms, mix.
"""
from types import SimpleNamespace

import numpy as np
import torch

MASTER_SEED = 15312
_STREAMS = ("weights", "context", "drafts", "gumbel", "uniforms", "mix")


def streams(cfg):
    """Independent numpy Generators for one config, by name."""
    kids = np.random.SeedSequence(MASTER_SEED * 10 + cfg.index).spawn(len(_STREAMS))
    return SimpleNamespace(**{n: np.random.Generator(np.random.PCG64(s))
                              for n, s in zip(_STREAMS, kids)})


def to_bf16_values(a):
    """float32 array whose values are the nearest bfloat16 values (library cast)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def _normal(rng, shape, std, bf16):
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return to_bf16_values(a) if bf16 else a


def make_weights(cfg, rng, std=0.02, qkv_bias=False):
    """Every matrix iid N(0, std^2) (then rounded to bfloat16 values for bf16
    configs); RMSNorm gains are 1.  Arrays are float32, row-major [out, in]."""
    bf = cfg.dtype == "bf16"
    d, hd, f = cfg.d_model, cfg.head_dim, cfg.d_ffn
    nq, nkv = cfg.n_q_heads * hd, cfg.n_kv_heads * hd
    w = {"embed": _normal(rng, (cfg.vocab, d), std, bf),
         "final_norm": np.ones(d, dtype=np.float32), "layers": []}
    for _ in range(cfg.n_layers):
        lw = {
            "attn_norm": np.ones(d, dtype=np.float32),
            "wq": _normal(rng, (nq, d), std, bf),
            "wk": _normal(rng, (nkv, d), std, bf),
            "wv": _normal(rng, (nkv, d), std, bf),
            "wo": _normal(rng, (d, nq), std, bf),
            "ffn_norm": np.ones(d, dtype=np.float32),
            "w_gate": _normal(rng, (f, d), std, bf),
            "w_up": _normal(rng, (f, d), std, bf),
            "w_down": _normal(rng, (d, f), std, bf),
        }
        if qkv_bias:
            lw["bq"] = _normal(rng, (nq,), std, bf)
            lw["bk"] = _normal(rng, (nkv,), std, bf)
            lw["bv"] = _normal(rng, (nkv,), std, bf)
        w["layers"].append(lw)
    return w


def make_context(vocab, n, rng):
    """n token ids uniform in [0, vocab)."""
    return rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def copy_span_drafts(context, k, p_copy, vocab, rng):
    """With probability p_copy the drafts are a random k-token span of the
    context (what a retrieval drafter proposes), otherwise k uniform ids."""
    if rng.random() < p_copy and len(context) > k:
        s = int(rng.integers(0, len(context) - k + 1))
        return np.asarray(context[s:s + k], dtype=np.int32)
    return rng.integers(0, vocab, size=k, dtype=np.int64).astype(np.int32)


def geometric_copy_drafts(context, k, mean_len, vocab, rng):
    """A copied context span of geometric length (mean mean_len, clipped to k)
    followed by uniform ids."""
    c = min(int(rng.geometric(1.0 / mean_len)), k)
    s = int(rng.integers(0, len(context) - c + 1))
    tail = rng.integers(0, vocab, size=k - c, dtype=np.int64)
    return np.concatenate([np.asarray(context[s:s + c], dtype=np.int64), tail]).astype(np.int32)


def inject_mismatch(continuation, e, vocab, rng):
    """Drafts equal to `continuation` (the target's own next k tokens) except
    that draft e (1-based) is replaced by a different id; e = k+1 leaves all k
    intact.  Sweeps the accepted count over 0..k."""
    d = np.asarray(continuation, dtype=np.int32).copy()
    if e <= len(d):
        wrong = int(rng.integers(0, vocab - 1))
        d[e - 1] = wrong if wrong < d[e - 1] else wrong + 1
    return d


def gumbel_drafts(next_logits, pending, k, temperature, scale, rng_gumbel, rng_u):
    """Drafts that carry a draft distribution: along the draft path,
    q_i = softmax(z_i / temperature + scale * g_i) with g_i iid standard Gumbel
    noise, x_i sampled from q_i by inverse CDF.

    next_logits(token) -> logits [V] of the target after feeding `token`
    (the callee keeps the running state).  Returns (drafts int32[k],
    q float32[k, V]).
    """
    drafts, qs = [], []
    tok = int(pending)
    for _ in range(k):
        z = np.asarray(next_logits(tok), dtype=np.float64)
        g = rng_gumbel.gumbel(size=z.shape)
        s = z / temperature + scale * g
        e = np.exp(s - s.max())
        q = (e / e.sum()).astype(np.float32)
        c = np.cumsum(q.astype(np.float64))
        tok = int(min(np.searchsorted(c, rng_u.random() * c[-1], side="right"), len(c) - 1))
        drafts.append(tok)
        qs.append(q)
    return np.asarray(drafts, dtype=np.int32), np.stack(qs)


def make_uniforms(rows, rng):
    """2*rows float32 uniforms in [0, 1): acceptance then replacement draws."""
    u = rng.random(2 * rows, dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


def rag_mix(cfg, rng, ctx_min=512, ctx_max=8192, sigma=0.6):
    """Batched RAG mix: per sequence a lognormal context length (median cfg.ctx,
    clipped), a draft length uniform in 1..cfg.k, an acceptance mode (both modes
    occur), and a block table that is a random permutation of the page pool."""
    b = cfg.batch
    ctx = np.clip(np.rint(np.exp(rng.normal(np.log(cfg.ctx), sigma, size=b))),
                  ctx_min, ctx_max).astype(np.int64)
    k = rng.integers(1, cfg.k + 1, size=b)
    while True:
        stochastic = rng.random(b) < 0.5
        if b < 2 or (stochastic.any() and not stochastic.all()):
            break
    pt = cfg.page_tokens
    pages_per_seq = [int(-(-(c + kk + 1) // pt)) for c, kk in zip(ctx, k)]
    n_pages = int(sum(pages_per_seq))
    perm = rng.permutation(n_pages).astype(np.int32)
    tables, o = [], 0
    for n in pages_per_seq:
        tables.append(perm[o:o + n].copy())
        o += n
    return SimpleNamespace(ctx=ctx, k=k, stochastic=stochastic, n_pages=n_pages,
                           block_tables=tables)
