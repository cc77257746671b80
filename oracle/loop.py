"""Decoding loops built from the oracle's verify and accept (test infrastructure).

plain_greedy   : one token per forward pass -- the sequence speculative
                 decoding must reproduce token for token (Sec. 3, lossless).
speculative    : draft -> verify -> accept -> commit, repeated (Sec. 4.3).
"""
import numpy as np

from .transformer import forward, verify
from .acceptance import greedy_accept, stochastic_accept


def truncate(cache, new_len):
    """Drop cache rows at positions >= new_len (rejected drafts)."""
    cache.k[:, :, new_len:] = 0
    cache.v[:, :, new_len:] = 0
    cache.len = new_len


def plain_greedy(spec, w, cache, pending, n_tokens, dt=np.float64):
    """Feed `pending`, emit arg-max, repeat; returns the n_tokens emitted."""
    out = []
    t = int(pending)
    for _ in range(n_tokens):
        z = forward(spec, w, cache, [t], dt)
        t = int(np.argmax(z[0].astype(np.float32)))
        out.append(t)
    return out


def speculative_step(spec, w, cache, pending, drafts, mode="greedy", q=None, u=None,
                     temperature=1.0, dt=np.float64):
    """One draft-verify step.  Returns (n_accept, out_tokens, y, z).

    State after the step: cache holds the context, the pending token and the
    accepted drafts (len grows by 1 + n_accept); the new pending token is
    out_tokens[-1].
    """
    ctx = cache.len
    z = verify(spec, w, cache, pending, drafts, dt)
    if mode == "greedy":
        a, out, y = greedy_accept(z, drafts)
    else:
        a, out, y = stochastic_accept(z, drafts, q, u, temperature)
    truncate(cache, ctx + 1 + a)
    return a, out, y, z


def speculative_greedy(spec, w, cache, pending, n_tokens, drafter, dt=np.float64):
    """Greedy speculative decoding until at least n_tokens are emitted.

    drafter(history_tokens, pending) -> list of draft ids (may be empty).
    Returns (emitted tokens, accepted count per step).
    """
    out, acc = [], []
    t = int(pending)
    while len(out) < n_tokens:
        drafts = list(drafter(out, t))
        a, toks, _, _ = speculative_step(spec, w, cache, t, drafts, "greedy", dt=dt)
        out.extend(int(v) for v in toks)
        acc.append(a)
        t = int(toks[-1])
    return out, acc
