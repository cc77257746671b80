"""Pins for the oracle's acceptance rules and decoding loops (no GPU)."""
import os

import numpy as np
import pytest

import oracle
from oracle.loop import plain_greedy, speculative_greedy, speculative_step
from oracle.acceptance import inverse_cdf, softmax_t
import workloads as wl
from util_oracle import spec_of, weights_of

HERE = os.path.dirname(os.path.abspath(__file__))
TINY = wl.CONFIGS["tiny_f32"]
SMALL = wl.scaled(TINY, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=61,
                  n_layers=2)


def _logits_with_argmax(y, vocab, rng):
    z = rng.standard_normal((len(y), vocab)).astype(np.float32)
    z[np.arange(len(y)), y] = 10.0
    return z


def test_greedy_accept_hand_worked_cases():
    rng = np.random.default_rng(0)
    n = 0
    for line in open(os.path.join(HERE, "golden", "accept_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        x, y, a, out = [np.array(f.split(), dtype=np.int32) for f in line.split("|")]
        z = _logits_with_argmax(y, 12, rng)
        got_a, got_out, got_y = oracle.greedy_accept(z, x)
        assert got_a == int(a[0]) and np.array_equal(got_out, out) and np.array_equal(got_y, y), line
        n += 1
    assert n == 9


def test_greedy_argmax_tie_takes_lowest_id():
    z = np.zeros((2, 8), dtype=np.float32)
    z[0, [5, 2, 7]] = 3.0
    z[1, :] = -1.0
    a, out, y = oracle.greedy_accept(z, [2])
    assert list(y) == [2, 0] and a == 1 and list(out) == [2, 0]
    # the decision is taken on float32 values: a gap below float32 resolution is a tie
    z64 = np.zeros((1, 4), dtype=np.float64)
    z64[0, 1] = 1.0
    z64[0, 3] = 1.0 + 1e-12
    assert oracle.greedy_accept(z64, [])[2][0] == 1


def _model(cfg=SMALL):
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights, std=0.3)   # wide weights: peaked, distinct predictions
    return spec_of(cfg), weights_of(wd), s


@pytest.mark.parametrize("kind", ["random", "copied", "perfect", "perfect_then_wrong", "empty"])
def test_speculative_greedy_equals_plain_greedy(kind):
    """Lossless: any drafter leaves the emitted sequence unchanged (Sec. 3)."""
    spec, w, s = _model()
    ctx = wl.make_context(SMALL.vocab, 20, s.context)
    base = oracle.KVCache(spec, 96)
    pending = oracle.first_token(oracle.prefill(spec, w, base, ctx, 8))
    want = plain_greedy(spec, w, base.clone(), pending, 24)
    rng = s.drafts

    def drafter(hist, t):
        pos = len(hist)
        if kind == "random":
            return wl.make_context(SMALL.vocab, 4, rng)
        if kind == "copied":
            return wl.copy_span_drafts(ctx, 5, 1.0, SMALL.vocab, rng)
        if kind == "perfect":
            return want[pos:pos + 3]
        if kind == "perfect_then_wrong":
            return wl.inject_mismatch(want[pos:pos + 4], int(rng.integers(1, 6)), SMALL.vocab, rng) \
                if pos + 4 <= len(want) else []
        return []
    got, acc = speculative_greedy(spec, w, base.clone(), pending, 24, drafter)
    assert got[:24] == want
    if kind == "perfect":
        assert all(a == 3 for a in acc[:-1])                  # closed form: all accepted + bonus
        assert len(acc) == 6
    if kind in ("random", "empty"):
        assert sum(acc) <= 2                                  # one token per step, as plain decoding
    if kind == "perfect_then_wrong":
        assert 0 < sum(acc) < 4 * len(acc)


def test_first_draft_wrong_emits_plain_next_token():
    spec, w, s = _model()
    ctx = wl.make_context(SMALL.vocab, 10, s.context)
    c = oracle.KVCache(spec, 32)
    pending = oracle.first_token(oracle.prefill(spec, w, c, ctx, 10))
    nxt = plain_greedy(spec, w, c.clone(), pending, 1)[0]
    a, out, y, _ = speculative_step(spec, w, c, pending, [(nxt + 1) % SMALL.vocab, 3, 4])
    assert a == 0 and list(out) == [nxt] and c.len == 11


# ---- stochastic rule: closed forms -------------------------------------------------------------

def test_inverse_cdf_definition():
    w = [0.0, 2.0, 0.0, 1.0, 1.0]                     # cdf 0,2,2,3,4 ; total 4
    assert inverse_cdf(w, 0.0) == 1                   # never an id of zero weight
    assert inverse_cdf(w, 0.4999) == 1
    assert inverse_cdf(w, 0.5) == 3
    assert inverse_cdf(w, 0.7499) == 3
    assert inverse_cdf(w, 0.75) == 4
    assert inverse_cdf(w, 0.999999) == 4


def test_softmax_temperature_closed_form():
    z = np.log(np.array([1, 2, 4, 8], dtype=np.float64)).astype(np.float32)
    assert np.allclose(softmax_t(z, 1.0), np.array([1, 2, 4, 8]) / 15.0, rtol=1e-6)
    assert np.allclose(softmax_t(z, 0.5), np.array([1, 4, 16, 64]) / 85.0, rtol=1e-6)   # p^(1/T)


def test_draft_distribution_equal_to_target_accepts_everything():
    rng = np.random.default_rng(4)
    k, v, tau = 5, 50, 0.8
    z = rng.standard_normal((k + 1, v)).astype(np.float32) * 3
    q = np.stack([softmax_t(z[i], tau) for i in range(k)]).astype(np.float32)
    for _ in range(20):
        drafts = rng.integers(0, v, k)
        u = wl.make_uniforms(k + 1, rng)
        # q is p rounded to float32: u*q < p can only fail if u is within 1e-7 of 1
        u[:k] = np.minimum(u[:k], 0.999)
        a, out, _ = oracle.stochastic_accept(z, drafts, q, u, tau)
        assert a == k and np.array_equal(out[:k], drafts)
        assert out[k] == inverse_cdf(softmax_t(z[k], tau), u[2 * k + 1])


def test_onehot_draft_accept_probability_is_target_probability():
    # deterministic drafter (q = None): draft accepted iff u < p(x); on reject the
    # replacement is never the rejected token
    p = np.array([0.1, 0.2, 0.3, 0.4])
    z = np.log(p).astype(np.float32)[None, :].repeat(2, axis=0)
    for x in range(4):
        for u0, want in ((p[x] - 1e-4, 1), (p[x] + 1e-4, 0)):
            for u1 in (0.0, 0.3, 0.77, 0.999):
                a, out, _ = oracle.stochastic_accept(z, [x], None, [u0, 0.0, u1, 0.5], 1.0)
                assert a == want
                if a == 0:
                    assert out[0] != x
                    r = p.copy()
                    r[x] = 0
                    assert out[0] == inverse_cdf(r, np.float32(u1))


def test_zero_draft_probability_with_positive_target_is_accepted():
    z = np.zeros((2, 3), dtype=np.float32)
    q = np.array([[0.0, 0.5, 0.5]], dtype=np.float32)
    a, _, _ = oracle.stochastic_accept(z, [0], q, [0.99, 0, 0, 0.2], 1.0)
    assert a == 1


def test_stochastic_y_is_rowwise_argmax():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((4, 9)).astype(np.float32)
    _, _, y = oracle.stochastic_accept(z, [1, 2, 3], None, wl.make_uniforms(4, rng), 0.7)
    assert np.array_equal(y, z.argmax(-1))
