"""Pins for the oracle's tree-structured verification (no GPU)."""
import os

import numpy as np
import pytest

import oracle
from oracle.loop import plain_greedy, truncate
from oracle.tree import children_of
from oracle.transformer import tree_depths
import workloads as wl
from util_oracle import spec_of, weights_of

HERE = os.path.dirname(os.path.abspath(__file__))
TINY = wl.CONFIGS["tiny_f32"]
SMALL = wl.scaled(TINY, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=61, n_layers=2)
U_MAX = float(np.float32(1.0 - 2.0 ** -24))


def _model(cfg, ctx_len=11, seed=3):
    wd = wl.make_weights(cfg, wl.streams(cfg).weights, std=0.2)
    spec, w = spec_of(cfg, False), weights_of(wd)
    cache = oracle.KVCache(spec, 64)
    ctx = np.random.default_rng(seed).integers(0, cfg.vocab, ctx_len)
    oracle.prefill(spec, w, cache, ctx, 4)
    return spec, w, cache


def _random_tree(rng, k, vocab):
    parents = [-1] + [int(rng.integers(0, i)) for i in range(1, k + 1)]
    tokens = rng.integers(0, vocab, k + 1)
    return tokens, parents


def _paths_to_leaves(parents):
    leaves = [i for i in range(len(parents)) if not children_of(parents, i)]
    out = []
    for leaf in leaves:
        p, a = [], leaf
        while a >= 0:
            p.append(a)
            a = parents[a]
        out.append(p[::-1])
    return out


def test_depths_and_malformed_trees():
    assert tree_depths([-1, 0, 0, 2, 3, 1]) == [0, 1, 1, 2, 3, 2]
    for bad in ([0, 0], [-1, 1], [-1, 0, 2], [-1, -1], []):
        with pytest.raises(ValueError):
            tree_depths(bad)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_tree_is_the_linear_verify(dtype):
    spec, w, cache = _model(wl.scaled(SMALL, dtype=dtype))
    toks = np.random.default_rng(1).integers(0, SMALL.vocab, 7)
    c1, c2 = cache.clone(), cache.clone()
    z1 = oracle.verify(spec, w, c1, toks[0], toks[1:])
    z2 = oracle.verify_tree(spec, w, c2, toks, [-1, 0, 1, 2, 3, 4, 5])
    assert np.array_equal(z1, z2) and np.array_equal(c1.k, c2.k) and np.array_equal(c1.v, c2.v)


@pytest.mark.parametrize("seed", range(4))
def test_every_node_sees_exactly_its_root_path(seed):
    """The logits of a node equal those of the last row of a linear verify of its root path, and
    after compaction the cache is the one that linear verify leaves."""
    spec, w, cache = _model(SMALL)
    rng = np.random.default_rng(seed)
    tokens, parents = _random_tree(rng, 9, SMALL.vocab)
    p0 = cache.len
    ct = cache.clone()
    z = oracle.verify_tree(spec, w, ct, tokens, parents)
    assert ct.len == p0 + 10
    for path in _paths_to_leaves(parents):
        cl = cache.clone()
        zl = oracle.verify(spec, w, cl, tokens[path[0]], tokens[path[1:]])
        np.testing.assert_allclose(z[path], zl, rtol=0, atol=1e-10)
        cc = ct.clone()
        oracle.compact(cc, p0, path)
        assert cc.len == cl.len == p0 + len(path)
        np.testing.assert_allclose(cc.k, cl.k, rtol=0, atol=1e-12)
        np.testing.assert_allclose(cc.v, cl.v, rtol=0, atol=1e-12)


def test_sibling_subtrees_do_not_see_each_other():
    """Changing a token in one branch leaves the logits of every node outside its subtree unchanged."""
    spec, w, cache = _model(SMALL)
    parents = [-1, 0, 0, 1, 2, 2]
    tokens = np.array([3, 10, 20, 11, 21, 22])
    z = oracle.verify_tree(spec, w, cache.clone(), tokens, parents)
    t2 = tokens.copy()
    t2[2] = 33                                    # rows 4 and 5 hang under row 2
    z2 = oracle.verify_tree(spec, w, cache.clone(), t2, parents)
    assert np.array_equal(z[[0, 1, 3]], z2[[0, 1, 3]])
    assert not np.array_equal(z[2], z2[2]) and not np.array_equal(z[4], z2[4]) and not np.array_equal(z[5], z2[5])


def _logits_with_argmax(y, vocab, rng):
    z = rng.standard_normal((len(y), vocab)).astype(np.float32)
    z[np.arange(len(y)), y] = 10.0
    return z


def test_tree_greedy_hand_worked_cases():
    rng = np.random.default_rng(0)
    n = 0
    for line in open(os.path.join(HERE, "golden", "tree_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tokens, parents, y, path, out = [[int(t) for t in f.split()] for f in line.split("|")]
        z = _logits_with_argmax(np.array(y), 12, rng)
        got_path, got_out, got_y = oracle.tree_greedy_accept(z, tokens, parents)
        assert got_path == path and list(got_out) == out and list(got_y) == y, line
        n += 1
    assert n == 7


def test_chain_greedy_cases_agree_with_the_linear_rule():
    rng = np.random.default_rng(0)
    for line in open(os.path.join(HERE, "golden", "accept_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        x, y, a, out = [np.array(f.split(), dtype=np.int32) for f in line.split("|")]
        z = _logits_with_argmax(y, 12, rng)
        path, got_out, _ = oracle.tree_greedy_accept(z, np.concatenate([[0], x]), [-1] + list(range(len(x))))
        assert path == list(range(int(a[0]) + 1)) and np.array_equal(got_out, out)


def test_greedy_tree_decoding_equals_plain_greedy_decoding():
    """Draft trees that sometimes contain the model's own continuation: the text produced by repeated
    tree verify + compaction is the plain greedy text, whatever the trees were (lossless)."""
    spec, w, cache = _model(SMALL, ctx_len=9)
    rng = np.random.default_rng(7)
    T = 5
    want = plain_greedy(spec, w, cache.clone(), T, 24)
    got, pending, steps, accepted = [], T, 0, 0
    while len(got) < 24:
        k = int(rng.integers(0, 9))
        tokens, parents = _random_tree(rng, k, SMALL.vocab)
        tokens[0] = pending
        # plant the true continuation along one random root path
        truth = want[len(got):]
        node, d = 0, 0
        while True:
            ch = children_of(parents, node)
            if not ch or d >= len(truth) or rng.random() < 0.2:
                break
            node = int(rng.choice(ch))
            tokens[node] = truth[d]
            d += 1
        p0 = cache.len
        z = oracle.verify_tree(spec, w, cache, tokens, parents)
        path, out, _ = oracle.tree_greedy_accept(z, tokens, parents)
        oracle.compact(cache, p0, path)
        got += [int(t) for t in out]
        pending = int(out[-1])
        steps += 1
        accepted += len(path) - 1
    assert got[:24] == [int(t) for t in want]
    assert accepted > 0 and steps < 24


def test_chain_stochastic_agrees_with_the_linear_one_hot_rule():
    rng = np.random.default_rng(2)
    for _ in range(200):
        k = int(rng.integers(0, 7))
        z = (rng.standard_normal((k + 1, 9)) * 2).astype(np.float32)
        drafts = rng.integers(0, 9, k)
        u = wl.make_uniforms(k + 1, rng)
        a, out, y = oracle.stochastic_accept(z, drafts, None, u, 0.8)
        path, out_t, y_t = oracle.tree_stochastic_accept(z, np.concatenate([[0], drafts]), [-1] + list(range(k)), u, 0.8)
        assert path == list(range(a + 1)) and np.array_equal(out, out_t) and np.array_equal(y, y_t)


def _bisect(pred, iters=44):
    if not pred(0.0):
        return 0.0
    if pred(U_MAX):
        return 1.0
    lo, hi = 0.0, 1.0
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if pred(mid) else (lo, mid)
    return 0.5 * (lo + hi)


@pytest.mark.parametrize("child_tokens", [[2], [0, 3], [1, 1, 4], [4, 3, 2, 1, 0], [2, 0, 2, 3]])
def test_sequential_rejection_among_siblings_is_lossless(child_tokens):
    """Black-box measurement of the rule at one node (V = 5): the probability that child j is kept
    given the earlier ones were refused, and the distribution of the token drawn when all are
    refused, by bisection on the uniforms; summed up, the token emitted at the node follows the
    target distribution."""
    V, tau = 5, 0.8
    rng = np.random.default_rng(len(child_tokens))
    n = len(child_tokens)
    z = (rng.standard_normal((n + 1, V)) * 1.5).astype(np.float32)
    tokens = [0] + child_tokens
    parents = [-1] + [0] * n
    m = n + 1
    p = oracle.acceptance.softmax_t(z[0], tau)
    emitted = np.zeros(V)
    reach = 1.0                                   # probability that children 0..j-1 were all refused
    u = np.zeros(2 * m)
    for j in range(n):
        def kept(uj):
            uu = u.copy()
            uu[j] = uj
            path, out, _ = oracle.tree_stochastic_accept(z, tokens, parents, uu, tau)
            return len(path) > 1 and path[1] == j + 1
        a = _bisect(kept)
        emitted[child_tokens[j]] += reach * a
        reach *= 1.0 - a
        u[j] = U_MAX                              # refuse child j from here on
    if reach > 0:
        bounds = [0.0]
        for t in range(V - 1):
            def at_most(ur):
                uu = u.copy()
                uu[m + 0] = ur
                path, out, _ = oracle.tree_stochastic_accept(z, tokens, parents, uu, tau)
                assert path == [0]
                return out[-1] <= t
            bounds.append(_bisect(at_most))
        bounds.append(1.0)
        emitted += reach * np.diff(bounds)
    np.testing.assert_allclose(emitted, p, rtol=0, atol=2e-7)
