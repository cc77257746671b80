"""Tree-structured draft verification through the C ABI against the oracle: logits of random trees
(float32 model on the general kernels, bfloat16 model on the persistent kernel and on the general
kernels, ragged batches), acceptance on crafted logits (bit-exact path, tokens, state), compaction
of the accepted path, and lossless greedy decoding with trees."""
import numpy as np
import pytest
import torch

import oracle
from oracle.loop import plain_greedy
from oracle.tree import children_of
import workloads as wl
import paper_2510_15312_amd as vf
from util_oracle import rel_inf
from util_gpu import DEV, Pair, tol_of, i32, f32

pytestmark = pytest.mark.gpu
C = wl.CONFIGS
GREEDY = (vf.VF_GREEDY, 0.0, None, None)


def _random_tree(rng, k, vocab, branchy=0.5):
    """Parents of a random tree with k drafts: chains with side branches."""
    parents = [-1]
    for i in range(1, k + 1):
        parents.append(i - 1 if rng.random() > branchy else int(rng.integers(0, i)))
    return rng.integers(0, vocab, k + 1).astype(np.int32), parents


def _gpu_accept_tree(pair, seqs, tokens, row_off, parents, params, logits=None):
    n, total = len(seqs), int(row_off[-1])
    n_acc = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    out, y, path = (torch.full((total,), -7, dtype=torch.int32, device=DEV) for _ in range(3))
    vf.vf_accept_tree(pair.model, seqs, tokens, row_off, parents, params, n_acc, out, y, path, logits)
    torch.cuda.synchronize()
    return n_acc.cpu().numpy(), out.cpu().numpy(), y.cpu().numpy(), path.cpu().numpy()


CASES = {
    # name: (config, context lengths of the batch, drafts per sequence, fast path option)
    "tiny_f32": (C["tiny_f32"], [70], [9], 1),
    "tiny_f32_batch": (C["tiny_f32"], [130, 5, 64], [32, 0, 7], 1),
    "1.5b_shape_persistent": (wl.scaled(C["1.5b_k16"], n_layers=2, vocab=4096), [200], [16], 1),
    "1.5b_shape_batch_persistent": (wl.scaled(C["1.5b_k16"], n_layers=2, vocab=4096), [97, 260], [32, 12], 1),
    "1.5b_shape_general": (wl.scaled(C["1.5b_k16"], n_layers=2, vocab=4096), [97, 260], [32, 12], 0),
    "0.5b_shape_persistent": (wl.scaled(C["0.5b_k8"], n_layers=2, vocab=4096), [150], [8], 1),
}


@pytest.mark.parametrize("name", list(CASES))
def test_tree_verify_logits_and_compaction_against_oracle(name):
    cfg, ctxs, ks, fast = CASES[name]
    print(f"case {name}: contexts {ctxs} drafts {ks} fast path {fast}", flush=True)
    tol = tol_of(cfg)
    rows = sum(k + 1 for k in ks)
    pair = Pair(cfg, max_rows=max(64, rows), max_positions=max(ctxs) + 80)
    vf.vf_set_option(pair.model, vf.VF_OPT_FAST_PATH, fast)
    rng = np.random.default_rng(11)
    seqs, caches, toks, pars, row_off = [], [], [], [], [0]
    for n_ctx, k in zip(ctxs, ks):
        cap = n_ctx + 2 * 33 + 2
        seq, cache = pair.new_seq(cap), oracle.KVCache(pair.spec, cap)
        pair.prefill_both(seq, cache, wl.make_context(cfg.vocab, n_ctx, rng), 64)
        t, p = _random_tree(rng, k, cfg.vocab)
        seqs.append(seq); caches.append(cache); toks.append(t); pars.append(p)
        row_off.append(row_off[-1] + k + 1)
    tokens = np.concatenate(toks)
    parents = [p for ps in pars for p in ps]
    tok_dev = i32(tokens)
    logits = torch.empty((rows, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify_tree(pair.model, seqs, tok_dev, row_off, parents, logits)
    torch.cuda.synchronize()
    z_gpu = logits.cpu().numpy()
    z_or = [oracle.verify_tree(pair.spec, pair.ow, c, t, p) for c, t, p in zip(caches, toks, pars)]
    err = rel_inf(z_gpu, np.concatenate(z_or)).max()
    print(f"tree verify: max rel-inf logit error {err:.3e} (tol {tol:g})", flush=True)
    assert np.isfinite(z_gpu).all() and err < tol
    # greedy acceptance on the GPU's own logits; the oracle walks the same logits
    n_acc, out, y, path = _gpu_accept_tree(pair, seqs, tok_dev, row_off, parents, [GREEDY] * len(seqs), logits)
    kv_tol = 1e-2 if cfg.dtype == "bf16" else 1e-5
    for b, (seq, cache, t, p, n_ctx) in enumerate(zip(seqs, caches, toks, pars, ctxs)):
        r0, r1 = row_off[b], row_off[b + 1]
        want_path, want_out, want_y = oracle.tree_greedy_accept(z_gpu[r0:r1], t, p)
        a = len(want_path) - 1
        assert n_acc[b] == a and list(path[r0:r0 + a + 1]) == want_path and np.all(path[r0 + a + 1:r1] == -1)
        assert np.array_equal(out[r0:r0 + a + 1], want_out) and np.array_equal(y[r0:r1], want_y)
        assert vf.vf_seq_get_state(seq) == (n_ctx + 1 + a, int(want_out[-1]))
        oracle.compact(cache, n_ctx, want_path)
        for layer in (0, cfg.n_layers - 1):
            (kg, vg), (ko, vo) = pair.kv_both(seq, cache, layer, n_ctx, a + 1)
            assert np.abs(kg - ko).max() <= kv_tol * np.abs(ko).max(), ("K", b, layer)
            assert np.abs(vg - vo).max() <= kv_tol * np.abs(vo).max(), ("V", b, layer)
    # the compacted caches carry on: one plain verify step on top of them
    nxt = [np.concatenate([[int(o_[-1])], rng.integers(0, cfg.vocab, 3)]).astype(np.int32)
           for o_ in (oracle.tree_greedy_accept(z_gpu[row_off[b]:row_off[b + 1]], toks[b], pars[b])[1]
                      for b in range(len(seqs)))]
    ro2 = [4 * i for i in range(len(seqs) + 1)]
    logits2 = torch.empty((ro2[-1], cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify(pair.model, seqs, i32(np.concatenate(nxt)), ro2, logits2)
    torch.cuda.synchronize()
    z2 = np.concatenate([oracle.verify(pair.spec, pair.ow, c, t[0], t[1:]) for c, t in zip(caches, nxt)])
    err2 = rel_inf(logits2.cpu().numpy(), z2).max()
    print(f"plain verify on the compacted cache: max rel-inf logit error {err2:.3e}", flush=True)
    assert err2 < tol


def test_chain_tree_equals_plain_verify_bit_for_bit():
    cfg = wl.scaled(C["1.5b_k16"], n_layers=2, vocab=4096)
    pair = Pair(cfg, max_rows=64, max_positions=256)
    rng = np.random.default_rng(4)
    ctx = i32(wl.make_context(cfg.vocab, 100, rng))
    toks = i32(rng.integers(0, cfg.vocab, 17))
    out = []
    for tree in (False, True):
        seq = pair.new_seq(200)
        vf.vf_prefill_chunk(pair.model, seq, ctx[:64]); vf.vf_prefill_chunk(pair.model, seq, ctx[64:])
        z = torch.empty((17, cfg.vocab), dtype=torch.float32, device=DEV)
        if tree:
            vf.vf_verify_tree(pair.model, [seq], toks, [0, 17], [-1] + list(range(16)), z)
        else:
            vf.vf_verify(pair.model, [seq], toks, [0, 17], z)
        torch.cuda.synchronize()
        out.append(z.cpu().numpy())
    assert np.array_equal(out[0], out[1])


def _stable(fn, u):
    """Oracle result, and whether it survives moving every uniform by a relative 1e-6 either way."""
    res = fn(u)
    for f in (1.0 - 1e-6, 1.0 + 1e-6):
        uu = np.minimum(u.astype(np.float64) * f, 1.0 - 2.0 ** -24).astype(np.float32)
        r2 = fn(uu)
        if r2[0] != res[0] or not np.array_equal(r2[1], res[1]):
            return res, False
    return res, True


def test_tree_accept_crafted_logits_bit_exact():
    cfg = wl.scaled(C["tiny_f32"], vocab=256)
    pair = Pair(cfg, max_rows=64, max_positions=256)
    V = cfg.vocab
    seq = pair.new_seq(200)
    rng = np.random.default_rng(21)
    checked = 0
    for case in range(150):
        k = int(rng.integers(0, 33))
        tokens, parents = _random_tree(rng, k, V, branchy=float(rng.choice([0.3, 0.7, 1.0])))
        z = (rng.standard_normal((k + 1, V)) * rng.choice([0.5, 2.0, 6.0])).astype(np.float32)
        yy = z.argmax(-1)
        # let most nodes carry their parent's prediction; duplicate some sibling tokens
        for c in range(1, k + 1):
            r = rng.random()
            if r < 0.6:
                tokens[c] = yy[parents[c]]
            elif r < 0.75:
                sib = [s_ for s_ in children_of(parents, parents[c]) if s_ < c]
                if sib:
                    tokens[c] = tokens[sib[0]]
        vf.vf_seq_set_len(seq, 10)
        tok_dev = i32(tokens)
        if case % 2 == 0:
            want, ok = oracle.tree_greedy_accept(z, tokens, parents), True
            params = [GREEDY]
        else:
            temp = float(rng.choice([0.5, 0.8, 1.3]))
            u = wl.make_uniforms(k + 1, rng)
            want, ok = _stable(lambda uu: oracle.tree_stochastic_accept(z, tokens, parents, uu, temp), u)
            params = [(vf.VF_STOCHASTIC, temp, None, f32(u))]
        n, out, y, path = _gpu_accept_tree(pair, [seq], tok_dev, [0, k + 1], parents, params, f32(z))
        assert np.array_equal(y, want[2]), case
        if ok:
            a = len(want[0]) - 1
            assert n[0] == a and list(path[:a + 1]) == want[0] and np.all(path[a + 1:] == -1), case
            assert np.array_equal(out[:a + 1], want[1]) and np.all(out[a + 1:] == -1), case
            assert vf.vf_seq_get_state(seq) == (10 + 1 + a, int(want[1][-1])), case
            checked += 1
    print(f"tree acceptance: {checked} of 150 seeded cases compared bit-exactly", flush=True)
    assert checked >= 140


def test_tree_argument_errors():
    cfg = wl.scaled(C["tiny_f32"], vocab=256)
    pair = Pair(cfg, max_rows=64, max_positions=256)
    seq = pair.new_seq(100)
    toks = i32([1, 2, 3])
    for bad in ([0, 0, 1], [-1, 1, 0], [-1, 0, 2], [-1, -1, 0]):
        with pytest.raises(vf.VfError) as e:
            vf.vf_verify_tree(pair.model, [seq], toks, [0, 3], bad)
        assert e.value.code == vf.VF_ERR_ARG
    assert vf.vf_seq_get_state(seq)[0] == 0
    z = torch.zeros((3, cfg.vocab), device=DEV)
    with pytest.raises(vf.VfError) as e:
        _gpu_accept_tree(pair, [seq], toks, [0, 3], [-1, 0, 0],
                         [(vf.VF_STOCHASTIC, 0.8, torch.zeros((2, cfg.vocab), device=DEV), f32(np.zeros(6)))], z)
    assert e.value.code == vf.VF_ERR_UNSUPPORTED


def test_greedy_tree_decoding_is_plain_greedy_decoding_on_the_gpu():
    cfg = C["tiny_f32"]
    pair = Pair(cfg, max_rows=64, max_positions=400)
    rng = np.random.default_rng(9)
    ctx = i32(wl.make_context(cfg.vocab, 90, rng))

    def fresh():
        seq = pair.new_seq(300)
        vf.vf_prefill_chunk(pair.model, seq, ctx[:64]); vf.vf_prefill_chunk(pair.model, seq, ctx[64:])
        vf.vf_seq_set_pending(seq, 17)
        return seq

    def step(seq, tokens, parents):
        k = len(tokens) - 1
        tok_dev = i32(tokens)
        vf.vf_verify_tree(pair.model, [seq], tok_dev, [0, k + 1], parents)
        n, out, _, _ = _gpu_accept_tree(pair, [seq], tok_dev, [0, k + 1], parents, [GREEDY])
        return [int(t) for t in out[:n[0] + 1]]

    plain_seq, want = fresh(), []
    while len(want) < 40:
        want += step(plain_seq, [vf.VF_PENDING], [-1])
    seq, got, steps = fresh(), [], 0
    while len(got) < 40:
        k = int(rng.integers(1, 13))
        tokens, parents = _random_tree(rng, k, cfg.vocab)
        tokens[0] = vf.VF_PENDING
        truth, node, d = want[len(got):], 0, 0
        while True:
            ch = children_of(parents, node)
            if not ch or d >= len(truth) or rng.random() < 0.15:
                break
            node = int(rng.choice(ch))
            tokens[node] = truth[d]
            d += 1
        got += step(seq, tokens, parents)
        steps += 1
    print(f"tree decoding: 40 tokens in {steps} steps", flush=True)
    assert got[:40] == want[:40] and steps < 40


@pytest.mark.parametrize("fast", [1, 0])
def test_tree_verify_on_paged_sequences_compacts_across_pages(fast):
    """Two sequences in one pool with shuffled block tables; the contexts end a few rows before a page
    boundary, so the tree's rows and the compaction both straddle pages."""
    cfg = wl.scaled(C["1.5b_k16"], n_layers=2, vocab=4096)
    pair = Pair(cfg, max_rows=128, max_positions=400)
    vf.vf_set_option(pair.model, vf.VF_OPT_FAST_PATH, fast)
    rng = np.random.default_rng(17)
    n_pages = 10
    pool = torch.empty(vf.vf_kv_bytes(pair.model, 64, n_pages), dtype=torch.uint8, device=DEV)
    perm = rng.permutation(n_pages)
    tables, ctxs, ks = [perm[:5], perm[5:]], [120, 61], [20, 9]
    seqs, caches, toks, pars, row_off = [], [], [], [], [0]
    for bt, n_ctx, k in zip(tables, ctxs, ks):
        seq = pair.new_seq(len(bt) * 64, pool=pool, block_table=i32(bt))
        cache = oracle.KVCache(pair.spec, len(bt) * 64)
        pair.prefill_both(seq, cache, wl.make_context(cfg.vocab, n_ctx, rng), 64)
        t, p = _random_tree(rng, k, cfg.vocab)
        seqs.append(seq); caches.append(cache); toks.append(t); pars.append(p)
        row_off.append(row_off[-1] + k + 1)
    rows = row_off[-1]
    parents = [p for ps in pars for p in ps]
    tok_dev = i32(np.concatenate(toks))
    logits = torch.empty((rows, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify_tree(pair.model, seqs, tok_dev, row_off, parents, logits)
    torch.cuda.synchronize()
    z_gpu = logits.cpu().numpy()
    z_or = np.concatenate([oracle.verify_tree(pair.spec, pair.ow, c, t, p) for c, t, p in zip(caches, toks, pars)])
    err = rel_inf(z_gpu, z_or).max()
    print(f"paged tree verify (fast path {fast}): max rel-inf logit error {err:.3e}", flush=True)
    assert err < 2e-2
    # accept along a path planted by hand: logits that make the deepest leaf's root path the greedy walk
    crafted = np.full((rows, cfg.vocab), -5.0, dtype=np.float32)
    want_paths = []
    for b, (t, p) in enumerate(zip(toks, pars)):
        depth = oracle.transformer.tree_depths(p)
        leaf = int(np.argmax(depth))
        path, a = [], leaf
        while a >= 0:
            path.append(a)
            a = p[a]
        path = path[::-1]
        want_paths.append(path)
        for parent, child in zip(path[:-1], path[1:]):
            crafted[row_off[b] + parent, t[child]] = 5.0
            # an earlier sibling with the same token would be taken instead: make those differ
            for sib in children_of(p, parent):
                if sib != child and t[sib] == t[child]:
                    t[sib] = (t[sib] + 1) % cfg.vocab
        crafted[row_off[b] + path[-1], 7] = 5.0
    tok_dev = i32(np.concatenate(toks))
    n_acc, out, y, path = _gpu_accept_tree(pair, seqs, tok_dev, row_off, parents, [GREEDY] * 2, f32(crafted))
    for b, (seq, cache, n_ctx) in enumerate(zip(seqs, caches, ctxs)):
        wp = want_paths[b]
        a = len(wp) - 1
        assert a >= 2 and n_acc[b] == a and list(path[row_off[b]:row_off[b] + a + 1]) == wp
        assert vf.vf_seq_get_state(seq) == (n_ctx + 1 + a, 7)
        oracle.compact(cache, n_ctx, wp)
        for layer in (0, cfg.n_layers - 1):
            (kg, vg), (ko, vo) = pair.kv_both(seq, cache, layer, n_ctx - 3, a + 4)
            assert np.abs(kg - ko).max() <= 1e-2 * np.abs(ko).max() and np.abs(vg - vo).max() <= 1e-2 * np.abs(vo).max()
