"""GPU parity at the full sizes of the workload configs (the launch configuration bench.py times).

The 0.5B and 1.5B shapes are checked element by element against the oracle run at full size.
For the 28-layer 1.5B model the oracle accumulates in float32, the precision the workload config
fixes ("bf16 weights/activations with fp32 accumulate"): at that depth, with random weights, the
logit metric is dominated by chaotic amplification of bfloat16 rounding flips -- the oracle run in
float32 and in float64 on these very inputs differs from itself by 1.4e-2 (last prefill row) and
1.6e-2 to 1.8e-2 (the 17 verify rows), so the stated 2e-2 bar sits at the noise floor; a 6-layer
model of the same widths measures the GPU's error against both oracle precisions where that noise
does not dominate.  The 3B shape is checked element by element against the oracle at its full
widths, vocabulary, context and row count with two layers, and at its full depth, where the oracle
would take minutes, through properties that hold at any size: a multi-row verify equals successive
single-row decodes, and greedy acceptance of the target's own continuation accepts every draft.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle.loop import truncate
import workloads as wl
import paper_2510_15312_amd as vf
from util_oracle import rel_inf, spec_of, weights_of
from util_gpu import DEV, Pair, i32, f32, gpu_accept, accept_margin_ok, stochastic_margins

pytestmark = pytest.mark.gpu
C = wl.CONFIGS


def test_config2_full_size_greedy_verify():
    cfg = C["0.5b_k8"]
    k = cfg.k
    pair = Pair(cfg, max_rows=cfg.chunk, max_positions=cfg.ctx + 64)
    s = pair.s
    ctx = wl.make_context(cfg.vocab, cfg.ctx, s.context)
    cache, seq = oracle.KVCache(pair.spec, cfg.ctx + 32), pair.new_seq(cfg.ctx + 32)
    z_or, z_gpu = pair.prefill_both(seq, cache, ctx, cfg.chunk)
    err = rel_inf(z_gpu[None], z_or[None]).max()
    print(f"0.5b full size: prefill last-row error {err:.3e}", flush=True)
    assert err < 2e-2
    pending = oracle.first_token(z_or)
    for attempt, drafts in enumerate([wl.copy_span_drafts(ctx, k, cfg.p_copy, cfg.vocab, s.drafts),
                                      None]):
        if drafts is None:      # supplementary drafts: the target's own continuation, one mismatch
            c2 = cache.clone()
            cont = oracle.loop.plain_greedy(pair.spec, pair.ow, c2, pending, k)
            drafts = wl.inject_mismatch(cont, 6, cfg.vocab, s.drafts)
        z = oracle.verify(pair.spec, pair.ow, cache, pending, drafts)
        truncate(cache, cfg.ctx)
        tokens = i32(np.concatenate([[pending], drafts]))
        logits = torch.empty((k + 1, cfg.vocab), dtype=torch.float32, device=DEV)
        vf.vf_verify(pair.model, [seq], tokens, [0, k + 1], logits)
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        err = rel_inf(zg, z).max()
        print(f"0.5b full size: verify error {err:.3e}", flush=True)
        assert err < 2e-2
        a_or, out_or, y_or = oracle.greedy_accept(z, drafts)
        n_acc, out, y = gpu_accept(pair, [seq], tokens, [0, k + 1], [(vf.VF_GREEDY, 0.0, None, None)])
        a2, out2, y2 = oracle.greedy_accept(zg, drafts)
        assert np.array_equal(y, y2) and n_acc[0] == a2 and np.array_equal(out[:a2 + 1], out2)
        if accept_margin_ok(z.astype(np.float32), drafts, "greedy", None, None, 1.0, 2 * err):
            assert n_acc[0] == a_or and np.array_equal(out[:a_or + 1], out_or)
            print(f"0.5b full size: direct match, accepted {a_or} of {k}", flush=True)
        vf.vf_seq_set_len(seq, cfg.ctx)


def test_config3_full_size_stochastic_steps():
    """1.5B shape, context 2048 in 256-token chunks, successive k=16 stochastic steps with a dense
    draft distribution; every step is teacher-forced from the oracle's trajectory."""
    cfg = C["1.5b_k16"]
    k, m, n_steps = cfg.k, cfg.k + 1, 8
    dt = np.float32          # the accumulation precision the config fixes; see the module docstring
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights)
    spec, ow = spec_of(cfg), weights_of(wd, dt)
    cap = cfg.ctx + (n_steps + 1) * m
    model = vf.vf_model_create(vf.config_from(cfg, cfg.chunk, cap), vf.upload_weights(wd, cfg.dtype, DEV), DEV)
    seq = vf.vf_seq_create(model, cap)
    ctx = wl.make_context(cfg.vocab, cfg.ctx, s.context)
    cache = oracle.KVCache(spec, cap, dt)
    print("1.5b full size: oracle prefill ...", flush=True)
    z_last = oracle.prefill(spec, ow, cache, ctx, cfg.chunk, dt)
    toks = i32(ctx)
    out = torch.empty(cfg.vocab, dtype=torch.float32, device=DEV)
    for c0 in range(0, cfg.ctx, cfg.chunk):
        last = c0 + cfg.chunk >= cfg.ctx
        vf.vf_prefill_chunk(model, seq, toks[c0:c0 + cfg.chunk], logits_mode=1 if last else 0,
                            logits_out=out if last else None)
    torch.cuda.synchronize()
    err = rel_inf(out.cpu().numpy()[None], z_last[None]).max()
    print(f"1.5b full size: prefill last-row error {err:.3e}", flush=True)
    assert err < 2e-2

    def import_cache(t0, t1):
        """The oracle's K and V for positions [t0, t1) of every layer replace the GPU's: the verify
        steps then start from the same cache on both sides, and what is measured is the verify
        step alone rather than it plus the drift the two prefills accumulated."""
        for layer in range(cfg.n_layers):
            ko = np.ascontiguousarray(cache.k[layer, :, t0:t1].transpose(1, 0, 2), dtype=np.float32)
            vo = np.ascontiguousarray(cache.v[layer, :, t0:t1].transpose(1, 0, 2), dtype=np.float32)
            vf.vf_kv_write(model, seq, layer, t0, f32(ko), f32(vo))
        torch.cuda.synchronize()
    import_cache(0, cfg.ctx)
    (kg, vg), _ = (vf.vf_kv_read(model, seq, 5, 100, 8), None)
    assert np.array_equal(kg.cpu().numpy(), cache.k[5, :, 100:108].transpose(1, 0, 2).astype(np.float32))
    assert np.array_equal(vg.cpu().numpy(), cache.v[5, :, 100:108].transpose(1, 0, 2).astype(np.float32))
    u0 = wl.make_uniforms(1, s.uniforms)
    pending = oracle.first_token(z_last, cfg.temperature, u0[1])
    worst, decisions, screened, asserted = 0.0, 0, 0, 0
    pair = type("P", (), {"model": model})
    for step in range(n_steps):
        scratch = cache.clone()

        def next_logits(tok, scratch=scratch):
            return oracle.forward(spec, ow, scratch, [tok], dt)[0]
        drafts, q = wl.gumbel_drafts(next_logits, pending, k, cfg.temperature, 0.5, s.gumbel, s.drafts)
        u = wl.make_uniforms(m, s.uniforms)
        ln = cache.len
        z = oracle.verify(spec, ow, cache, pending, drafts, dt)
        a_or, out_or, y_or = oracle.stochastic_accept(z, drafts, q, u, cfg.temperature)
        truncate(cache, ln + 1 + a_or)
        if step:
            import_cache(ln_prev, ln)                    # the rows the previous step kept
        ln_prev = ln
        tokens = i32(np.concatenate([[pending], drafts]))
        logits = torch.empty((m, cfg.vocab), dtype=torch.float32, device=DEV)
        vf.vf_seq_set_len(seq, ln)                       # teacher forcing: the oracle's state
        vf.vf_set_option(model, vf.VF_OPT_PERSISTENT, 0)  # one kernel per GEMM: logits only
        vf.vf_verify(model, [seq], tokens, [0, m], logits)
        torch.cuda.synchronize()
        errs_c = rel_inf(logits.cpu().numpy(), z)
        worst = max(worst, errs_c.max())
        vf.vf_set_option(model, vf.VF_OPT_PERSISTENT, 1)  # the persistent kernel (the default): acceptance runs on these logits
        vf.vf_verify(model, [seq], tokens, [0, m], logits)
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        errs = rel_inf(zg, z)
        err = errs.max()
        worst = max(worst, err)
        print(f"1.5b full size: step {step}: row errors mean {errs.mean():.3e} max {err:.3e} "
              f"(one kernel per GEMM: mean {errs_c.mean():.3e} max {errs_c.max():.3e})", flush=True)
        params = [(vf.VF_STOCHASTIC, cfg.temperature, f32(q), f32(u))]
        n_acc, out_t, y = gpu_accept(pair, [seq], tokens, [0, m], params)
        a2, out2, y2 = oracle.stochastic_accept(zg, drafts, q, u, cfg.temperature)
        assert np.array_equal(y, y2)
        if accept_margin_ok(zg, drafts, "stochastic", q, u, cfg.temperature, 1e-9):
            assert n_acc[0] == a2 and np.array_equal(out_t[:a2 + 1], out2)
        # directly against the oracle's trajectory: where no decision of the oracle can flip under
        # twice the measured logit error, counts and accepted ids must be the oracle's
        _, safe, draw_safe = stochastic_margins(z, drafts, q, u, cfg.temperature, 2 * np.abs(zg - z).max())
        decisions += 1
        if safe:
            assert n_acc[0] == a_or and np.array_equal(out_t[:a_or], out_or[:a_or]), (step, n_acc[0], a_or)
            asserted += 1
        if draw_safe:
            assert out_t[a_or] == out_or[-1], step
        if n_acc[0] != a_or:
            screened += 1                                # only possible inside the margin (asserted above)
        print(f"1.5b full size: step {step}: oracle accepted {a_or}, gpu {n_acc[0]}; decisions safe: {safe}", flush=True)
        pending = int(out_or[-1])
    print(f"1.5b full size: worst logit error {worst:.3e}; steps {decisions}, compared directly {asserted}, "
          f"differing accept counts inside the margin {screened}", flush=True)
    assert worst < 2e-2
    assert asserted >= 1


def test_config3_widths_depth6_error_against_both_oracle_precisions():
    """What the 28-layer comparison cannot tell apart from noise, measured where noise does not
    dominate: full 1.5B widths and vocabulary, context 2048 in 256-token chunks, 6 layers, 17 verify
    rows, prefill and verify together (no cache import).  The oracle in float64 is the truth; the
    oracle accumulating in float32 is what exact arithmetic at the precision the config fixes
    ("fp32 accumulate") gives.  The GPU's error against the truth may not exceed the float32
    oracle's own error by more than a quarter (row mean; half for the worst row)."""
    cfg = wl.scaled(C["1.5b_k16"], n_layers=6)
    k, m = cfg.k, cfg.k + 1
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights)
    spec = spec_of(cfg)
    ctx = wl.make_context(cfg.vocab, cfg.ctx, s.context)
    drafts = wl.copy_span_drafts(ctx, k, 1.0, cfg.vocab, s.drafts)
    z_last, z_ver = {}, {}
    for dt in (np.float64, np.float32):
        ow = weights_of(wd, dt)
        cache = oracle.KVCache(spec, cfg.ctx + m, dt)
        z_last[dt] = oracle.prefill(spec, ow, cache, ctx, cfg.chunk, dt)
        if dt is np.float64:
            pending = oracle.first_token(z_last[dt])
        z_ver[dt] = oracle.verify(spec, ow, cache, pending, drafts, dt)
        del ow, cache
        print(f"depth 6: oracle in {np.dtype(dt).name} done", flush=True)
    model = vf.vf_model_create(vf.config_from(cfg, cfg.chunk, cfg.ctx + 2 * m), vf.upload_weights(wd, cfg.dtype, DEV), DEV)
    del wd
    seq = vf.vf_seq_create(model, cfg.ctx + 2 * m)
    toks = i32(ctx)
    out = torch.empty(cfg.vocab, dtype=torch.float32, device=DEV)
    for c0 in range(0, cfg.ctx, cfg.chunk):
        last = c0 + cfg.chunk >= cfg.ctx
        vf.vf_prefill_chunk(model, seq, toks[c0:c0 + cfg.chunk], logits_mode=1 if last else 0,
                            logits_out=out if last else None)
    tokens = i32(np.concatenate([[pending], drafts]))
    logits = torch.empty((m, cfg.vocab), dtype=torch.float32, device=DEV)
    ref32 = rel_inf(z_ver[np.float32], z_ver[np.float64])
    ref32_last = rel_inf(z_last[np.float32][None], z_last[np.float64][None]).max()
    e_last = rel_inf(out.cpu().numpy()[None], z_last[np.float64][None]).max()
    print(f"depth 6: last prefill row: gpu {e_last:.3e}, float32 oracle {ref32_last:.3e}", flush=True)
    assert e_last < 2e-2
    for persistent in (1, 0):
        vf.vf_set_option(model, vf.VF_OPT_PERSISTENT, persistent)
        vf.vf_verify(model, [seq], tokens, [0, m], logits)
        torch.cuda.synchronize()
        e = rel_inf(logits.cpu().numpy(), z_ver[np.float64])
        print(f"depth 6: verify rows ({'persistent kernel' if persistent else 'one kernel per GEMM'}): gpu mean {e.mean():.3e} "
              f"max {e.max():.3e}; float32 oracle mean {ref32.mean():.3e} max {ref32.max():.3e}", flush=True)
        assert e.max() < 2e-2
        assert e.mean() <= 1.25 * ref32.mean(), (e.mean(), ref32.mean())
        assert e.max() <= 1.5 * ref32.max(), (e.max(), ref32.max())


def test_config4_widths_against_oracle():
    """3B widths (d 3072, 24/8 heads, ffn 8192), the full 128256 vocabulary, context 4096 in
    256-token chunks, 33 verify rows, two layers, against the oracle element by element: the
    persistent kernel here stages its activations in K slices and shares the keys of a block out
    over several workgroups, and the prefill attention merges key parts with its second kernel."""
    cfg = wl.scaled(C["3b_k32"], n_layers=2)
    k, m = cfg.k, cfg.k + 1
    pair = Pair(cfg, max_rows=cfg.chunk, max_positions=cfg.ctx + 2 * m)
    s = pair.s
    ctx = wl.make_context(cfg.vocab, cfg.ctx, s.context)
    cache, seq = oracle.KVCache(pair.spec, cfg.ctx + m), pair.new_seq(cfg.ctx + 2 * m)
    z_or, z_gpu = pair.prefill_both(seq, cache, ctx, cfg.chunk)
    err = rel_inf(z_gpu[None], z_or[None]).max()
    (kg, vg), (ko, vo) = pair.kv_both(seq, cache, cfg.n_layers - 1, 0, cfg.ctx)
    ek, ev = np.abs(kg - ko).max() / np.abs(ko).max(), np.abs(vg - vo).max() / np.abs(vo).max()
    print(f"3b widths: prefill last-row error {err:.3e}, last-layer K {ek:.2e}, V {ev:.2e}", flush=True)
    assert err < 2e-2 and ek <= 1e-2 and ev <= 1e-2
    pending = oracle.first_token(z_or)
    cont = oracle.loop.plain_greedy(pair.spec, pair.ow, cache.clone(), pending, k)
    drafts = wl.inject_mismatch(cont, 23, cfg.vocab, s.drafts)
    z = oracle.verify(pair.spec, pair.ow, cache, pending, drafts)
    tokens = i32(np.concatenate([[pending], drafts]))
    logits = torch.empty((m, cfg.vocab), dtype=torch.float32, device=DEV)
    a_or, out_or, y_or = oracle.greedy_accept(z.astype(np.float32), drafts)
    greedy = [(vf.VF_GREEDY, 0.0, None, None)]
    for name, fast, persistent in (("persistent kernel", 1, 1), ("one kernel per GEMM", 1, 0), ("general kernels", 0, 1)):
        vf.vf_set_option(pair.model, vf.VF_OPT_FAST_PATH, fast)
        vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, persistent)
        vf.vf_seq_set_len(seq, cfg.ctx)
        vf.vf_verify(pair.model, [seq], tokens, [0, m], logits)
        torch.cuda.synchronize()
        zg = logits.cpu().numpy()
        errs = rel_inf(zg, z)
        print(f"3b widths: 33 verify rows, {name}: error mean {errs.mean():.3e} max {errs.max():.3e}", flush=True)
        assert np.isfinite(zg).all() and errs.max() < 2e-2
        (kg, vg), (ko, vo) = pair.kv_both(seq, cache, cfg.n_layers - 1, cfg.ctx, m)
        assert np.abs(kg - ko).max() <= 2e-2 * np.abs(ko).max() and np.abs(vg - vo).max() <= 2e-2 * np.abs(vo).max()
        n_acc, out, y = gpu_accept(pair, [seq], tokens, [0, m], greedy)
        a2, out2, y2 = oracle.greedy_accept(zg, drafts)
        assert np.array_equal(y, y2) and n_acc[0] == a2 and np.array_equal(out[:a2 + 1], out2)
        if accept_margin_ok(z.astype(np.float32), drafts, "greedy", None, None, 1.0, 2 * errs.max()):
            assert n_acc[0] == a_or and np.array_equal(out[:a_or + 1], out_or)
            print(f"3b widths: {name}: direct match with the oracle, accepted {a_or} of {k}", flush=True)
    vf.vf_set_option(pair.model, vf.VF_OPT_FAST_PATH, 1)
    vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, 1)
    vf.vf_seq_get_state(seq)                             # would report a grid barrier that gave up


def test_config4_full_size_properties():
    """3B shape, context 4096, k = 32 (33 rows): properties that need no oracle."""
    cfg = C["3b_k32"]
    k, m = cfg.k, cfg.k + 1
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights)
    cap = cfg.ctx + 2 * m
    model = vf.vf_model_create(vf.config_from(cfg, cfg.chunk, cap), vf.upload_weights(wd, cfg.dtype, DEV), DEV)
    del wd
    seq = vf.vf_seq_create(model, cap)
    ctx = wl.make_context(cfg.vocab, cfg.ctx, s.context)
    toks = i32(ctx)
    print("3b full size: prefill ...", flush=True)
    for c0 in range(0, cfg.ctx, cfg.chunk):
        vf.vf_prefill_chunk(model, seq, toks[c0:c0 + cfg.chunk], sample_first=c0 + cfg.chunk >= cfg.ctx)
    ln, pending = vf.vf_seq_get_state(seq)
    assert ln == cfg.ctx
    # greedy continuation by single-row steps (verify with no drafts + accept = plain decoding)
    n_acc = torch.zeros(1, dtype=torch.int32, device=DEV)
    out_t = torch.zeros(m, dtype=torch.int32, device=DEV)
    y_t = torch.zeros(m, dtype=torch.int32, device=DEV)
    single = torch.empty((m, cfg.vocab), dtype=torch.float32, device=DEV)
    cont, tok = [], pending
    for i in range(m):
        t = i32([tok])
        vf.vf_verify(model, [seq], t, [0, 1], single[i:i + 1])
        vf.vf_accept(model, [seq], t, [0, 1], [(vf.VF_GREEDY, 0.0, None, None)], n_acc, out_t, y_t)
        tok = int(out_t[0].item())
        cont.append(tok)
    assert vf.vf_seq_get_state(seq)[0] == cfg.ctx + m
    # the same rows in one verify: logits of row i must match the i-th single-row decode
    vf.vf_seq_set_len(seq, cfg.ctx)
    drafts = cont[:k]
    tokens = i32([pending] + drafts)
    multi = torch.empty((m, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify(model, [seq], tokens, [0, m], multi)
    torch.cuda.synchronize()
    err = rel_inf(multi.cpu().numpy(), single.cpu().numpy()).max()
    print(f"3b full size: 33-row verify vs 33 single-row decodes: {err:.3e}", flush=True)
    # both sides are GPU results, each allowed 2e-2 against the exact model: 4e-2 between them
    assert err < 4e-2
    # greedy speculative step on the target's own continuation: all accepted (up to logit ties)
    vf.vf_accept(model, [seq], tokens, [0, m], [(vf.VF_GREEDY, 0.0, None, None)], n_acc, out_t, y_t)
    torch.cuda.synchronize()
    a = int(n_acc.item())
    y = y_t.cpu().numpy()
    zs = single.cpu().numpy()
    first_diff = next((i for i in range(k) if y[i] != drafts[i]), k)
    assert a == first_diff
    if a < k:   # a flip is only allowed where the top-2 gap is within the logit error
        top2 = np.partition(zs[a], -2)[-2:]
        assert top2[1] - top2[0] <= 2 * err * np.abs(zs[a]).max(), (a, top2)
    print(f"3b full size: accepted {a} of {k} drafts from the target's own continuation", flush=True)
    assert vf.vf_seq_get_state(seq)[0] == cfg.ctx + 1 + a


def test_config3_full_size_tree_properties():
    """1.5B shape at full size, context 2048: properties of the tree verify that hold at any size.
    A chain is the plain verify bit for bit; a node of a random tree gets the logits that a plain
    verify of its root path gives to the path's last row (both are GPU results, each allowed 2e-2
    against the exact model); after acceptance along a planted path the compacted cache continues
    like the cache of that plain verify."""
    cfg = C["1.5b_k16"]
    k, m = cfg.k, cfg.k + 1
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights)
    cap = cfg.ctx + 4 * m
    model = vf.vf_model_create(vf.config_from(cfg, cfg.chunk, cap), vf.upload_weights(wd, cfg.dtype, DEV), DEV)
    del wd
    seq = vf.vf_seq_create(model, cap)
    toks_ctx = i32(wl.make_context(cfg.vocab, cfg.ctx, s.context))
    print("1.5b full size tree: prefill ...", flush=True)
    for c0 in range(0, cfg.ctx, cfg.chunk):
        vf.vf_prefill_chunk(model, seq, toks_ctx[c0:c0 + cfg.chunk])
    rng = np.random.default_rng(33)
    tokens = rng.integers(0, cfg.vocab, m).astype(np.int32)
    tok_dev = i32(tokens)

    def run(fn):
        z = torch.empty((m, cfg.vocab), dtype=torch.float32, device=DEV)
        vf.vf_seq_set_len(seq, cfg.ctx)
        fn(z)
        torch.cuda.synchronize()
        return z.cpu().numpy()

    plain = run(lambda z: vf.vf_verify(model, [seq], tok_dev, [0, m], z))
    chain = run(lambda z: vf.vf_verify_tree(model, [seq], tok_dev, [0, m], [-1] + list(range(k)), z))
    assert np.array_equal(plain, chain)
    parents = [-1] + [i - 1 if rng.random() > 0.5 else int(rng.integers(0, i)) for i in range(1, m)]
    tree = run(lambda z: vf.vf_verify_tree(model, [seq], tok_dev, [0, m], parents, z))
    depth = [0] * m
    for i in range(1, m):
        depth[i] = depth[parents[i]] + 1
    worst = 0.0
    for leaf in (int(np.argmax(depth)), m - 1):
        path, a = [], leaf
        while a >= 0:
            path.append(a)
            a = parents[a]
        path = path[::-1]
        pt = i32(tokens[path])
        zp = torch.empty((len(path), cfg.vocab), dtype=torch.float32, device=DEV)
        vf.vf_seq_set_len(seq, cfg.ctx)
        vf.vf_verify(model, [seq], pt, [0, len(path)], zp)
        torch.cuda.synchronize()
        err = rel_inf(tree[path], zp.cpu().numpy()).max()
        worst = max(worst, err)
        print(f"1.5b full size tree: path of depth {len(path) - 1} to row {leaf}: tree vs plain verify {err:.3e}", flush=True)
        assert err < 4e-2
    # acceptance along the deepest path (crafted logits), compaction, then one more plain step:
    # its logits must match the same step taken after a plain verify + accept of that path
    leaf = int(np.argmax(depth))
    path, a = [], leaf
    while a >= 0:
        path.append(a)
        a = parents[a]
    path = path[::-1]
    crafted = np.full((m, cfg.vocab), -5.0, dtype=np.float32)
    tk = tokens.copy()
    for parent, child in zip(path[:-1], path[1:]):
        crafted[parent, tk[child]] = 5.0
        for sib in range(1, m):
            if parents[sib] == parent and sib != child and tk[sib] == tk[child]:
                tk[sib] = (tk[sib] + 1) % cfg.vocab
    crafted[path[-1], 11] = 5.0
    n_acc = torch.zeros(1, dtype=torch.int32, device=DEV)
    o_t, y_t, p_t = (torch.zeros(m, dtype=torch.int32, device=DEV) for _ in range(3))
    greedy = [(vf.VF_GREEDY, 0.0, None, None)]
    nxt = i32([vf.VF_PENDING, 5, 6, 7])
    after = []
    for use_tree in (True, False):
        vf.vf_seq_set_len(seq, cfg.ctx)
        if use_tree:
            vf.vf_verify_tree(model, [seq], i32(tk), [0, m], parents)
            vf.vf_accept_tree(model, [seq], i32(tk), [0, m], parents, greedy, n_acc, o_t, y_t, p_t, f32(crafted))
            assert int(n_acc.item()) == len(path) - 1 and p_t.cpu().tolist()[:len(path)] == path
        else:
            pt = i32(tk[path])
            vf.vf_verify(model, [seq], pt, [0, len(path)])
            vf.vf_accept(model, [seq], pt, [0, len(path)], greedy, n_acc, o_t[:len(path)], y_t[:len(path)],
                         f32(crafted[path]))
            assert int(n_acc.item()) == len(path) - 1
        assert vf.vf_seq_get_state(seq) == (cfg.ctx + len(path), 11)
        z = torch.empty((4, cfg.vocab), dtype=torch.float32, device=DEV)
        vf.vf_verify(model, [seq], nxt, [0, 4], z)
        torch.cuda.synchronize()
        after.append(z.cpu().numpy())
    err = rel_inf(after[0], after[1]).max()
    print(f"1.5b full size tree: next step on the compacted cache vs on the plain cache {err:.3e}", flush=True)
    assert err < 4e-2
