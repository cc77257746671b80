"""GPU parity: the HIP path against the CPU oracle, element by element, through the C ABI.

Sizes are chosen so that the oracle finishes in seconds while every kernel still spans
several tiles and a ragged tail: full layer widths of each workload config, fewer layers, a
reduced vocabulary where the full one adds nothing but time.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle.loop import plain_greedy, truncate
import workloads as wl
import paper_2510_15312_amd as vf
from util_oracle import rel_inf
from util_gpu import DEV, Pair, tol_of, i32, f32, gpu_accept, accept_margin_ok, stochastic_margins

pytestmark = pytest.mark.gpu

C = wl.CONFIGS
CASES = {
    # name: (config, context, chunk, k, mode)
    "tiny_f32": (C["tiny_f32"], 512, 128, 4, "greedy"),
    "tiny_f32_ragged": (C["tiny_f32"], 301, 128, 7, "stochastic"),
    "0.5b_shape": (wl.scaled(C["0.5b_k8"], n_layers=2, vocab=4096), 300, 128, 8, "greedy"),
    "1.5b_shape": (wl.scaled(C["1.5b_k16"], n_layers=2, vocab=8192), 333, 256, 16, "stochastic"),
    "3b_shape": (wl.scaled(C["3b_k32"], n_layers=1, vocab=4096), 200, 256, 32, "greedy"),
}


def _check_logits(got, want, tol, what):
    err = rel_inf(np.atleast_2d(got), np.atleast_2d(want)).max()
    print(f"{what}: max rel-inf logit error {err:.3e} (tol {tol:g})", flush=True)
    assert np.isfinite(got).all(), what
    assert err < tol, (what, err)
    return err


@pytest.mark.parametrize("name", list(CASES))
def test_prefill_verify_accept_against_oracle(name):
    cfg, n_ctx, chunk, k, mode = CASES[name]
    print(f"case {name}: ctx {n_ctx} chunk {chunk} k {k} {mode}", flush=True)
    tol = tol_of(cfg)
    pair = Pair(cfg, max_rows=max(chunk, k + 1), max_positions=n_ctx + 4 * (k + 1) + 8)
    s = pair.s
    ctx = wl.make_context(cfg.vocab, n_ctx, s.context)
    cap = n_ctx + 2 * (k + 1)
    cache = oracle.KVCache(pair.spec, cap)
    seq = pair.new_seq(cap)

    # ---- chunked prefill -----------------------------------------------------------------
    z_or, z_gpu = pair.prefill_both(seq, cache, ctx, chunk)
    _check_logits(z_gpu, z_or, tol, "prefill last row")
    assert vf.vf_seq_get_state(seq)[0] == n_ctx
    for layer in (0, cfg.n_layers - 1):
        (kg, vg), (ko, vo) = pair.kv_both(seq, cache, layer, 0, n_ctx)
        kv_tol = 1e-2 if cfg.dtype == "bf16" else 1e-5
        assert np.abs(kg - ko).max() <= kv_tol * np.abs(ko).max(), ("K", layer)
        assert np.abs(vg - vo).max() <= kv_tol * np.abs(vo).max(), ("V", layer)
    pending = oracle.first_token(z_or)

    # ---- drafts: the target's own continuation with one mismatch injected (accepted counts
    #      sweep 0..k), so that acceptance is not vacuous with random weights --------------------
    cont = plain_greedy(pair.spec, pair.ow, cache.clone(), pending, k)
    e = int(s.drafts.integers(1, k + 2))
    drafts = wl.inject_mismatch(cont, e, cfg.vocab, s.drafts)
    q = u = None
    temp = 0.8
    if mode == "stochastic":
        u = wl.make_uniforms(k + 1, s.uniforms)
        qs = s.gumbel.dirichlet(np.full(cfg.vocab, 0.05), size=k).astype(np.float32)
        qs[np.arange(k), drafts] += 0.5
        q = (qs / qs.sum(-1, keepdims=True, dtype=np.float64)).astype(np.float32)

    # ---- verify ----------------------------------------------------------------------------
    z = oracle.verify(pair.spec, pair.ow, cache, pending, drafts)
    tokens = i32(np.concatenate([[pending], drafts]))
    row_off = [0, k + 1]
    logits = torch.empty((k + 1, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify(pair.model, [seq], tokens, row_off, logits)
    torch.cuda.synchronize()
    zg = logits.cpu().numpy()
    err = _check_logits(zg, z, tol, "verify rows")
    if cfg.dtype == "bf16":
        # the same rows through the general (any row count) kernels
        vf.vf_set_option(pair.model, vf.VF_OPT_FAST_PATH, 0)
        logits_gen = torch.empty_like(logits)
        vf.vf_verify(pair.model, [seq], tokens, row_off, logits_gen)
        torch.cuda.synchronize()
        vf.vf_set_option(pair.model, vf.VF_OPT_FAST_PATH, 1)
        _check_logits(logits_gen.cpu().numpy(), z, tol, "verify rows, general kernels")
        # and through the few-row kernels launched one per GEMM instead of the persistent kernel
        vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, 0)
        vf.vf_verify(pair.model, [seq], tokens, row_off, logits_gen)
        torch.cuda.synchronize()
        vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, 1)
        _check_logits(logits_gen.cpu().numpy(), z, tol, "verify rows, one kernel per GEMM")
        print(f"persistent kernel vs one kernel per GEMM: {rel_inf(zg, logits_gen.cpu().numpy()).max():.3e}", flush=True)
        vf.vf_verify(pair.model, [seq], tokens, row_off, logits)
        torch.cuda.synchronize()
        assert np.array_equal(logits.cpu().numpy(), zg), "verify is not bit-reproducible run to run"
        vf.vf_seq_get_state(seq)                         # would report a grid barrier that gave up
    (kg, vg), (ko, vo) = pair.kv_both(seq, cache, cfg.n_layers - 1, n_ctx, k + 1)
    kv_tol = 2e-2 if cfg.dtype == "bf16" else 1e-5
    assert np.abs(kg - ko).max() <= kv_tol * np.abs(ko).max()
    assert np.abs(vg - vo).max() <= kv_tol * np.abs(vo).max()

    # ---- accept, tier 1: same logits on both sides -> bit-exact -------------------------------
    z32 = z.astype(np.float32)
    if mode == "greedy":
        a_or, out_or, y_or = oracle.greedy_accept(z32, drafts)
        params = [(vf.VF_GREEDY, 0.0, None, None)]
    else:
        a_or, out_or, y_or = oracle.stochastic_accept(z32, drafts, q, u, temp)
        params = [(vf.VF_STOCHASTIC, temp, f32(q), f32(u))]
    n_acc, out, y = gpu_accept(pair, [seq], tokens, row_off, params, logits=f32(z32))
    assert np.array_equal(y, y_or)
    if accept_margin_ok(z32, drafts, mode, q, u, temp, 1e-9):
        assert n_acc[0] == a_or
        assert np.array_equal(out[:a_or + 1], out_or) and np.all(out[a_or + 1:] == -1)
        ln, pend = vf.vf_seq_get_state(seq)
        assert ln == n_ctx + 1 + a_or and pend == out_or[-1]
    else:
        print("tier-1 decision inside the 1e-9 margin: screened", flush=True)

    # ---- accept, tier 2: the GPU's own logits; oracle rule applied to them must agree, and
    #      where the oracle's margins exceed the logit error the oracle's own result too -------
    vf.vf_seq_set_len(seq, n_ctx)
    if mode == "greedy":
        a2, out2, y2 = oracle.greedy_accept(zg, drafts)
    else:
        a2, out2, y2 = oracle.stochastic_accept(zg, drafts, q, u, temp)
    n_acc, out, y = gpu_accept(pair, [seq], tokens, row_off, params, logits=None)
    assert np.array_equal(y, y2)
    if accept_margin_ok(zg, drafts, mode, q, u, temp, 1e-9):
        assert n_acc[0] == a2 and np.array_equal(out[:a2 + 1], out2)
    if mode == "greedy" and accept_margin_ok(z32, drafts, mode, q, u, temp, 2 * err):
        assert n_acc[0] == a_or and np.array_equal(out[:a_or + 1], out_or)
        print(f"tier-2 direct: accepted {a_or} of {k} (mismatch injected at {e})", flush=True)
    if mode == "stochastic":
        _, safe, draw_safe = stochastic_margins(z32, drafts, q, u, temp, 2 * np.abs(zg - z).max())
        if safe:
            assert n_acc[0] == a_or and np.array_equal(out[:a_or], out_or[:a_or])
        if draw_safe:
            assert out[a_or] == out_or[-1]
        print(f"tier-2 direct (stochastic): accepted {a_or} of {k}; decisions safe {safe}, draw safe {draw_safe}", flush=True)


@pytest.mark.parametrize("persistent", [1, 0])
def test_verify_repeats_bit_exactly(persistent):
    """Both few-row paths exchange partial results between workgroups through memory (split-K
    tiles; the persistent kernel everything behind its grid barriers).  Two different inputs are
    verified in turn, many times: every result must equal the first result for that input bit
    for bit -- a read that returns what an earlier launch or phase left in a buffer shows up as a
    differing run -- and must agree with the other path; no barrier may give up."""
    cfg = wl.scaled(C["1.5b_k16"], n_layers=8, vocab=8192)
    k, n_ctx, reps = 16, 700, int(__import__('os').environ.get('VF_REPS', '500'))
    pair = Pair(cfg, max_rows=256, max_positions=n_ctx + 64)
    seq = pair.new_seq(n_ctx + 64)
    toks = i32(wl.make_context(cfg.vocab, n_ctx, pair.s.context))
    for c0 in range(0, n_ctx, 256):
        vf.vf_prefill_chunk(pair.model, seq, toks[c0:c0 + 256])
    inputs = [i32(wl.make_context(cfg.vocab, k + 1, pair.s.drafts)) for _ in range(2)]
    new = lambda: torch.empty((k + 1, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, 1 - persistent)
    ref = []
    for rows in inputs:                                   # the other path: a yardstick
        out = new()
        vf.vf_verify(pair.model, [seq], rows, [0, k + 1], out)
        ref.append(out)
    vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, persistent)
    first, differing = [None, None], []
    again = new()
    for rep in range(reps):
        for j, rows in enumerate(inputs):
            vf.vf_verify(pair.model, [seq], rows, [0, k + 1], again)
            if first[j] is None:
                first[j] = again.clone()
                err = rel_inf(again.cpu().numpy(), ref[j].cpu().numpy()).max()
                print(f"persistent={persistent}: input {j}, first run vs the other path: {err:.3e}", flush=True)
                assert err < 2e-2
            elif not torch.equal(first[j], again):
                differing.append((rep, j, int((first[j] != again).sum()), float((first[j] - again).abs().max())))
    assert vf.vf_seq_get_state(seq)[0] == n_ctx            # also reports a grid barrier that gave up
    print(f"persistent={persistent}: {len(differing)} of {2 * reps - 2} repeats differ {differing[:6]}", flush=True)
    assert not differing
