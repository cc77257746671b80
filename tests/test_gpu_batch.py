"""GPU parity of the batched, ragged, paged verify step (the RAG-mix workload) and of the
invariants the paper states, on the GPU itself.

The batched mix keeps the 1.5B layer widths, 64-token pages, a block table that is a random
permutation of the pool, ragged draft lengths and mixed greedy / stochastic acceptance; layers,
vocabulary and context lengths are reduced so that the oracle finishes in seconds.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle.loop import plain_greedy, truncate
import workloads as wl
import paper_2510_15312_amd as vf
from util_oracle import rel_inf
from util_gpu import DEV, Pair, i32, f32, accept_margin_ok, stochastic_margins

pytestmark = pytest.mark.gpu
C = wl.CONFIGS


def _paged_setup(pair, cfg, mix, check_kv=False):
    """Pool + one paged sequence per entry of the mix, prefilled on both sides."""
    pool = torch.empty(vf.vf_kv_bytes(pair.model, 64, mix.n_pages), dtype=torch.uint8, device=DEV)
    seqs, caches, pendings, ctxs = [], [], [], []
    for b in range(len(mix.ctx)):
        n_ctx, k = int(mix.ctx[b]), int(mix.k[b])
        cap = len(mix.block_tables[b]) * 64
        bt = i32(mix.block_tables[b])
        seq = pair.new_seq(cap, pool=pool, block_table=bt)
        cache = oracle.KVCache(pair.spec, n_ctx + k + 1)
        ctx = wl.make_context(cfg.vocab, n_ctx, pair.s.context)
        z_or, z_gpu = pair.prefill_both(seq, cache, ctx, cfg.chunk)
        assert rel_inf(z_gpu[None], z_or[None]).max() < 2e-2, b
        if check_kv:   # the deepest layer's K/V carry every attention pass below it
            (kg, vg), (ko, vo) = pair.kv_both(seq, cache, cfg.n_layers - 1, 0, n_ctx)
            ek, ev = np.abs(kg - ko).max() / np.abs(ko).max(), np.abs(vg - vo).max() / np.abs(vo).max()
            print(f"sequence {b}: context {n_ctx}: prefill last-row error "
                  f"{rel_inf(z_gpu[None], z_or[None]).max():.3e}, K {ek:.2e}, V {ev:.2e}", flush=True)
            assert ek <= 1e-2 and ev <= 1e-2, (b, ek, ev)
        seqs.append(seq)
        caches.append(cache)
        ctxs.append(ctx)
        pendings.append(oracle.first_token(z_or))
    return pool, seqs, caches, pendings, ctxs


def _run_mix(cfg, mix, expect_fast, persistent=True, check_kv=False):
    total = int(np.sum(mix.k + 1))
    pair = Pair(cfg, max_rows=max(cfg.chunk, total), max_positions=int(mix.ctx.max()) + 64 + 64)
    s = pair.s
    assert vf.lib.vf_set_option(pair.model.handle, vf.VF_OPT_FAST_PATH, 1) == 0
    vf.vf_set_option(pair.model, vf.VF_OPT_PERSISTENT, int(persistent))
    pool, seqs, caches, pendings, ctxs = _paged_setup(pair, cfg, mix, check_kv)
    B = len(seqs)
    temp = cfg.temperature
    # inputs per sequence: the target's own continuation with one mismatch; stochastic sequences
    # carry uniforms; one of them a dense draft distribution, the others a deterministic drafter
    tokens, row_off, params, per_seq = [], [0], [], []
    dense_done = False
    for b in range(B):
        k = int(mix.k[b])
        if k:
            cont = plain_greedy(pair.spec, pair.ow, caches[b].clone(), pendings[b], k)
            drafts = wl.inject_mismatch(cont, int(s.drafts.integers(1, k + 2)), cfg.vocab, s.drafts)
        else:
            drafts = np.zeros(0, dtype=np.int64)          # no drafts: the step is one plain decoding step
        q = u = None
        if mix.stochastic[b]:
            u = wl.make_uniforms(k + 1, s.uniforms)
            if not dense_done and k:
                qs = s.gumbel.dirichlet(np.full(cfg.vocab, 0.05), size=k).astype(np.float32)
                qs[np.arange(k), drafts] += 0.5
                q = (qs / qs.sum(-1, keepdims=True, dtype=np.float64)).astype(np.float32)
                dense_done = True
            params.append((vf.VF_STOCHASTIC, temp, None if q is None else f32(q), f32(u)))
        else:
            params.append((vf.VF_GREEDY, 0.0, None, None))
        tokens += [pendings[b]] + [int(t) for t in drafts]
        row_off.append(row_off[-1] + k + 1)
        per_seq.append((drafts, q, u))
    tok_dev = i32(tokens)
    logits = torch.empty((total, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify(pair.model, seqs, tok_dev, row_off, logits)
    n_acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    out = torch.full((total,), -7, dtype=torch.int32, device=DEV)
    y = torch.full((total,), -7, dtype=torch.int32, device=DEV)
    vf.vf_accept(pair.model, seqs, tok_dev, row_off, params, n_acc, out, y)
    torch.cuda.synchronize()
    zg, n_acc, out, y = logits.cpu().numpy(), n_acc.cpu().numpy(), out.cpu().numpy(), y.cpu().numpy()
    worst, direct = 0.0, 0
    for b in range(B):
        drafts, q, u = per_seq[b]
        k, r0, r1 = len(drafts), row_off[b], row_off[b + 1]
        z = oracle.verify(pair.spec, pair.ow, caches[b], pendings[b], drafts)
        err = rel_inf(zg[r0:r1], z).max()
        worst = max(worst, err)
        assert err < 2e-2, (b, err)
        mode = "stochastic" if mix.stochastic[b] else "greedy"
        if mode == "greedy":
            a2, out2, y2 = oracle.greedy_accept(zg[r0:r1], drafts)
        else:
            a2, out2, y2 = oracle.stochastic_accept(zg[r0:r1], drafts, q, u, temp)
        assert np.array_equal(y[r0:r1], y2), b
        if accept_margin_ok(zg[r0:r1], drafts, mode, q, u, temp, 1e-9):
            assert n_acc[b] == a2 and np.array_equal(out[r0:r0 + a2 + 1], out2), (b, mode)
            assert np.all(out[r0 + a2 + 1:r1] == -1)
            ln, pend = vf.vf_seq_get_state(seqs[b])
            assert ln == int(mix.ctx[b]) + 1 + a2 and pend == out2[-1], b
        # directly against the oracle's own decisions, wherever these cannot flip under twice the
        # measured logit error
        z32 = z.astype(np.float32)
        if mode == "greedy":
            a_or, out_or, _ = oracle.greedy_accept(z32, drafts)
            if accept_margin_ok(z32, drafts, "greedy", None, None, 1.0, 2 * err):
                assert n_acc[b] == a_or and np.array_equal(out[r0:r0 + a_or + 1], out_or), (b, "direct")
                direct += 1
        else:
            a_or, out_or, _ = oracle.stochastic_accept(z32, drafts, q, u, temp)
            _, safe, draw_safe = stochastic_margins(z32, drafts, q, u, temp, 2 * np.abs(zg[r0:r1] - z).max())
            if safe:
                assert n_acc[b] == a_or and np.array_equal(out[r0:r0 + a_or], out_or[:a_or]), (b, "direct")
                direct += 1
            if draw_safe:
                assert out[r0 + a_or] == out_or[-1], (b, "direct draw")
    print(f"mix of {B} sequences, {total} rows ({'persistent' if persistent and expect_fast else 'few-row' if expect_fast else 'general'} kernels): "
          f"worst logit error {worst:.3e}; accepted {n_acc.tolist()} of {mix.k.tolist()}; "
          f"{direct} of {B} sequences compared directly with the oracle's decisions", flush=True)
    return pair, seqs, ctxs, pendings, per_seq, zg, row_off


def test_rag_mix_batched_paged_verify_against_oracle():
    cfg = wl.scaled(C["1.5b_rag_mix"], n_layers=2, vocab=8192, ctx=256)
    mix = wl.rag_mix(cfg, wl.streams(cfg).mix, ctx_min=64, ctx_max=1024)
    assert int(np.sum(mix.k + 1)) > 48                   # takes the general (any row count) kernels
    pair, seqs, ctxs, pendings, per_seq, zg, row_off = _run_mix(cfg, mix, expect_fast=False)
    # batch / paging invariance: every sequence alone, in a private contiguous cache
    for b in (0, 7, 15):
        drafts = per_seq[b][0]
        n_ctx, k = int(mix.ctx[b]), len(drafts)
        solo = pair.new_seq(n_ctx + k + 1)
        toks = i32(ctxs[b])
        for c0 in range(0, n_ctx, cfg.chunk):
            vf.vf_prefill_chunk(pair.model, solo, toks[c0:c0 + cfg.chunk])
        lg = torch.empty((k + 1, cfg.vocab), dtype=torch.float32, device=DEV)
        vf.vf_verify(pair.model, [solo], i32([pendings[b]] + [int(t) for t in drafts]), [0, k + 1], lg)
        torch.cuda.synchronize()
        err = rel_inf(lg.cpu().numpy(), zg[row_off[b]:row_off[b + 1]]).max()
        print(f"sequence {b}: alone + contiguous vs batched + paged: {err:.3e}", flush=True)
        assert err < 2e-2


def test_rag_mix_full_widths_long_contexts_against_oracle():
    """Six sequences of the real mix at their real context lengths (4416 and 3375 tokens among
    them), full 1.5B layer widths, two layers: contexts of more than 2048 keys share their keys out
    over several workgroups in the many-row attention, whose records a second kernel merges; here
    that path is compared with the oracle element by element, in the prefill (K/V of the last layer,
    last-row logits) and in the batched verify step (121 rows, mixed acceptance)."""
    from types import SimpleNamespace
    cfg = wl.scaled(C["1.5b_rag_mix"], n_layers=2, vocab=32768)
    full = wl.rag_mix(cfg, wl.streams(cfg).mix)
    pick = [5, 7, 3, 11, 0, 9]
    mix = SimpleNamespace(ctx=full.ctx[pick], k=full.k[pick], stochastic=full.stochastic[pick],
                          n_pages=full.n_pages, block_tables=[full.block_tables[i] for i in pick])
    assert sorted(mix.ctx.tolist())[-2:] == [3375, 4416] and int(np.sum(mix.k + 1)) > 48
    assert mix.stochastic.any() and not mix.stochastic.all()
    _run_mix(cfg, mix, expect_fast=False, check_kv=True)


def test_small_paged_batch_through_the_few_row_kernels():
    cfg = wl.scaled(C["1.5b_rag_mix"], n_layers=2, vocab=8192, ctx=200, batch=3, k=12)
    mix = wl.rag_mix(cfg, wl.streams(cfg).mix, ctx_min=70, ctx_max=400)
    assert int(np.sum(mix.k + 1)) <= 48
    _run_mix(cfg, mix, expect_fast=True, persistent=False)


def test_small_paged_batch_through_the_persistent_kernel():
    """Three paged sequences with ragged draft counts (up to 39 rows), then two (at most 20 rows),
    through the persistent whole-pass kernel."""
    cfg = wl.scaled(C["1.5b_rag_mix"], n_layers=2, vocab=8192, ctx=200, batch=3, k=12)
    mix = wl.rag_mix(cfg, wl.streams(cfg).mix, ctx_min=70, ctx_max=400)
    _run_mix(cfg, mix, expect_fast=True, persistent=True)
    cfg = wl.scaled(C["1.5b_rag_mix"], n_layers=3, vocab=4096, ctx=300, batch=2, k=9)
    mix = wl.rag_mix(cfg, wl.streams(cfg).mix, ctx_min=100, ctx_max=500)
    assert int(np.sum(mix.k + 1)) <= 32
    _run_mix(cfg, mix, expect_fast=True, persistent=True)


@pytest.mark.parametrize("rows", [48, 49])
def test_full_batch_at_the_row_limit_of_the_few_row_kernels(rows):
    """As many sequences as a call may hold (VF_MAX_BATCH), half of them without any draft, with 48 rows
    in all (the most the persistent kernel takes) and with 49 (the first call that goes to the kernels
    for any row count): both against the oracle, sequence by sequence."""
    B = vf.VF_MAX_BATCH
    cfg = wl.scaled(C["1.5b_rag_mix"], n_layers=2, vocab=4096, ctx=120, batch=B, k=3)
    mix = wl.rag_mix(cfg, wl.streams(cfg).mix, ctx_min=40, ctx_max=300)
    with_draft = rows - B                                  # sequences with one draft; the others have none
    mix.k = np.array([1] * with_draft + [0] * (B - with_draft))   # never more than the drafts the pages were sized for
    assert int(np.sum(mix.k + 1)) == rows and len(mix.k) == B
    _run_mix(cfg, mix, expect_fast=rows <= 48, persistent=True)


def test_multi_row_verify_equals_single_row_decodes_on_the_gpu():
    """The equivalence the paper states for its long and short graphs (Sec. 4.1), and the
    lossless property (Sec. 3): greedy speculative decoding emits exactly the plain greedy
    sequence, here with both sides on the GPU."""
    cfg = wl.scaled(C["0.5b_k8"], n_layers=3, vocab=4096)
    pair = Pair(cfg, max_rows=128, max_positions=512)
    s = pair.s
    ctx = wl.make_context(cfg.vocab, 150, s.context)
    toks = i32(ctx)
    greedy = [(vf.VF_GREEDY, 0.0, None, None)]

    def fresh():
        seq = pair.new_seq(400)
        for c0 in range(0, 150, 128):
            vf.vf_prefill_chunk(pair.model, seq, toks[c0:c0 + 128], sample_first=c0 + 128 >= 150)
        return seq
    n_acc = torch.zeros(1, dtype=torch.int32, device=DEV)
    out_t = torch.zeros(33, dtype=torch.int32, device=DEV)
    y_t = torch.zeros(33, dtype=torch.int32, device=DEV)
    # plain greedy decoding: verify with no drafts, one token per step
    seq = fresh()
    pending0 = vf.vf_seq_get_state(seq)[1]
    pend = i32([vf.VF_PENDING])
    plain, single = [], []
    lg1 = torch.empty((1, cfg.vocab), dtype=torch.float32, device=DEV)
    for _ in range(40):
        vf.vf_verify(pair.model, [seq], pend, [0, 1], lg1)        # pending token taken from device state
        vf.vf_accept(pair.model, [seq], pend, [0, 1], greedy, n_acc, out_t, y_t)
        plain.append(int(out_t[0].item()))
        single.append(lg1[0].cpu().numpy().copy())
    # one 9-row verify of [T, first 8 plain tokens]: logits equal the 9 single-row decodes
    seq2 = fresh()
    lg = torch.empty((9, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify(pair.model, [seq2], i32([pending0] + plain[:8]), [0, 9], lg)
    torch.cuda.synchronize()
    multi = lg.cpu().numpy()
    err = rel_inf(multi, np.stack(single[:9])).max()
    print(f"9-row verify vs 9 single-row decodes: {err:.3e} (bit-equal: {np.array_equal(multi, np.stack(single[:9]))})",
          flush=True)
    assert err < 1e-2
    # speculative greedy decoding with drafts of mixed quality reproduces the plain sequence
    for kind in ("random", "perfect", "half"):
        seq3 = fresh()
        emitted, steps = [], 0
        rng = np.random.default_rng(5)
        while len(emitted) < 32:
            pos = len(emitted)
            k = int(rng.integers(0, 9))
            if kind == "random":
                drafts = rng.integers(0, cfg.vocab, k).tolist()
            elif kind == "perfect":
                drafts = plain[pos:pos + k]
            else:
                drafts = plain[pos:pos + k]
                if k > 2:
                    drafts[k // 2] = (drafts[k // 2] + 1) % cfg.vocab
            t = i32([vf.VF_PENDING] + drafts)
            vf.vf_verify(pair.model, [seq3], t, [0, k + 1])
            vf.vf_accept(pair.model, [seq3], t, [0, k + 1], greedy, n_acc, out_t, y_t)
            a = int(n_acc.item())
            emitted += out_t[:a + 1].cpu().tolist()
            steps += 1
        # identical up to logit ties between the two kernel shapes
        first_bad = next((i for i in range(32) if emitted[i] != plain[i]), None)
        print(f"speculative greedy ({kind} drafts): {steps} steps for 32 tokens, first difference {first_bad}", flush=True)
        assert first_bad is None, (kind, first_bad)
