"""The draft-verify loop end to end on the GPU: generation with the retrieval drafter and the reuse
pool produces exactly the plain greedy text."""
import numpy as np
import pytest

import oracle
from oracle.drafter import suffix_match_draft
from oracle.loop import plain_greedy, speculative_greedy
import workloads as wl
import paper_2510_15312_amd as vf
from paper_2510_15312_amd.generate import generate
from util_gpu import Pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k", [16, 5])
def test_generate_equals_plain_greedy(k):
    cfg = wl.CONFIGS["tiny_f32"]
    pair = Pair(cfg, max_rows=128, max_positions=600)
    rng = np.random.default_rng(1)
    span = rng.integers(0, cfg.vocab, 23).tolist()
    prompt = (span * 9)[:200] + rng.integers(0, cfg.vocab, 13).tolist() + span[:7]   # a repetitive context
    plain, st0 = generate(pair.model, pair.new_seq(600), prompt, 80, k=0, chunk=128)
    spec, st = generate(pair.model, pair.new_seq(600), prompt, 80, k=k, chunk=128)
    print(f"k {k}: plain {st0['steps']} steps; draft-verify {st['steps']} steps, {st['accepted_drafts']} of "
          f"{st['drafted']} drafts accepted, {st['tokens_per_step']:.2f} tokens per step", flush=True)
    assert st0["steps"] == 79 and spec == plain
    assert st["steps"] <= st0["steps"]


def test_generate_with_rejected_drafts_runs_up_to_capacity():
    """Drafts that are almost always refused: every step writes k + 1 rows and keeps one.  The
    host-side bound of the length must follow the true length (vf_seq_note_len), or the capacity
    check refuses steps long before the cache is full."""
    cfg = wl.CONFIGS["tiny_f32"]
    pair = Pair(cfg, max_rows=128, max_positions=600)
    rng = np.random.default_rng(2)
    prompt = rng.integers(0, cfg.vocab, 220).tolist()
    cap, k = 600, 16
    n_new = cap - len(prompt) - (k + 1) - 1                # the last step still fits k + 1 rows
    plain, st0 = generate(pair.model, pair.new_seq(cap), prompt, n_new, k=0, chunk=128)
    draft_rng = np.random.default_rng(3)
    spec, st = generate(pair.model, pair.new_seq(cap), prompt, n_new, k=k, chunk=128,
                        drafter=lambda text, kk: draft_rng.integers(0, cfg.vocab, kk).tolist())
    print(f"low acceptance: {st['steps']} steps, {st['accepted_drafts']} of {st['drafted']} drafts accepted", flush=True)
    assert spec == plain
    assert st["drafted"] > 10 * max(1, st["accepted_drafts"])


def test_generate_against_the_oracle_loops():
    """The library's generation loop against the oracle's: plain greedy decoding and the oracle's own
    draft-verify loop (its verify, its acceptance, its suffix-match drafter) from the same prompt on
    the float32 model, token for token; the accepted counts per step of the two draft-verify loops
    agree as well when both use the plain drafter (no reuse pool)."""
    cfg = wl.CONFIGS["tiny_f32"]
    pair = Pair(cfg, max_rows=128, max_positions=600)
    rng = np.random.default_rng(4)
    span = rng.integers(0, cfg.vocab, 19).tolist()
    prompt = (span * 8)[:140] + rng.integers(0, cfg.vocab, 9).tolist() + span[:6]
    n_new, k = 60, 8
    cache = oracle.KVCache(pair.spec, 600)
    z_last = oracle.prefill(pair.spec, pair.ow, cache, np.asarray(prompt), 128)
    first = oracle.first_token(z_last)
    want = [first] + plain_greedy(pair.spec, pair.ow, cache.clone(), first, n_new - 1)

    def drafter(emitted, pending):
        return suffix_match_draft(list(prompt) + [first] + [int(t) for t in emitted], k, 8, 1)
    spec_or, acc_or = speculative_greedy(pair.spec, pair.ow, cache.clone(), first, n_new - 1, drafter)
    assert [first] + spec_or[:n_new - 1] == want            # the oracle's own loop is lossless
    got_plain, _ = generate(pair.model, pair.new_seq(600), prompt, n_new, k=0, chunk=128)
    got_spec, st = generate(pair.model, pair.new_seq(600), prompt, n_new, k=k, chunk=128, reuse=False)
    print(f"oracle loop: {len(acc_or)} steps, accepted {sum(acc_or)}; library loop: {st['steps']} steps, "
          f"accepted {st['accepted_drafts']}", flush=True)
    assert got_plain == want
    assert got_spec == want
    assert st["steps"] == len(acc_or) and st["accepted_drafts"] == sum(acc_or)


def test_generate_on_a_bf16_model_equals_plain_decoding_on_the_gpu():
    """1.5B layer widths in bfloat16 (reduced depth and vocabulary): the draft-verify loop through
    the persistent kernel against plain one-token decoding on the same GPU."""
    cfg = wl.scaled(wl.CONFIGS["1.5b_k16"], n_layers=3, vocab=8192)
    pair = Pair(cfg, max_rows=256, max_positions=700)
    rng = np.random.default_rng(6)
    span = rng.integers(0, cfg.vocab, 31).tolist()
    prompt = (span * 9)[:260] + rng.integers(0, cfg.vocab, 5).tolist() + span[:9]
    plain, st0 = generate(pair.model, pair.new_seq(700), prompt, 48, k=0)
    spec, st = generate(pair.model, pair.new_seq(700), prompt, 48, k=16)
    first_bad = next((i for i in range(48) if spec[i] != plain[i]), None)
    print(f"bf16 1.5B widths: plain {st0['steps']} steps; draft-verify {st['steps']} steps, {st['accepted_drafts']} of "
          f"{st['drafted']} drafts accepted; first difference {first_bad}", flush=True)
    assert first_bad is None
