"""The draft-verify loop end to end on the GPU: generation with the retrieval drafter and the reuse
pool produces exactly the plain greedy text."""
import numpy as np
import pytest

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
