"""The reuse-segment kernel through the C ABI against the oracle: the hand-worked cases, seeded
random batches over every draft count, and the predictions of a real verify + accept."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle.loop import plain_greedy
from oracle.reuse import reuse_segment
import workloads as wl
import paper_2510_15312_amd as vf
from util_gpu import DEV, Pair, i32, gpu_accept

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def _select(cases):
    """cases: list of (x, y, a).  Lays them out as one ragged batch ([T, x_1..x_n] per sequence, y per
    row) and runs the kernel."""
    toks, ys, ro = [], [], [0]
    for x, y, a in cases:
        toks += [7] + list(x)
        ys += list(y)
        ro.append(ro[-1] + len(x) + 1)
    seg = torch.full((2 * len(cases),), -7, dtype=torch.int32, device=DEV)
    print("reuse_select batch of", len(cases), "sequences,", ro[-1], "rows", flush=True)
    vf.vf_reuse_select(i32(toks), ro, i32(ys), i32([a for _, _, a in cases]), seg)
    torch.cuda.synchronize()
    return seg.cpu().numpy().reshape(-1, 2)


def test_hand_worked_cases_on_the_gpu():
    cases, want = [], []
    for line in open(os.path.join(HERE, "golden", "reuse_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        x, y, a, w = [[int(t) for t in f.split()] for f in line.split("|")]
        cases.append((x, y, a[0]))
        want.append(w)
    got = _select(cases)
    assert got.tolist() == want
    assert got.tolist() == [list(reuse_segment(*c)) for c in cases]


def test_random_batches_bit_exact():
    rng = np.random.default_rng(15312)
    counts = list(range(0, 33)) * 4
    rng.shuffle(counts)
    for lo in range(0, len(counts), vf.VF_MAX_BATCH):
        cases = []
        for n in counts[lo:lo + vf.VF_MAX_BATCH]:
            alphabet = int(rng.choice([2, 3, 50]))
            x = rng.integers(0, alphabet, n)
            y = np.where(rng.random(n + 1) < 0.6, np.append(x, 0), rng.integers(0, alphabet, n + 1))
            cases.append((x.tolist(), y.tolist(), int(rng.integers(0, n + 1))))
        got = _select(cases)
        assert got.tolist() == [list(reuse_segment(*c)) for c in cases]


def test_segments_of_a_real_verify_step():
    cfg = wl.scaled(wl.CONFIGS["tiny_f32"], vocab=64)
    pair = Pair(cfg, max_rows=64, max_positions=256)
    rng = np.random.default_rng(5)
    ctx = wl.make_context(cfg.vocab, 40, rng)
    seq = pair.new_seq(128)
    cache = oracle.KVCache(pair.spec, 128)
    pair.prefill_both(seq, cache, ctx, 16)
    # drafts: the model's own greedy continuation with two tokens replaced, so that predictions
    # re-align with the draft after the first replacement
    k = 12
    T = int(rng.integers(0, cfg.vocab))
    cont = plain_greedy(pair.spec, pair.ow, cache.clone(), T, k)
    drafts = np.array(cont, dtype=np.int32)
    drafts[3] = (drafts[3] + 1) % cfg.vocab
    drafts[8] = (drafts[8] + 1) % cfg.vocab
    tokens = np.concatenate([[T], drafts]).astype(np.int32)
    z_or = oracle.verify(pair.spec, pair.ow, cache.clone(), T, drafts)
    a_or, _, y_or = oracle.greedy_accept(z_or, drafts)
    vf.vf_seq_set_pending(seq, T)
    tok_dev = i32(tokens)
    vf.vf_verify(pair.model, [seq], tok_dev, [0, k + 1])
    n_acc, _, y = gpu_accept(pair, [seq], tok_dev, [0, k + 1], [(vf.VF_GREEDY, 0.0, None, None)])
    assert n_acc[0] == a_or == 3 and np.array_equal(y, y_or)
    seg = torch.zeros(2, dtype=torch.int32, device=DEV)
    vf.vf_reuse_select(tok_dev, [0, k + 1], i32(y), i32(n_acc), seg)
    torch.cuda.synchronize()
    assert tuple(seg.cpu().tolist()) == reuse_segment(drafts.tolist(), y_or.tolist(), a_or)
