"""vf_accept_static (acceptance with the library's static device scratch, for callers that cannot
allocate) against vf_accept, through the C ABI: same logits, drafts, draft distributions and
uniforms on both, two calls in a row, the second with a smaller input; every output and the
committed state must be identical, bit for bit."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2510_15312_amd as vf
from util_gpu import DEV, Pair, i32, f32

pytestmark = pytest.mark.gpu


def _inputs(rng, V, ks, dense):
    """Crafted logits with a clear winner per row, drafts that follow the winners up to a planted
    mismatch, uniforms, and (for `dense` sequences) full draft distributions."""
    tokens, row_off, params, modes = [], [0], [], []
    total = int(sum(k + 1 for k in ks))
    z = rng.normal(0.0, 2.0, (total, V)).astype(np.float32)
    for b, k in enumerate(ks):
        r0 = row_off[-1]
        best = z[r0:r0 + k + 1].argmax(-1)
        drafts = best[:k].copy()
        e = int(rng.integers(0, k + 1))
        if e < k:
            drafts[e] = (drafts[e] + 1 + int(rng.integers(0, V - 1))) % V
        stochastic = b % 2 == 1
        q = u = None
        if stochastic:
            u = rng.random(2 * (k + 1)).astype(np.float32)
            if b in dense and k:
                qs = rng.dirichlet(np.full(V, 0.05), size=k).astype(np.float32)
                qs[np.arange(k), drafts] += 0.5
                q = (qs / qs.sum(-1, keepdims=True, dtype=np.float64)).astype(np.float32)
        params.append((vf.VF_STOCHASTIC if stochastic else vf.VF_GREEDY, 0.8 if stochastic else 0.0,
                       None if q is None else f32(q), None if u is None else f32(u)))
        tokens += [int(rng.integers(0, V))] + [int(t) for t in drafts]
        row_off.append(r0 + k + 1)
    return i32(tokens), row_off, params, f32(z), total


def _run(fn, pair, seqs, lens, tokens, row_off, params, z, total):
    for s, n in zip(seqs, lens):
        vf.vf_seq_set_len(s, n)
        vf.vf_seq_set_pending(s, 0)
    n_acc = torch.full((len(seqs),), -7, dtype=torch.int32, device=DEV)
    out = torch.full((total,), -7, dtype=torch.int32, device=DEV)
    y = torch.full((total,), -7, dtype=torch.int32, device=DEV)
    fn(pair.model, seqs, tokens, row_off, params, n_acc, out, y, z)
    torch.cuda.synchronize()
    state = [vf.vf_seq_get_state(s) for s in seqs]
    return n_acc.cpu().numpy(), out.cpu().numpy(), y.cpu().numpy(), state


def test_accept_static_equals_accept_on_two_calls():
    cfg = wl.scaled(wl.CONFIGS["0.5b_k8"], n_layers=1, vocab=4096)
    pair = Pair(cfg, max_rows=256, max_positions=512)
    rng = np.random.default_rng(77)
    seqs = [pair.new_seq(400) for _ in range(6)]
    lens = [100 + 7 * i for i in range(6)]
    for ks, dense in (([32, 17, 9, 32, 1, 0], {1, 3}), ([5, 3], {1})):   # 97 rows, then 10 rows
        n = len(ks)
        tokens, row_off, params, z, total = _inputs(rng, cfg.vocab, ks, dense)
        want = _run(vf.vf_accept, pair, seqs[:n], lens[:n], tokens, row_off, params, z, total)
        got = _run(vf.vf_accept_static, pair, seqs[:n], lens[:n], tokens, row_off, params, z, total)
        for w, g, what in zip(want, got, ("n_accept", "out_tokens", "y", "state")):
            assert np.array_equal(np.asarray(w), np.asarray(g)), what
        assert all(0 <= a <= k for a, k in zip(want[0], ks))
        assert [st[0] for st in got[3]] == [l + 1 + int(a) for l, a in zip(lens, got[0])]
        print(f"vf_accept_static == vf_accept on {total} rows: accepted {got[0].tolist()} of {ks}", flush=True)
    # beyond the static scratch: refused on the host, nothing launched
    big = [32] * 16                                                          # 528 rows > 512
    more = [pair.new_seq(100) for _ in range(10)]
    tokens, row_off, params, z, total = _inputs(rng, 64, big, set())
    with pytest.raises(vf.VfError) as e:
        big_pair_rows = torch.zeros(total, dtype=torch.int32, device=DEV)
        vf.vf_accept_static(pair.model, seqs + more, tokens, row_off, params,
                            torch.zeros(16, dtype=torch.int32, device=DEV), big_pair_rows, big_pair_rows.clone(), z)
    assert e.value.code in (vf.VF_ERR_CAP,)
