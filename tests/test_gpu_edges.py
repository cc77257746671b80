"""GPU edge cases through the C ABI: acceptance on crafted logits (ties, all accepted, no drafts,
one-hot and dense draft distributions over many seeded cases), error paths that must leave the
state untouched, biases, and the sampled first token."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2510_15312_amd as vf
from util_oracle import rel_inf
from util_gpu import DEV, Pair, i32, f32, gpu_accept, accept_margin_ok

pytestmark = pytest.mark.gpu
C = wl.CONFIGS
SMALL = wl.scaled(C["tiny_f32"], vocab=256)


@pytest.fixture(scope="module")
def small_pair():
    return Pair(SMALL, max_rows=64, max_positions=256)


def _accept_on(pair, seq, logits, drafts, params, k):
    tokens = i32(np.concatenate([[0], drafts]).astype(np.int32))
    return gpu_accept(pair, [seq], tokens, [0, k + 1], params, logits=f32(logits))


def test_accept_crafted_cases_bit_exact(small_pair):
    pair = small_pair
    V = SMALL.vocab
    seq = pair.new_seq(200)
    rng = np.random.default_rng(3)
    greedy = [(vf.VF_GREEDY, 0.0, None, None)]
    # ties: lowest id wins, on every row
    z = np.zeros((3, V), dtype=np.float32)
    z[0, [200, 17, 90]] = 2.5
    z[1, :] = -1.0
    z[2, [255, 254]] = 1.0
    n, out, y = _accept_on(pair, seq, z, np.array([17, 0]), greedy, 2)
    assert list(y) == [17, 0, 254] and n[0] == 2 and list(out) == [17, 0, 254]
    # no drafts at all: plain decoding
    vf.vf_seq_set_len(seq, 5)
    n, out, y = _accept_on(pair, seq, z[:1], np.array([], dtype=np.int32), greedy, 0)
    assert n[0] == 0 and list(out) == [17] and vf.vf_seq_get_state(seq) == (6, 17)
    # many seeded cases, all draft counts 0..32, both drafter kinds, against the oracle
    checked = 0
    for case in range(120):
        k = int(rng.integers(0, 33))
        zz = (rng.standard_normal((k + 1, V)) * rng.choice([0.5, 2.0, 6.0])).astype(np.float32)
        temp = float(rng.choice([0.5, 0.8, 1.0, 1.7]))
        yy = zz.argmax(-1)
        drafts = np.where(rng.random(k) < 0.7, yy[:k], rng.integers(0, V, k)).astype(np.int32)
        mode = ["greedy", "onehot", "dense"][case % 3]
        u = wl.make_uniforms(k + 1, rng)
        q = None
        if mode == "dense" and k:
            q = rng.dirichlet(np.full(V, 0.3), size=k).astype(np.float32)
            q[np.arange(k), drafts] += rng.choice([0.0, 0.3, 2.0], size=k).astype(np.float32)
            q = (q / q.sum(-1, keepdims=True, dtype=np.float64)).astype(np.float32)
        vf.vf_seq_set_len(seq, 10)
        if mode == "greedy":
            a, o, yo = oracle.greedy_accept(zz, drafts)
            params = greedy
        else:
            a, o, yo = oracle.stochastic_accept(zz, drafts, q, u, temp)
            params = [(vf.VF_STOCHASTIC, temp, None if q is None else f32(q), f32(u))]
        n, out, y = _accept_on(pair, seq, zz, drafts, params, k)
        assert np.array_equal(y, yo), case
        if accept_margin_ok(zz, drafts, "greedy" if mode == "greedy" else "stochastic", q, u, temp, 1e-9):
            assert n[0] == a and np.array_equal(out[:a + 1], o) and np.all(out[a + 1:] == -1), (case, mode, k)
            assert vf.vf_seq_get_state(seq) == (10 + 1 + a, int(o[-1])), case
            checked += 1
    print(f"acceptance: {checked} of 120 seeded cases compared bit-exactly (rest screened by the 1e-9 margin)",
          flush=True)
    assert checked >= 110


def test_equal_draft_and_target_distributions_accept_everything(small_pair):
    pair = small_pair
    V, k, temp = SMALL.vocab, 6, 0.8
    seq = pair.new_seq(64)
    rng = np.random.default_rng(8)
    z = (rng.standard_normal((k + 1, V)) * 3).astype(np.float32)
    t = np.float64(np.float32(temp))
    e = np.exp((z[:k].astype(np.float64) - z[:k].max(-1, keepdims=True)) / t)
    q = (e / e.sum(-1, keepdims=True)).astype(np.float32)
    drafts = rng.integers(0, V, k).astype(np.int32)
    u = np.minimum(wl.make_uniforms(k + 1, rng), np.float32(0.999))
    n, out, _ = _accept_on(pair, seq, z, drafts, [(vf.VF_STOCHASTIC, temp, f32(q), f32(u))], k)
    assert n[0] == k and np.array_equal(out[:k], drafts)


def test_capacity_and_argument_errors_leave_state_unchanged(small_pair):
    pair = small_pair
    seq = pair.new_seq(70)
    toks = i32(wl.make_context(SMALL.vocab, 64, np.random.default_rng(0)))
    vf.vf_prefill_chunk(pair.model, seq, toks)
    assert vf.vf_seq_get_state(seq)[0] == 64
    with pytest.raises(vf.VfError) as e:
        vf.vf_verify(pair.model, [seq], i32([1] * 8), [0, 8])        # 64 + 8 > 70
    assert e.value.code == vf.VF_ERR_CAP
    with pytest.raises(vf.VfError) as e:
        vf.vf_prefill_chunk(pair.model, seq, toks[:7])               # 64 + 7 > 70
    assert e.value.code == vf.VF_ERR_CAP
    with pytest.raises(vf.VfError) as e:
        vf.vf_prefill_chunk(pair.model, pair.new_seq(200), i32([1] * 65))   # more rows than max_rows
    assert e.value.code == vf.VF_ERR_CAP
    with pytest.raises(vf.VfError) as e:
        vf.vf_verify(pair.model, [seq], i32([1] * 40), [0, 40])      # more than 33 rows per sequence
    assert e.value.code == vf.VF_ERR_ARG
    with pytest.raises(vf.VfError) as e:
        vf.vf_verify(pair.model, [seq, seq], i32([1] * 4), [0, 2, 4])   # the same sequence twice
    assert e.value.code == vf.VF_ERR_ARG
    with pytest.raises(vf.VfError) as e:
        vf.vf_seq_set_len(seq, 71)
    assert e.value.code == vf.VF_ERR_ARG
    assert vf.vf_seq_get_state(seq)[0] == 64
    # still usable: 6 rows fit exactly
    vf.vf_verify(pair.model, [seq], i32([1] * 6), [0, 6])
    n, out, y = gpu_accept(pair, [seq], i32([1] * 6), [0, 6], [(vf.VF_GREEDY, 0.0, None, None)])
    assert 0 <= n[0] <= 5 and vf.vf_seq_get_state(seq)[0] == 65 + n[0]
    # accept without a matching verify
    with pytest.raises(vf.VfError):
        gpu_accept(pair, [seq], i32([1] * 3), [0, 3], [(vf.VF_GREEDY, 0.0, None, None)])
    with pytest.raises(vf.VfError):
        gpu_accept(pair, [seq], i32([1] * 3), [0, 3], [(vf.VF_STOCHASTIC, 0.0, None, None)],
                   logits=torch.zeros((3, SMALL.vocab), device=DEV))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_qkv_bias_and_sampled_first_token(dtype):
    cfg = wl.scaled(C["tiny_f32"], dtype=dtype, vocab=1024, n_kv_heads=2)
    pair = Pair(cfg, max_rows=64, max_positions=256, qkv_bias=True, std=0.05)
    tol = 2e-2 if dtype == "bf16" else 1e-5
    ctx = wl.make_context(cfg.vocab, 100, pair.s.context)
    cache, seq = oracle.KVCache(pair.spec, 160), pair.new_seq(160)
    z_or = oracle.prefill(pair.spec, pair.ow, cache, ctx, 64)
    toks = i32(ctx)
    lg = torch.empty(cfg.vocab, dtype=torch.float32, device=DEV)
    u = f32([0.37])
    vf.vf_prefill_chunk(pair.model, seq, toks[:64])
    vf.vf_prefill_chunk(pair.model, seq, toks[64:], logits_mode=1, logits_out=lg, sample_first=True, u=u,
                        temperature=0.9)
    torch.cuda.synchronize()
    zg = lg.cpu().numpy()
    assert rel_inf(zg[None], z_or[None]).max() < tol
    ln, pend = vf.vf_seq_get_state(seq)
    assert ln == 100 and pend == oracle.first_token(zg, 0.9, np.float32(0.37))
    # all-position logits of a chunk (the input of the paper's calibration step, Sec. 4.2)
    seq2 = pair.new_seq(160)
    allz = torch.empty((64, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_prefill_chunk(pair.model, seq2, toks[:64], logits_mode=2, logits_out=allz)
    torch.cuda.synchronize()
    c2 = oracle.KVCache(pair.spec, 64)
    z_all = oracle.forward(pair.spec, pair.ow, c2, ctx[:64])
    assert rel_inf(allz.cpu().numpy(), z_all).max() < tol
    # verify with biases through whichever kernels apply
    drafts = wl.make_context(cfg.vocab, 9, pair.s.drafts)
    z = oracle.verify(pair.spec, pair.ow, cache, int(pend), drafts)
    out = torch.empty((10, cfg.vocab), dtype=torch.float32, device=DEV)
    vf.vf_verify(pair.model, [seq], i32([vf.VF_PENDING] + drafts.tolist()), [0, 10], out)
    torch.cuda.synchronize()
    err = rel_inf(out.cpu().numpy(), z).max()
    print(f"qkv bias, {dtype}: verify error {err:.3e}", flush=True)
    assert err < tol


@pytest.mark.parametrize("name", ["0.5b_k8", "1.5b_k16"])
def test_kv_cache_layout_round_trip(name):
    """Every (position, kv head, feature) of a cache has a place of its own: K and V rows written at
    arbitrary offsets of a paged cache (head_dim 64 and 128) come back exactly, and rows written
    later leave the earlier ones alone.  The cache keeps its pages in the order the attention MFMAs
    consume them, so this is a test of that index map, not of a copy."""
    cfg = wl.scaled(C[name], n_layers=2, vocab=512)
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights)
    model = vf.vf_model_create(vf.config_from(cfg, 64, 512), vf.upload_weights(wd, cfg.dtype, DEV), DEV)
    n_pages = 5
    pool = torch.zeros(vf.vf_kv_bytes(model, 64, n_pages), dtype=torch.uint8, device=DEV)
    seq = vf.vf_seq_create(model, 4 * 64, pool, i32([3, 0, 4, 1]), DEV)
    rng = np.random.default_rng(7)
    shape = (4 * 64, cfg.n_kv_heads, cfg.head_dim)
    want = {}
    for layer in range(cfg.n_layers):
        k = rng.standard_normal(shape).astype(np.float32)
        v = rng.standard_normal(shape).astype(np.float32)
        k, v = (torch.tensor(a).to(torch.bfloat16).float().numpy() for a in (k, v))   # values the cache can hold
        want[layer] = (k, v)
        for t0, n in ((0, 37), (37, 1), (38, 90), (128, 128)):                       # ragged pieces, page borders inside
            vf.vf_kv_write(model, seq, layer, t0, f32(k[t0:t0 + n]), f32(v[t0:t0 + n]))
    torch.cuda.synchronize()
    for layer in range(cfg.n_layers):
        for t0, n in ((0, 256), (63, 2), (100, 57)):
            kg, vg = vf.vf_kv_read(model, seq, layer, t0, n)
            torch.cuda.synchronize()
            assert np.array_equal(kg.cpu().numpy(), want[layer][0][t0:t0 + n])
            assert np.array_equal(vg.cpu().numpy(), want[layer][1][t0:t0 + n])
