"""Pins for the oracle's transformer forward (no GPU).

Each test checks the oracle against something other than itself: a closed
form, an invariant the paper states, a special case that reduces to a textbook
identity, or library routines (torch CPU).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import transformer as T
from oracle.loop import truncate
import workloads as wl
from util_oracle import spec_of, weights_of, rel_inf

TINY = wl.CONFIGS["tiny_f32"]
SMALL = wl.scaled(TINY, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=97,
                  n_layers=2)


def _setup(cfg, qkv_bias=False, dt=np.float64):
    s = wl.streams(cfg)
    wd = wl.make_weights(cfg, s.weights, qkv_bias=qkv_bias)
    return spec_of(cfg, qkv_bias), weights_of(wd, dt), wd, s


# ---- number format -----------------------------------------------------------------------------

def test_bf16_rounding_known_values_and_library():
    # ties-to-even on the 8-bit significand boundary, worked by hand
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -(1.0 + 2.0 ** -8), 3.0e-39, 0.0], dtype=np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -1.0, 0.0, 0.0], dtype=np.float32)
    got = oracle.round_bf16(x)
    # 3e-39 is subnormal: bf16 keeps the exponent range, so it rounds to a bf16 subnormal, not 0
    assert np.array_equal(got[:5], want[:5]) and got[6] == 0.0
    rng = np.random.default_rng(0)
    r = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    lib = torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.round_bf16(r), lib)
    assert np.array_equal(oracle.round_bf16(got), got)          # idempotent


# ---- P5: textbook special cases ----------------------------------------------------------------

def test_rmsnorm_constant_vector():
    g = np.linspace(0.5, 2.0, 32)
    for c in (3.0, -0.25):
        out = T.rmsnorm(np.full((2, 32), c), g, 0.0)
        assert np.allclose(out, np.sign(c) * g[None, :], rtol=0, atol=1e-15)


def test_rope_position_zero_is_identity_and_norm_preserving():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 2, 16))
    cos, sin = T.rope_tables(np.array([0, 0, 0]), 16, 1e4)
    assert np.array_equal(T.rope(x, cos, sin), x)
    cos, sin = T.rope_tables(np.array([5, 77, 4000]), 16, 1e4)
    y = T.rope(x, cos, sin)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-6)


def test_rope_is_complex_rotation_of_pairs():
    # pair (i, i+hd/2) as a complex number times exp(j*pos*theta^(-2i/hd))
    rng = np.random.default_rng(2)
    hd, theta = 32, 5e5
    x = rng.standard_normal((4, 1, hd))
    pos = np.array([1, 2, 300, 8191])
    cos, sin = T.rope_tables(pos, hd, theta)
    y = T.rope(x, cos, sin)
    zc = x[..., :hd // 2] + 1j * x[..., hd // 2:]
    ang = pos[:, None] * theta ** (-np.arange(0, hd, 2) / hd)[None, :]
    rot = zc * np.exp(1j * ang)[:, None, :]
    assert np.allclose(y[..., :hd // 2], rot.real, atol=1e-6)
    assert np.allclose(y[..., hd // 2:], rot.imag, atol=1e-6)


def test_rope_relative_position_property():
    # <rope(q,p+s), rope(k,t+s)> does not depend on the shift s
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal((1, 1, 64)), rng.standard_normal((1, 1, 64))
    dots = []
    for s in (0, 9, 1000):
        cq, sq = T.rope_tables(np.array([17 + s]), 64, 1e4)
        ck, sk = T.rope_tables(np.array([3 + s]), 64, 1e4)
        dots.append(float(np.sum(T.rope(q, cq, sq) * T.rope(k, ck, sk))))
    assert np.allclose(dots, dots[0], atol=2e-4)            # tables are float32


def test_zero_output_projections_give_head_of_normed_embedding():
    spec, w, _, s = _setup(SMALL)
    for lw in w.layers:
        lw.wo[:] = 0
        lw.w_down[:] = 0
    toks = wl.make_context(SMALL.vocab, 7, s.context)
    z = oracle.forward(spec, w, oracle.KVCache(spec, 16), toks)
    e = w.embed[toks]
    want = (e / np.sqrt((e * e).mean(-1, keepdims=True) + spec.rms_eps)) @ w.embed.T
    assert np.allclose(z, want, rtol=1e-12, atol=1e-14)


def test_zero_query_attention_is_running_mean_of_values():
    # 1 layer, MHA, Wq = 0 (uniform causal softmax), Wv = Wo = I, FFN off:
    # h_out[r] = h[r] + mean_{t<=r} rmsnorm(h[t])
    cfg = wl.scaled(SMALL, n_layers=1, n_kv_heads=4)
    spec, w, _, s = _setup(cfg)
    lw = w.layers[0]
    lw.wq[:] = 0
    lw.wv[:] = np.eye(cfg.d_model)
    lw.wo[:] = np.eye(cfg.d_model)
    lw.w_down[:] = 0
    toks = wl.make_context(cfg.vocab, 9, s.context)
    cache = oracle.KVCache(spec, 16)
    z = oracle.forward(spec, w, cache, toks[:4])          # in two pieces: cache path too
    z = np.concatenate([z, oracle.forward(spec, w, cache, toks[4:])])
    h = w.embed[toks]
    xn = h / np.sqrt((h * h).mean(-1, keepdims=True) + spec.rms_eps)
    run_mean = np.cumsum(xn, axis=0) / np.arange(1, 10)[:, None]
    h2 = h + run_mean
    want = (h2 / np.sqrt((h2 * h2).mean(-1, keepdims=True) + spec.rms_eps)) @ w.embed.T
    assert np.allclose(z, want, rtol=1e-10, atol=1e-12)


def test_gqa_equals_mha_with_replicated_kv_heads():
    spec, w, _, s = _setup(SMALL)                       # 4 q heads, 2 kv heads
    toks = wl.make_context(SMALL.vocab, 11, s.context)
    z_gqa = oracle.forward(spec, w, oracle.KVCache(spec, 16), toks)
    mha = wl.scaled(SMALL, n_kv_heads=4)
    spec2 = spec_of(mha)
    hd = SMALL.head_dim
    w2 = w.astype(np.float64)
    for lw in w2.layers:
        for name in ("wk", "wv"):
            a = getattr(lw, name).reshape(2, hd, -1)
            setattr(lw, name, np.repeat(a, 2, axis=0).reshape(4 * hd, -1))
    z_mha = oracle.forward(spec2, w2, oracle.KVCache(spec2, 16), toks)
    assert np.allclose(z_gqa, z_mha, rtol=1e-12, atol=1e-14)


# ---- P6: library cross-check -------------------------------------------------------------------

def _torch_reference(cfg, wd, toks, qkv_bias=False):
    """The same model from torch CPU library routines (float64), RoPE written as a
    complex multiplication -- an independent formulation."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    n, hq, hkv, hd = len(toks), cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    h = F.embedding(torch.from_numpy(np.asarray(toks, dtype=np.int64)), t(wd["embed"]))
    ang = torch.arange(n, dtype=torch.float64)[:, None] * \
        cfg.rope_theta ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)

    def rope(x):
        xc = torch.complex(x[..., :hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([xc.real, xc.imag], dim=-1)
    for lw in wd["layers"]:
        x = F.rms_norm(h, (cfg.d_model,), t(lw["attn_norm"]), cfg.rms_eps)
        q = F.linear(x, t(lw["wq"]), t(lw["bq"]) if qkv_bias else None).view(n, hq, hd)
        k = F.linear(x, t(lw["wk"]), t(lw["bk"]) if qkv_bias else None).view(n, hkv, hd)
        v = F.linear(x, t(lw["wv"]), t(lw["bv"]) if qkv_bias else None).view(n, hkv, hd)
        q, k = rope(q), rope(k)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True,
                                           enable_gqa=True)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(n, hq * hd), t(lw["wo"]))
        x = F.rms_norm(h, (cfg.d_model,), t(lw["ffn_norm"]), cfg.rms_eps)
        h = h + F.linear(F.silu(F.linear(x, t(lw["w_gate"]))) * F.linear(x, t(lw["w_up"])),
                         t(lw["w_down"]))
    return F.linear(F.rms_norm(h, (cfg.d_model,), t(wd["final_norm"]), cfg.rms_eps),
                    t(wd["embed"])).numpy()


@pytest.mark.parametrize("qkv_bias", [False, True])
def test_forward_matches_torch_library_routines(qkv_bias):
    cfg = wl.scaled(TINY, vocab=512)                     # the tiny config's real widths
    spec, w, wd, s = _setup(cfg, qkv_bias)
    toks = wl.make_context(cfg.vocab, 40, s.context)
    z = oracle.forward(spec, w, oracle.KVCache(spec, 64), toks)
    ref = _torch_reference(cfg, wd, toks, qkv_bias)
    # the oracle's angle tables are float32-rounded, the library path's are not
    assert rel_inf(z, ref).max() < 1e-5
    # chunked (cache path) against the same library result
    cache = oracle.KVCache(spec, 64)
    zc = np.concatenate([oracle.forward(spec, w, cache, toks[a:b]) for a, b in ((0, 16), (16, 17), (17, 40))])
    assert rel_inf(zc, ref).max() < 1e-5


# ---- P1 / P4: the equivalences the paper states ------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_multi_row_verify_equals_sequential_single_row_decodes(dtype):
    cfg = wl.scaled(SMALL, dtype=dtype)
    spec, w, _, s = _setup(cfg)
    ctx = wl.make_context(cfg.vocab, 24, s.context)
    base = oracle.KVCache(spec, 48)
    oracle.prefill(spec, w, base, ctx, 8)
    rows = wl.make_context(cfg.vocab, 6, s.drafts)
    c1 = base.clone()
    z_multi = oracle.verify(spec, w, c1, rows[0], rows[1:])
    c2 = base.clone()
    z_seq = np.concatenate([oracle.forward(spec, w, c2, [t]) for t in rows])
    assert c1.len == c2.len == 30
    assert np.allclose(z_multi, z_seq, rtol=1e-11, atol=1e-13)
    assert np.allclose(c1.k, c2.k, rtol=1e-12, atol=0) and np.allclose(c1.v, c2.v, rtol=1e-12, atol=0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prefill_chunk_size_invariance(dtype):
    cfg = wl.scaled(SMALL, dtype=dtype)
    spec, w, _, s = _setup(cfg)
    ctx = wl.make_context(cfg.vocab, 37, s.context)
    ref_cache = oracle.KVCache(spec, 40)
    z_ref = oracle.prefill(spec, w, ref_cache, ctx, 37)
    for chunk in (16, 4, 1):
        c = oracle.KVCache(spec, 40)
        z = oracle.prefill(spec, w, c, ctx, chunk)
        assert np.allclose(z, z_ref, rtol=1e-11, atol=1e-13)
        assert np.allclose(c.k, ref_cache.k, rtol=1e-12) and np.allclose(c.v, ref_cache.v, rtol=1e-12)


def test_truncate_then_continue_equals_never_having_drafted():
    # rows written for rejected drafts must not influence later steps
    spec, w, _, s = _setup(SMALL)
    ctx = wl.make_context(SMALL.vocab, 12, s.context)
    a = oracle.KVCache(spec, 32)
    oracle.prefill(spec, w, a, ctx, 4)
    b = a.clone()
    oracle.verify(spec, w, a, 5, [6, 7, 8, 9])
    truncate(a, 13)                                      # keep only the pending token's row
    oracle.forward(spec, w, b, [5])
    za = oracle.forward(spec, w, a, [11, 12])
    zb = oracle.forward(spec, w, b, [11, 12])
    assert np.allclose(za, zb, rtol=1e-12, atol=1e-14)


def test_bf16_mode_rounds_only_where_stated():
    # cache contents and nothing else observable must be bf16 values; logits are not
    cfg = wl.scaled(SMALL, dtype="bf16")
    spec, w, _, s = _setup(cfg)
    c = oracle.KVCache(spec, 16)
    z = oracle.forward(spec, w, c, wl.make_context(cfg.vocab, 9, s.context))
    assert np.array_equal(oracle.round_bf16(c.k), c.k) and np.array_equal(oracle.round_bf16(c.v), c.v)
    assert not np.array_equal(oracle.round_bf16(z), z)
    # and the bf16 model stays close to the unrounded one (rounding is a perturbation, not a bug)
    spec32 = spec_of(wl.scaled(cfg, dtype="f32"))
    z32 = oracle.forward(spec32, w, oracle.KVCache(spec32, 16), wl.make_context(cfg.vocab, 9, wl.streams(cfg).context))
    assert rel_inf(z, z32).max() < 3e-2


def test_logit_rows_selects_rows_of_the_full_result():
    """forward(..., logit_rows=r) is rows r of forward(...): the head is row-wise."""
    spec, w, _, _ = _setup(SMALL)
    toks = [3, 9, 1, 7, 7, 2]
    a, b = oracle.KVCache(spec, 16), oracle.KVCache(spec, 16)
    full = oracle.forward(spec, w, a, toks)
    some = oracle.forward(spec, w, b, toks, logit_rows=[5, 0, 2])
    assert some.shape == (3, spec.vocab)
    assert np.allclose(some, full[[5, 0, 2]], rtol=1e-12, atol=1e-14)
    assert np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v)
