"""The seeded generators are deterministic and have the stated structure (no GPU)."""
import numpy as np

import workloads as wl


def test_streams_are_reproducible_and_independent():
    cfg = wl.CONFIGS["tiny_f32"]
    a, b = wl.streams(cfg), wl.streams(cfg)
    assert np.array_equal(wl.make_context(cfg.vocab, 50, a.context), wl.make_context(cfg.vocab, 50, b.context))
    assert not np.array_equal(a.drafts.integers(0, 1 << 30, 8), b.uniforms.integers(0, 1 << 30, 8))
    other = wl.streams(wl.CONFIGS["0.5b_k8"])
    assert not np.array_equal(wl.make_context(4096, 50, wl.streams(cfg).context),
                              wl.make_context(4096, 50, other.context))


def test_weights_shapes_and_bf16_values():
    cfg = wl.scaled(wl.CONFIGS["0.5b_k8"], n_layers=1, vocab=300)
    w = wl.make_weights(cfg, wl.streams(cfg).weights)
    lw = w["layers"][0]
    assert w["embed"].shape == (300, 896) and lw["wq"].shape == (896, 896) and lw["wk"].shape == (128, 896)
    assert lw["w_gate"].shape == (4864, 896) and lw["w_down"].shape == (896, 4864)
    assert np.all(w["final_norm"] == 1.0)
    bits = lw["wq"].view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)                       # exactly representable in bfloat16
    assert abs(float(lw["w_up"].std()) - 0.02) < 1e-3


def test_byte_counts_match_the_stated_shapes():
    c3 = wl.CONFIGS["1.5b_k16"]
    assert c3.weight_bytes() == 2_620_391_424 + 466_747_392
    assert c3.kv_bytes_per_token() == 28_672
    assert wl.CONFIGS["0.5b_k8"].weight_bytes() == 715_653_120 + 272_269_312
    assert wl.CONFIGS["3b_k32"].weight_bytes() == 5_637_144_576 + 788_004_864


def test_draft_generators():
    rng = np.random.default_rng(0)
    ctx = wl.make_context(1000, 200, rng)
    d = wl.copy_span_drafts(ctx, 8, 1.0, 1000, rng)
    assert any(np.array_equal(d, ctx[s:s + 8]) for s in range(193))
    g = wl.geometric_copy_drafts(ctx, 32, 12, 1000, rng)
    assert g.shape == (32,) and g.dtype == np.int32
    cont = np.arange(10, 16, dtype=np.int32)
    for e in range(1, 8):
        m = wl.inject_mismatch(cont, e, 1000, rng)
        assert np.sum(m != cont) == (1 if e <= 6 else 0)
        if e <= 6:
            assert m[e - 1] != cont[e - 1]
    u = wl.make_uniforms(5, rng)
    assert u.shape == (10,) and u.dtype == np.float32 and u.min() >= 0 and u.max() < 1


def test_gumbel_drafts_carry_a_distribution():
    rng = np.random.default_rng(1)
    table = rng.standard_normal((7, 7))
    drafts, q = wl.gumbel_drafts(lambda t: table[t], 3, 4, 0.8, 0.5, rng, rng)
    assert drafts.shape == (4,) and q.shape == (4, 7) and q.dtype == np.float32
    assert np.allclose(q.sum(-1), 1.0, atol=1e-6) and np.all(q[np.arange(4), drafts] > 0)


def test_rag_mix_structure():
    cfg = wl.CONFIGS["1.5b_rag_mix"]
    mix = wl.rag_mix(cfg, wl.streams(cfg).mix)
    assert len(mix.ctx) == 16 and mix.ctx.min() >= 512 and mix.ctx.max() <= 8192
    assert mix.k.min() >= 1 and mix.k.max() <= 32
    assert mix.stochastic.any() and not mix.stochastic.all()
    pages = np.concatenate(mix.block_tables)
    assert sorted(pages.tolist()) == list(range(mix.n_pages))           # a permutation of the pool
    for c, k, t in zip(mix.ctx, mix.k, mix.block_tables):
        assert len(t) * 64 >= c + k + 1
