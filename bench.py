#!/usr/bin/env python3
"""Benchmark of the draft-verify step on one MI355X.

A step = one vf_verify + vf_accept over one batch (all rows of the hot path: embedding, 28
decoder layers against the prefilled KV cache, output head, acceptance, state commit).
Workload: the 1.5B-shaped model, context 2048 prefilled in 256-token chunks, k = 16 drafts per
step, stochastic acceptance at temperature 0.8 with a dense draft distribution (the target
softmax perturbed by Gumbel noise of scale 0.5).  All inputs are seeded and synthetic and are
resident in HBM before the timed region.

Prints one JSON line.  `value` is the achieved HBM bandwidth of the whole step (algorithmic
bytes per step / mean step time); ms_per_step is the verify-step latency.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the gate/up GEMM kernel from hardware counters (FETCH_SIZE + WRITE_SIZE,
# each scaled by what the same counter reads for a plain 1 GiB copy); 56,474,000 when last taken, see
# profiles/gateup_gemm_1.5b_k16_pmc.md.  None: the kernel's source has changed since.
GATEUP_TRAFFIC_BYTES = None
# The same for one launch of the persistent whole-pass kernel (profiles/verify_fused_1.5b_k16_pmc.md); set to
# None whenever that kernel changes.
FUSED_TRAFFIC_BYTES = 3_550_400_000


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_model(cfg, vf, wl, torch, max_rows, max_positions):
    t0 = time.time()
    wd = wl.make_weights(cfg, wl.streams(cfg).weights)
    log(f"[bench] weights generated on host in {time.time() - t0:.1f}s")
    dw = vf.upload_weights(wd, cfg.dtype)
    model = vf.vf_model_create(vf.config_from(cfg, max_rows, max_positions), dw)
    torch.cuda.synchronize()
    del dw
    torch.cuda.empty_cache()
    return model, wd


def draft_with_distribution(vf, torch, model, seq, pending, k, temperature, scale, gen):
    """Drafter (untimed input generation): k autoregressive single-row passes of the target,
    each giving q_i = softmax(z_i / T + scale * Gumbel) and a draft sampled from q_i."""
    V = model.cfg.vocab
    len0, _ = vf.vf_seq_get_state(seq)
    z = torch.empty((1, V), dtype=torch.float32, device="cuda:0")
    tok = torch.tensor([pending], dtype=torch.int32, device="cuda:0")
    drafts, qs = [], []
    for i in range(k):
        vf.vf_verify(model, [seq], tok, [0, 1], z)
        g = -torch.log(-torch.log(torch.rand(V, device="cuda:0", generator=gen, dtype=torch.float64)
                                  .clamp_(1e-300, 1 - 1e-16)))
        q = torch.softmax(z[0].double() / temperature + scale * g, dim=0)
        c = torch.cumsum(q, 0)
        u = torch.rand((), device="cuda:0", generator=gen, dtype=torch.float64) * c[-1]
        x = int(torch.searchsorted(c, u, right=True).clamp_(max=V - 1))
        drafts.append(x)
        qs.append(q.float())
        tok = torch.tensor([x], dtype=torch.int32, device="cuda:0")
        vf.vf_seq_set_len(seq, len0 + i + 1)
    vf.vf_seq_set_len(seq, len0)
    return drafts, torch.stack(qs).contiguous()


def cpu_baseline(cfg, wd, ctx_len, k, temperature):
    """The oracle's verify + accept on the host: 4 of the 28 layers plus the full output head and
    acceptance are timed on a cache of ctx_len random rows (about 5 s of repeats each for the
    0-layer and the 4-layer model), and the step is extrapolated linearly in the layer count."""
    import oracle
    from oracle.transformer import LayerWeights
    import workloads as wl
    cores = len(os.sched_getaffinity(0))
    rng = np.random.default_rng(7)
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    layers = [LayerWeights(**{n: f64(v) for n, v in lw.items()}) for lw in wd["layers"][:4]]
    embed, fnorm = f64(wd["embed"]), f64(wd["final_norm"])
    m = k + 1
    toks = rng.integers(0, cfg.vocab, m)
    q = rng.dirichlet(np.full(cfg.vocab, 0.05), size=k).astype(np.float32)
    u = wl.make_uniforms(m, rng)
    times = {}
    for nl in (0, 4):
        spec = oracle.ModelSpec(nl, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                                cfg.vocab, cfg.dtype, cfg.rope_theta, cfg.rms_eps)
        w = oracle.Weights(embed, fnorm, layers[:nl])
        cache = oracle.KVCache(spec, ctx_len + m)
        if nl:
            cache.k[:, :, :ctx_len] = oracle.round_bf16(rng.standard_normal(cache.k[:, :, :ctx_len].shape))
            cache.v[:, :, :ctx_len] = oracle.round_bf16(rng.standard_normal(cache.v[:, :, :ctx_len].shape))
        best, t_start = [], time.perf_counter()
        while len(best) < 3 or time.perf_counter() - t_start < 5.0:
            cache.len = ctx_len
            t0 = time.perf_counter()
            z = oracle.verify(spec, w, cache, toks[0], toks[1:])
            oracle.stochastic_accept(z.astype(np.float32), toks[1:], q, u, temperature)
            best.append(time.perf_counter() - t0)
        times[nl] = float(np.median(best))
    per_layer = (times[4] - times[0]) / 4
    full = times[0] + cfg.n_layers * per_layer
    return {"value": round(full * 1e6, 1), "unit": "us/step", "cores": cores, "kind": "oracle",
            "sample": f"numpy float64 oracle verify+accept, {m} rows, ctx {ctx_len}: 4 of {cfg.n_layers} "
                      f"layers ({per_layer * 1e3:.1f} ms/layer) + full output head and acceptance "
                      f"({times[0] * 1e3:.1f} ms), extrapolated linearly to {cfg.n_layers} layers"}


def wl_depths(parents):
    d = [0] * len(parents)
    for i in range(1, len(parents)):
        d[i] = d[parents[i]] + 1
    return d


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="1.5b_k16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--persistent", type=int, default=None,
                    help="1: the persistent whole-pass kernel, 0: one kernel per GEMM (default: the library's default)")
    ap.add_argument("--no-side-measurements", action="store_true",
                    help="skip the tree step, the top-k prefill and the prefill through the verify shape (profile "
                         "runs: every launch of the step's kernel then belongs to the timed workload)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="for counter-collection runs: also run one plain 1 GiB device copy (the yardstick for hardware "
                         "byte counters) and skip the side measurements (tree step, top-k prefill)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the draft-verify step is a single-GPU path here "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    import paper_2510_15312_amd as vf

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(3)
    cfg = wl.CONFIGS[args.config]
    k, m, K, W = cfg.k, cfg.k + 1, args.steps, args.warmup
    n_traj = max(K, W)
    cap = (cfg.ctx + (n_traj + 1) * m + 63) // 64 * 64
    model, wd = build_model(cfg, vf, wl, torch, max(cfg.chunk, m), cap)
    if args.persistent is not None:
        vf.vf_set_option(model, vf.VF_OPT_PERSISTENT, args.persistent)
    s = wl.streams(cfg)
    V = cfg.vocab
    stochastic = cfg.mode == "stochastic"
    temp = cfg.temperature if stochastic else 0.0

    # ---- chunked prefill (untimed here) -----------------------------------------------------
    seq = vf.vf_seq_create(model, cap)
    ctx = torch.as_tensor(wl.make_context(V, cfg.ctx, s.context), device="cuda:0")
    u0 = torch.as_tensor(wl.make_uniforms(1, s.uniforms)[:1], device="cuda:0")
    # twice: the first pass also loads the kernels; the second one, over the same positions, is timed
    for timed in (False, True):
        vf.vf_seq_set_len(seq, 0)
        torch.cuda.synchronize()
        t0 = time.time()
        for c0 in range(0, cfg.ctx, cfg.chunk):
            last = c0 + cfg.chunk >= cfg.ctx
            vf.vf_prefill_chunk(model, seq, ctx[c0:c0 + cfg.chunk], sample_first=last, u=u0, temperature=temp)
        torch.cuda.synchronize()
        prefill_ms = (time.time() - t0) * 1e3
    len0, pending0 = vf.vf_seq_get_state(seq)
    assert len0 == cfg.ctx
    # flops of the chunked prefill: every layer weight twice per token, plus Q K^T and P V over the causal context
    layer_params = (cfg.weight_bytes() - V * cfg.d_model * 2) // 2
    prefill_flops = 2.0 * cfg.ctx * layer_params + \
        4.0 * cfg.n_layers * cfg.n_q_heads * cfg.head_dim * (cfg.ctx * (cfg.ctx + 1) / 2)
    log(f"[bench] prefill of {cfg.ctx} tokens: {prefill_ms:.1f} ms")

    # ---- trajectory pre-pass: generates every step's inputs, leaves them in HBM ----------------
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(15312 * 10 + cfg.index)
    steps_in, lens = [], []
    n_acc = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    out_t = torch.zeros(m, dtype=torch.int32, device="cuda:0")
    y_t = torch.zeros(m, dtype=torch.int32, device="cuda:0")
    pending = pending0
    acc_ref = []
    for i in range(n_traj):
        ln, pending = vf.vf_seq_get_state(seq)
        lens.append(ln)
        if stochastic:
            drafts, q = draft_with_distribution(vf, torch, model, seq, pending, k, temp, 0.5, gen)
            u = torch.as_tensor(wl.make_uniforms(m, s.uniforms), device="cuda:0")
            params = [(vf.VF_STOCHASTIC, temp, q, u)]
        else:
            drafts = wl.copy_span_drafts(ctx.cpu().numpy(), k, cfg.p_copy, V, s.drafts).tolist()
            q = u = None
            params = [(vf.VF_GREEDY, 0.0, None, None)]
        tokens = torch.tensor([pending] + drafts, dtype=torch.int32, device="cuda:0")
        steps_in.append((tokens, params))
        vf.vf_verify(model, [seq], tokens, [0, m])
        vf.vf_accept(model, [seq], tokens, [0, m], params, n_acc, out_t, y_t)
        acc_ref.append(int(n_acc.item()))
    lens.append(vf.vf_seq_get_state(seq)[0])
    log(f"[bench] trajectory: accepted drafts per step mean {np.mean(acc_ref):.2f} of {k}, "
        f"len {lens[0]} -> {lens[-1]}")

    def reset():
        vf.vf_seq_set_len(seq, len0)
        vf.vf_seq_set_pending(seq, pending0)

    def run(n, events=None):
        for i in range(n):
            tokens, params = steps_in[i]
            vf.vf_verify(model, [seq], tokens, [0, m])
            vf.vf_accept(model, [seq], tokens, [0, m], params, n_acc, out_t, y_t)
            if events is not None:
                events[i + 1].record()

    # ---- warm-up, then the timed region ------------------------------------------------------
    reset()
    run(W)
    reset()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    run(K, ev)
    torch.cuda.synchronize()
    total_ms = ev[0].elapsed_time(ev[K])
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(K)]) * 1e3
    ln_end, _ = vf.vf_seq_get_state(seq)

    kvb = cfg.kv_bytes_per_token()
    logit_bytes = 2 * m * V * 4                       # logits written once, read once
    bytes_step = np.array([cfg.weight_bytes() + (lens[i] + m) * kvb + m * kvb + logit_bytes for i in range(K)],
                          dtype=np.float64)
    ms_per_step = total_ms / K
    gbs = float(bytes_step.mean() / (ms_per_step * 1e-3) / 1e9)

    # ---- instrumented pass over the same steps: per-kernel-site durations -----------------------
    reset()
    vf.vf_profile(model, True)
    run(K)
    torch.cuda.synchronize()
    vf.vf_profile(model, False)
    prof = vf.vf_profile_read(model)
    # dominant kernel: the persistent whole-pass kernel when it ran (algorithmic bytes per launch =
    # all weights once + the KV cache read + the new KV rows and the logits written), else the
    # gate/up GEMM of the per-GEMM chain (its weight matrix once)
    if prof["step"][1]:
        kern = "verify_fused_kernel (embedding, 28 decoder layers, output head in one persistent launch)"
        k_bytes = float(np.mean([cfg.weight_bytes() + (lens[i] + m) * kvb + m * kvb + m * V * 4 for i in range(K)]))
        avg_us = prof["step"][0] / prof["step"][1] * 1e3
        traffic = FUSED_TRAFFIC_BYTES
    else:
        kern = "gemm_fast_kernel<2,2,6,EPI_SWIGLU,4> (gate/up GEMM + SwiGLU)"
        k_bytes = float(2 * cfg.d_ffn * cfg.d_model * 2)
        avg_us = prof["gateup"][0] / prof["gateup"][1] * 1e3
        traffic = GATEUP_TRAFFIC_BYTES
    achieved = k_bytes / (avg_us * 1e-6) / 1e9
    site_tbl = {n: {"us_per_step": round(prof[n][0] / K * 1e3, 1), "launches_per_step": prof[n][1] // K}
                for n in prof}
    log("[bench] per-site time per step (instrumented pass): " + json.dumps(site_tbl))

    res = {
        "metric": "verify-step latency (us) + achieved HBM GB/s vs peak, 1.5B shape k=16",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers}L d{cfg.d_model} {cfg.n_q_heads}/{cfg.n_kv_heads} heads "
                               f"hd{cfg.head_dim} ffn{cfg.d_ffn} vocab{V}, ctx {cfg.ctx} prefilled in "
                               f"{cfg.chunk}-token chunks, {K} successive verify steps, k={k} ({m} rows), "
                               f"{cfg.mode} acceptance" + (f" T={temp}, dense draft distribution" if stochastic else ""),
                   "batch": 1, "rows_per_step": m},
        "us_per_step": round(ms_per_step * 1e3, 1),
        "us_per_step_p10_p50_p90": [round(float(np.percentile(per, p)), 1) for p in (10, 50, 90)],
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "algorithmic_bytes_per_step": int(bytes_step.mean()),
        "accepted_drafts_per_step": round(float(np.mean(acc_ref[:K])), 3),
        "us_per_emitted_token": round(ms_per_step * 1e3 / (1 + float(np.mean(acc_ref[:K]))), 1),
        "prefill_ms": round(prefill_ms, 1),
        "prefill": {"tokens": cfg.ctx, "chunk": cfg.chunk, "ms": round(prefill_ms, 1),
                    "TFLOP/s": round(prefill_flops / (prefill_ms * 1e-3) / 1e12, 1),
                    "frac_of_bf16_mfma_peak": round(prefill_flops / (prefill_ms * 1e-3) / 2.5e15, 4)},
        "roofline": {"bound": "hbm", "kernel": kern,
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "avg_launch_us": round(avg_us, 2), "bytes_per_launch": int(k_bytes)},
        "sites_us_per_step": {n: site_tbl[n]["us_per_step"] for n in site_tbl},
    }
    # yardstick: how fast this GPU reads the same weights with nothing else to do
    for _ in range(3):
        nbytes = vf.vf_stream_read(model)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        vf.vf_stream_read(model)
    e1.record()
    torch.cuda.synchronize()
    stream_gbs = nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    res["stream_read"] = {"GB/s": round(stream_gbs, 1), "bytes": nbytes, "frac_of_peak": round(stream_gbs / HBM_PEAK_GBS, 4),
                          "step_vs_stream_read": round(gbs / stream_gbs, 4)}
    # determinism: the timed replay must have walked the recorded trajectory
    assert ln_end == lens[K], (ln_end, lens[K])
    # (skipped in profile runs, whose per-kernel averages should cover the timed workload only)
    if not (args.pmc_calibration or args.no_side_measurements):
        # the same step on tree-structured drafts: m rows as a random tree (chains with side branches),
        # greedy acceptance with compaction of the accepted path; the length is put back before each step
        trng = np.random.default_rng(15312)
        parents = [-1] + [i - 1 if trng.random() > 0.5 else int(trng.integers(0, i)) for i in range(1, m)]
        ttok = torch.as_tensor(trng.integers(0, V, m).astype(np.int32), device="cuda:0")
        path_t = torch.zeros(m, dtype=torch.int32, device="cuda:0")
        tparams = [(vf.VF_GREEDY, 0.0, None, None)]
        reset()

        def tree_step():
            vf.vf_seq_set_len(seq, len0)
            vf.vf_verify_tree(model, [seq], ttok, [0, m], parents)
            vf.vf_accept_tree(model, [seq], ttok, [0, m], parents, tparams, n_acc, out_t, y_t, path_t)

        for _ in range(3):
            tree_step()
        e0.record()
        for _ in range(10):
            tree_step()
        e1.record()
        torch.cuda.synchronize()
        # chunked prefill that also hands back the top-8 successors of every position (the input of the
        # calibration step), against the same prefill returning all logits followed by a library top-k
        seq2 = vf.vf_seq_create(model, cfg.ctx + 8)
        tv = torch.empty((cfg.chunk, 8), dtype=torch.float32, device="cuda:0")
        ti = torch.empty((cfg.chunk, 8), dtype=torch.int32, device="cuda:0")
        zall = torch.empty((cfg.chunk, V), dtype=torch.float32, device="cuda:0")

        def prefill_topk(fused):
            vf.vf_seq_set_len(seq2, 0)
            for c0 in range(0, cfg.ctx, cfg.chunk):
                if fused:
                    vf.vf_prefill_chunk_topk(model, seq2, ctx[c0:c0 + cfg.chunk], 8, tv, ti)
                else:
                    vf.vf_prefill_chunk(model, seq2, ctx[c0:c0 + cfg.chunk], logits_mode=2, logits_out=zall)
                    torch.topk(zall, 8, dim=-1)

        topk_ms = {}
        for fused in (True, False):
            prefill_topk(fused)
            torch.cuda.synchronize()
            t0 = time.time()
            prefill_topk(fused)
            torch.cuda.synchronize()
            topk_ms[fused] = (time.time() - t0) * 1e3
        res["prefill_top8"] = {"ms": round(topk_ms[True], 1), "ms_all_logits_then_library_topk": round(topk_ms[False], 1),
                               "tokens": cfg.ctx, "chunk": cfg.chunk}
        # the same context pushed through the verify path in pieces of 32 rows (what a graph fixed to the
        # verify shape would do with a prefill chunk): 64 passes over the weights instead of 8
        def prefill_by_verify(rows=32):
            vf.vf_seq_set_len(seq2, 0)
            for c0 in range(0, cfg.ctx, rows):
                vf.vf_verify(model, [seq2], ctx[c0:c0 + rows], [0, rows])
                vf.vf_seq_set_len(seq2, c0 + rows)

        prefill_by_verify()
        torch.cuda.synchronize()
        t0 = time.time()
        prefill_by_verify()
        torch.cuda.synchronize()
        res["prefill_top8"]["ms_through_the_verify_path_32_rows"] = round((time.time() - t0) * 1e3, 1)
        del seq2, zall
        res["tree_verify"] = {"us_per_step": round(e0.elapsed_time(e1) * 100.0, 1), "rows": m,
                              "depth": int(max(wl_depths(parents))), "acceptance": "greedy, path compacted"}
    if args.pmc_calibration:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                                  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    if not args.no_cpu_baseline:
        del model
        torch.cuda.empty_cache()
        t0 = time.time()
        res["cpu_baseline"] = cpu_baseline(cfg, wd, cfg.ctx, k, cfg.temperature or 1.0)
        log(f"[bench] cpu baseline took {time.time() - t0:.1f}s")
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
