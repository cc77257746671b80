"""Shared harness of the GPU parity tests: runs the HIP path and the oracle on the same
seeded inputs."""
import numpy as np
import torch

import oracle
from oracle.loop import truncate
import workloads as wl
import paper_2510_15312_amd as vf
from util_oracle import spec_of, weights_of, rel_inf

DEV = "cuda:0"


def tol_of(cfg):
    """Logit tolerance (per-row max abs error over max abs logit): 2e-2 for bfloat16 models,
    1e-5 for float32 models."""
    return 2e-2 if cfg.dtype == "bf16" else 1e-5


def i32(a):
    return torch.as_tensor(np.asarray(a, dtype=np.int32), device=DEV)


def f32(a):
    return torch.as_tensor(np.asarray(a, dtype=np.float32), device=DEV)


class Pair:
    """One model on both sides: oracle (float64) and the HIP library."""

    def __init__(self, cfg, max_rows, max_positions, qkv_bias=False, std=0.02):
        self.cfg = cfg
        self.s = wl.streams(cfg)
        wd = wl.make_weights(cfg, self.s.weights, std=std, qkv_bias=qkv_bias)
        self.spec = spec_of(cfg, qkv_bias)
        self.ow = weights_of(wd)
        self.vcfg = vf.config_from(cfg, max_rows, max_positions, qkv_bias)
        self.dw = vf.upload_weights(wd, cfg.dtype, DEV)
        self.model = vf.vf_model_create(self.vcfg, self.dw, DEV)
        torch.cuda.synchronize()

    def new_seq(self, capacity, pool=None, block_table=None):
        return vf.vf_seq_create(self.model, capacity, pool, block_table, DEV)

    def prefill_both(self, seq, cache, ctx, chunk):
        """Chunked prefill on both sides; returns (oracle last-row logits, GPU last-row logits)."""
        z_or = oracle.prefill(self.spec, self.ow, cache, ctx, chunk)
        out = torch.empty(self.cfg.vocab, dtype=torch.float32, device=DEV)
        toks = i32(ctx)
        for s in range(0, len(ctx), chunk):
            last = s + chunk >= len(ctx)
            vf.vf_prefill_chunk(self.model, seq, toks[s:s + chunk], logits_mode=1 if last else 0,
                                logits_out=out if last else None)
        torch.cuda.synchronize()
        return z_or, out.cpu().numpy()

    def kv_both(self, seq, cache, layer, t0, n):
        k, v = vf.vf_kv_read(self.model, seq, layer, t0, n)
        torch.cuda.synchronize()
        ko = cache.k[layer, :, t0:t0 + n].transpose(1, 0, 2)
        vo = cache.v[layer, :, t0:t0 + n].transpose(1, 0, 2)
        return (k.cpu().numpy(), v.cpu().numpy()), (ko, vo)


def accept_margin_ok(z, drafts, mode, q, u, temperature, eps):
    """True if no decision of the oracle's acceptance on logits z lies within a relative margin
    eps of flipping (arg-max gap for greedy rows that decide; |u q - p| for stochastic)."""
    z = np.asarray(z, dtype=np.float32).astype(np.float64)
    k = len(drafts)
    if mode == "greedy":
        a, _, y = oracle.greedy_accept(z, drafts)
        for i in range(min(a + 1, k + 1)):
            top2 = np.partition(z[i], -2)[-2:]
            if (top2[1] - top2[0]) <= eps * np.abs(z[i]).max():
                return False
        return True
    a, out, _ = oracle.stochastic_accept(z, drafts, q, u, temperature)
    t = np.float64(np.float32(temperature))
    for i in range(min(a + 1, k)):
        e = np.exp((z[i] - z[i].max()) / t)
        p = e / e.sum()
        x = int(drafts[i])
        qx = 1.0 if q is None else float(q[i][x])
        if abs(float(u[i]) * qx - p[x]) <= eps * p[x]:
            return False
    # the replacement / bonus draw: distance of u' * total to the CDF steps around the emitted id
    i = a
    e = np.exp((z[i] - z[i].max()) / t)
    p = e / e.sum()
    if i < k:
        if q is None:
            r = p.copy()
            r[int(drafts[i])] = 0.0
        else:
            r = np.maximum(p - np.asarray(q[i], dtype=np.float64), 0.0)
        if r.sum() == 0.0:
            r = p
    else:
        r = p
    c = np.cumsum(r)
    tgt = float(u[k + 1 + i]) * c[-1]
    w = int(out[-1])
    lo = c[w - 1] if w > 0 else 0.0
    return (c[w] - tgt) > eps * c[-1] and (tgt - lo) >= 0 and ((tgt - lo) > eps * c[-1] or w == 0 or r[:w].sum() == 0)


def gpu_accept(pair, seqs, tokens, row_off, params, logits=None):
    n = len(seqs)
    total = int(row_off[-1])
    n_acc = torch.full((n,), -7, dtype=torch.int32, device=DEV)
    out = torch.full((total,), -7, dtype=torch.int32, device=DEV)
    y = torch.full((total,), -7, dtype=torch.int32, device=DEV)
    vf.vf_accept(pair.model, seqs, tokens, row_off, params, n_acc, out, y, logits)
    torch.cuda.synchronize()
    return n_acc.cpu().numpy(), out.cpu().numpy(), y.cpu().numpy()


def stochastic_margins(z, drafts, q, u, temperature, abs_err):
    """How far the oracle's stochastic decisions on logits z are from flipping, measured against a
    perturbation of every logit by at most abs_err.

    p(x) = exp((z_x - lse) / T): moving every logit by at most abs_err moves log p(x) by at most
    2 * abs_err / T (z_x one way, the normaliser the other), so p(x) changes by a factor within
    exp(+-2 abs_err / T).  A draft's decision u q(x) < p(x) cannot flip if u q(x) lies outside
    [p e^-c, p e^c], c = 2 abs_err / T.  The replacement / bonus draw is safe if u' * total stays
    inside the chosen id's CDF step when every weight changes by that factor (taken as a shift of
    at most (e^c - 1) * total of either edge).

    Returns (n_accept, accept_safe, draw_safe)."""
    z = np.asarray(z, dtype=np.float32).astype(np.float64)
    k = len(drafts)
    t = np.float64(np.float32(temperature))
    c = 2.0 * abs_err / t
    a, out, _ = oracle.stochastic_accept(z, drafts, q, u, temperature)
    accept_safe = True
    for i in range(min(a + 1, k)):
        e = np.exp((z[i] - z[i].max()) / t)
        p = e / e.sum()
        x = int(drafts[i])
        qx = 1.0 if q is None else float(q[i][x])
        uq = float(u[i]) * qx
        if p[x] * np.exp(-c) <= uq <= p[x] * np.exp(c):
            accept_safe = False
    i = a
    e = np.exp((z[i] - z[i].max()) / t)
    p = e / e.sum()
    if i < k:
        if q is None:
            r = p.copy()
            r[int(drafts[i])] = 0.0
        else:
            r = np.maximum(p - np.asarray(q[i], dtype=np.float64), 0.0)
        if r.sum() == 0.0:
            r = p
    else:
        r = p
    cdf = np.cumsum(r)
    tgt = float(u[k + 1 + i]) * cdf[-1]
    w = int(out[-1])
    lo = cdf[w - 1] if w > 0 else 0.0
    shift = np.expm1(c) * cdf[-1]
    draw_safe = bool(accept_safe and (cdf[w] - tgt) > shift and (tgt - lo) > shift)
    if q is not None and i < k:
        draw_safe = False      # a residual max(0, p - q) can change by more than the factor e^c near p = q
    return a, accept_safe, draw_safe
