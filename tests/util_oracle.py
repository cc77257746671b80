"""Glue between the workload generators and the oracle (tests only)."""
import numpy as np

import oracle
from oracle.transformer import LayerWeights


def spec_of(cfg, qkv_bias=False):
    return oracle.ModelSpec(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                            cfg.d_ffn, cfg.vocab, cfg.dtype, cfg.rope_theta, cfg.rms_eps, qkv_bias)


def weights_of(wd, dt=np.float64):
    """Workload weight dict -> oracle.Weights in dtype dt."""
    c = lambda a: np.asarray(a, dtype=dt)
    layers = [LayerWeights(**{k: c(v) for k, v in lw.items()}) for lw in wd["layers"]]
    return oracle.Weights(c(wd["embed"]), c(wd["final_norm"]), layers)


def rel_inf(a, b):
    """Per-row inf-norm relative error: max_v |a-b| / max_v |b|."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return np.max(np.abs(a - b), axis=-1) / np.max(np.abs(b), axis=-1)
