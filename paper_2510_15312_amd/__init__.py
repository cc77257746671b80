"""MI355X-native draft-verify step (chunked prefill, k-draft verify, acceptance).

The compute lives in libvf.so (HIP kernels for gfx950 behind a C ABI, see
include/vf.h); this package is its thin ctypes binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS, VfError, Model, Seq, make_config


def upload_weights(wd, dtype, device="cuda:0"):
    """numpy weight dict (float32 arrays, row-major [out, in]) -> device tensors: matrices in the
    model dtype, vectors float32."""
    import numpy as np
    import torch
    mt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def up(a):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        return (t.to(mt) if a.ndim == 2 else t).to(device).contiguous()
    out = {"embed": up(wd["embed"]), "final_norm": up(wd["final_norm"]), "layers": []}
    if wd.get("lm_head") is not None:
        out["lm_head"] = up(wd["lm_head"])
    for lw in wd["layers"]:
        out["layers"].append({k: up(v) for k, v in lw.items()})
    return out


def config_from(cfg, max_rows, max_positions, qkv_bias=False):
    """vf_config from a workloads.WorkloadConfig-like object."""
    return make_config(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                       cfg.vocab, cfg.dtype, cfg.rope_theta, cfg.rms_eps, max_rows, max_positions,
                       qkv_bias=qkv_bias)
