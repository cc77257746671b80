"""Where the time of one persistent verify launch goes: for every grid barrier, when each of the 256
workgroups arrived and when it left the wait.

Needs a library built with the arrival stamps compiled in (a debug option, off by default):

    VF_HIPCC_FLAGS=-DFUSED_ARRIVALS python -m paper_2510_15312_amd.build
    python -m paper_2510_15312_amd.phase_timeline [config]      # default 1.5b_k16
    python -m paper_2510_15312_amd.build                        # back to the normal build

A phase's time is measured from the last arrival at the barrier before it to the last arrival at the
barrier behind it (the chain of last arrivals is the launch's critical path).  Printed per kind of
phase: that time, how long after the last arrival the median workgroup is released, when the median
and the earliest tenth of the workgroups arrive, and which workgroups arrive last.
"""
import collections
import ctypes as C
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import workloads as wl                      # noqa: E402
import paper_2510_15312_amd as vf           # noqa: E402


def main():
    if not hasattr(vf.lib, "vf_debug_arrivals"):
        sys.exit("libvf.so has no arrival stamps: rebuild with VF_HIPCC_FLAGS=-DFUSED_ARRIVALS (see the module docstring)")
    cfg = wl.CONFIGS[sys.argv[1] if len(sys.argv) > 1 else "1.5b_k16"]
    m = cfg.k + 1
    wd = wl.make_weights(cfg, wl.streams(cfg).weights)
    cap = cfg.ctx + 4 * m
    model = vf.vf_model_create(vf.config_from(cfg, 256, cap), vf.upload_weights(wd, cfg.dtype, "cuda:0"), "cuda:0")
    seq = vf.vf_seq_create(model, cap)
    ctx = torch.as_tensor(wl.make_context(cfg.vocab, cfg.ctx, np.random.default_rng(0)), device="cuda:0")
    for c0 in range(0, cfg.ctx, cfg.chunk):
        vf.vf_prefill_chunk(model, seq, ctx[c0:c0 + cfg.chunk])
    toks = torch.randint(0, cfg.vocab, (m,), dtype=torch.int32, device="cuda:0")
    for _ in range(4):                       # the stamps of the last launch are read; logits stay in the workspace
        vf.vf_verify(model, [seq], toks, [0, m])
    torch.cuda.synchronize()
    L, G = cfg.n_layers, 256
    nb = 1 + 5 * L + 1
    buf = (C.c_ulonglong * (nb * 2 * G))()
    vf.lib.vf_debug_arrivals.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
    if vf.lib.vf_debug_arrivals(model.handle, buf, nb) != 0:
        sys.exit(vf.lib.vf_last_error().decode())
    a = np.array(buf, dtype=np.uint64).reshape(nb, 2, G).astype(np.int64)
    arr, rel = a[:, 0, :] / 100.0, a[:, 1, :] / 100.0          # the clock counts 10 ns
    names = ["embed"] + ["qkv", "attn", "o", "gateup", "down"] * L + ["head"]
    last = arr.max(1)
    print(f"{cfg.name}: {m} rows, context {cfg.ctx}: launch {last[-1] - arr[0].min():.1f} us from the first arrival "
          f"at the first barrier to the end of the output head")
    agg = collections.defaultdict(list)
    for e in range(1, nb):
        agg[names[e]].append((last[e] - last[e - 1], np.median(rel[e - 1]) - last[e - 1],
                              np.median(arr[e]) - last[e - 1], np.percentile(arr[e], 10) - last[e - 1], int(arr[e].argmax())))
    print("| phase | launches | us (last arrival to last arrival) | median release after the last arrival | median workgroup arrives at | earliest tenth at | workgroups most often last |")
    print("|---|---|---|---|---|---|---|")
    total = 0.0
    for kind in ["qkv", "attn", "o", "gateup", "down", "head"]:
        v = np.array([x[:4] for x in agg[kind]])
        who = collections.Counter([x[4] for x in agg[kind]]).most_common(4)
        total += v[:, 0].sum()
        print(f"| {kind} | {len(v)} | {v[:, 0].mean():.2f} | {v[:, 1].mean():.2f} | {v[:, 2].mean():.2f} | {v[:, 3].mean():.2f} | "
              f"{', '.join(str(w) for w, _ in who)} |")
    print(f"sum over all phases {total:.1f} us; per layer {sum(np.array([x[0] for x in agg[k]]).mean() for k in ['qkv', 'attn', 'o', 'gateup', 'down']):.2f} us")


if __name__ == "__main__":
    main()
