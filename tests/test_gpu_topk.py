"""Top successors of every prefill position through the C ABI: bit-exact against the top-k (oracle
rule) of the library's own all-row logits, on both routes (candidates from the GEMM epilogue for
many rows, from the logits for few rows and float32 models), and against the oracle's logits
wherever the gap to the next value exceeds the logit error."""
import numpy as np
import pytest
import torch

import oracle
from oracle.calibration import topk_rows
import workloads as wl
import paper_2510_15312_amd as vf
from util_gpu import DEV, Pair, tol_of, i32, f32

pytestmark = pytest.mark.gpu
C = wl.CONFIGS
CASES = {
    # name: (config, rows of the chunk, context before it, k)
    "tiny_f32_rows100": (C["tiny_f32"], 100, 37, 8),
    "tiny_f32_rows5": (C["tiny_f32"], 5, 0, 3),
    "1.5b_shape_rows256_epilogue": (wl.scaled(C["1.5b_k16"], n_layers=1, vocab=20000), 256, 64, 8),
    "1.5b_shape_rows200_epilogue": (wl.scaled(C["1.5b_k16"], n_layers=1, vocab=20000), 200, 0, 5),
    "0.5b_shape_rows130_narrow_tile": (wl.scaled(C["0.5b_k8"], n_layers=1, vocab=4096), 130, 10, 1),
    "1.5b_shape_rows40_from_logits": (wl.scaled(C["1.5b_k16"], n_layers=1, vocab=20000), 40, 30, 8),
}


@pytest.mark.parametrize("name", list(CASES))
def test_prefill_topk(name):
    cfg, rows, before, k = CASES[name]
    print(f"case {name}: rows {rows}, context {before}, k {k}", flush=True)
    pair = Pair(cfg, max_rows=256, max_positions=before + rows + 8)
    rng = np.random.default_rng(3)
    ctx = wl.make_context(cfg.vocab, before + rows, rng)
    toks = i32(ctx)
    outs = []
    for use_topk in (False, True):
        seq = pair.new_seq(before + rows + 8)
        if before:
            vf.vf_prefill_chunk(pair.model, seq, toks[:before])
        if use_topk:
            tv = torch.full((rows, k), -7.0, dtype=torch.float32, device=DEV)
            ti = torch.full((rows, k), -7, dtype=torch.int32, device=DEV)
            u = f32([0.37])
            vf.vf_prefill_chunk_topk(pair.model, seq, toks[before:], k, tv, ti, sample_first=True, u=u, temperature=0.8)
            torch.cuda.synchronize()
            outs.append((tv.cpu().numpy(), ti.cpu().numpy(), vf.vf_seq_get_state(seq)))
        else:
            z = torch.empty((rows, cfg.vocab), dtype=torch.float32, device=DEV)
            u = f32([0.37])
            vf.vf_prefill_chunk(pair.model, seq, toks[before:], logits_mode=2, logits_out=z, sample_first=True, u=u,
                                temperature=0.8)
            torch.cuda.synchronize()
            outs.append((z.cpu().numpy(), vf.vf_seq_get_state(seq)))
    (z_gpu, state_plain), (tv, ti, state_topk) = outs
    want_v, want_i = topk_rows(z_gpu, k)
    assert np.array_equal(ti, want_i) and np.array_equal(tv, want_v)
    assert state_topk == state_plain == (before + rows, state_plain[1])      # same length, same first token
    # against the oracle's logits: ids agree wherever the k-th value is clear of the (k+1)-th by more
    # than twice the logit error, and the values agree within the tolerance
    cache = oracle.KVCache(pair.spec, before + rows + 8)
    if before:
        oracle.forward(pair.spec, pair.ow, cache, ctx[:before])
    z_or = oracle.forward(pair.spec, pair.ow, cache, ctx[before:]).astype(np.float32)
    tol = tol_of(cfg)
    ov, oi = topk_rows(z_or, k + 1)
    scale = np.abs(z_or).max(-1)
    # every row: the chosen ids are, by the oracle's logits, within the error margin of its k-th
    # value, and the returned values are the oracle's logits at those ids within the tolerance
    z_at = np.take_along_axis(z_or, ti.astype(np.int64), axis=1)
    assert np.all(z_at >= (ov[:, k - 1] - 2 * tol * scale)[:, None])
    assert np.all(np.abs(tv - z_at) <= tol * scale[:, None])
    # rows whose first k + 1 values are all clear of one another: the same ids in the same order
    clear = np.all(-np.diff(ov, axis=1) > 2 * tol * scale[:, None], axis=1)
    assert np.array_equal(ti[clear], oi[clear, :k])
    print(f"top-{k}: all {rows} rows within the margin of the oracle's top-{k}; {int(clear.sum())} rows with "
          f"clear gaps agree id for id", flush=True)


def test_topk_argument_errors():
    pair = Pair(wl.scaled(C["tiny_f32"], vocab=256), max_rows=64, max_positions=128)
    seq = pair.new_seq(100)
    toks = i32([1, 2, 3])
    tv = torch.zeros((3, 9), dtype=torch.float32, device=DEV)
    ti = torch.zeros((3, 9), dtype=torch.int32, device=DEV)
    for k in (0, vf.VF_TOPK_MAX + 1):
        with pytest.raises(vf.VfError) as e:
            vf.vf_prefill_chunk_topk(pair.model, seq, toks, k, tv, ti)
        assert e.value.code == vf.VF_ERR_ARG
    with pytest.raises(vf.VfError):
        vf.vf_prefill_chunk_topk(pair.model, seq, toks, 4, None, ti)
    assert vf.vf_seq_get_state(seq)[0] == 0
