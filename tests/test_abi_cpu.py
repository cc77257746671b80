"""The C-ABI library loads without a GPU, exports every function include/vf.h declares, and
its host-side argument checks report errors instead of launching anything (no GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2510_15312_amd as vf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "vf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vf_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported():
    names = _declared()
    assert "vf_prefill_chunk" in names and "vf_verify" in names and "vf_accept" in names
    raw = C.CDLL(vf.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(vf.EXPORTS) == names


def test_constants_match_header():
    text = open(os.path.join(ROOT, "include", "vf.h")).read()
    for name in ("VF_MAX_BATCH", "VF_MAX_DRAFTS", "VF_TOPK_MAX", "VF_F32", "VF_BF16", "VF_GREEDY", "VF_STOCHASTIC"):
        m = re.search(rf"#define\s+{name}\s+\(?(-?\d+)\)?", text)
        assert int(m.group(1)) == getattr(vf, name), name
    assert C.sizeof(vf.binding.vf_config) == 14 * 4
    assert C.sizeof(vf.binding.vf_layer_w) == 12 * 8


def _cfg(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024, vocab=4096,
                dtype="f32", rope_theta=1e4, rms_eps=1e-6, max_rows=128, max_positions=1024)
    base.update(kw)
    return vf.make_config(**base)


def test_packed_bytes_grows_with_the_model_and_counts_the_weights():
    a = vf.vf_model_packed_bytes(_cfg())
    b = vf.vf_model_packed_bytes(_cfg(n_layers=3))
    per_layer = 4 * (3 * 256 * 256 + 256 * 256 + 3 * 1024 * 256)
    assert per_layer <= b - a < per_layer + 16384
    bf = vf.vf_model_packed_bytes(_cfg(dtype="bf16"))
    assert bf < a


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=48), vf.VF_ERR_UNSUPPORTED), (dict(d_model=250), vf.VF_ERR_UNSUPPORTED),
    (dict(vocab=4097), vf.VF_ERR_UNSUPPORTED), (dict(n_kv_heads=3), vf.VF_ERR_ARG),
    (dict(n_layers=0), vf.VF_ERR_ARG), (dict(rope_theta=0.0), vf.VF_ERR_ARG),
    (dict(max_rows=5000), vf.VF_ERR_UNSUPPORTED),
])
def test_bad_configs_are_refused(kw, code):
    cfg = _cfg(**kw)
    assert vf.lib.vf_model_packed_bytes(C.byref(cfg)) == 0
    out = C.c_void_p()
    w = vf.binding.vf_weights()
    rc = vf.lib.vf_model_create(C.byref(cfg), C.byref(w), None, 0, None, C.byref(out))
    assert rc == code, vf.lib.vf_last_error()
    assert vf.lib.vf_last_error()


def test_null_handles_are_errors_not_crashes():
    L = vf.lib
    assert L.vf_model_destroy(None) == vf.VF_ERR_ARG
    assert L.vf_seq_destroy(None) == vf.VF_ERR_ARG
    assert L.vf_seq_set_len(None, 0, None) == vf.VF_ERR_ARG
    assert L.vf_seq_set_pending(None, 0, None) == vf.VF_ERR_ARG
    assert L.vf_seq_get_state(None, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_kv_read(None, None, 0, 0, 0, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_kv_write(None, None, 0, 0, 0, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_stream_read(None, None, None) == vf.VF_ERR_ARG
    assert L.vf_prefill_chunk(None, None, None, 1, 0, None, 0, None, 0.0, None) == vf.VF_ERR_ARG
    assert L.vf_verify(None, None, 1, None, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_accept(None, None, 1, None, None, None, None, None, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_kv_bytes(None, 0, 16) == 0 and L.vf_seq_state_bytes(None) == 0
    cfg = _cfg()
    out = C.c_void_p()
    assert L.vf_model_create(C.byref(cfg), None, None, 0, None, C.byref(out)) == vf.VF_ERR_ARG
    assert b"NULL" in L.vf_last_error()
