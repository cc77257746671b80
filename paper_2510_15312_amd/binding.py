"""ctypes binding of libvf.so: argument marshalling only.

Functions carry the names of the C entry points (include/vf.h).  torch is used
for device memory and for the current HIP stream; every step of the path runs
in the library's kernels.  There is no fallback: if the library is missing the
import fails.
"""
import ctypes as C
import os

import torch  # first: brings the HIP runtime the library links against into the process

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvf.so")

VF_OK, VF_ERR_ARG, VF_ERR_CAP, VF_ERR_HIP, VF_ERR_UNSUPPORTED = 0, -1, -2, -3, -4
VF_F32, VF_BF16 = 0, 1
VF_GREEDY, VF_STOCHASTIC = 0, 1
VF_PENDING = -1
VF_MAX_BATCH, VF_MAX_DRAFTS = 32, 32
VF_TOPK_MAX = 8
VF_ACCEPT_STATIC_MAX_ROWS = 512
VF_OPT_FAST_PATH = 1
VF_OPT_PERSISTENT = 2

EXPORTS = [
    "vf_last_error", "vf_model_packed_bytes", "vf_model_create", "vf_model_destroy",
    "vf_seq_state_bytes", "vf_kv_bytes", "vf_seq_create", "vf_seq_destroy", "vf_seq_set_len",
    "vf_seq_set_pending", "vf_seq_get_state", "vf_seq_note_len", "vf_kv_read", "vf_kv_write", "vf_prefill_chunk", "vf_verify",
    "vf_accept", "vf_accept_static", "vf_profile", "vf_profile_read", "vf_set_option", "vf_stream_read",
    "vf_reuse_select", "vf_reuse_pool_init", "vf_reuse_pool_update", "vf_reuse_pool_extend",
    "vf_verify_tree", "vf_accept_tree", "vf_prefill_chunk_topk", "vf_draft_suffix_match",
]
SITES = ["qkv", "o", "gateup", "down", "head", "attn", "small", "accept", "step"]


class VfError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"vf error {code}: {msg}")
        self.code = code


class vf_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_ffn", "vocab", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("tie_embeddings", "qkv_bias", "max_rows", "max_positions")]


class vf_layer_w(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "wo",
                                          "ffn_norm", "w_gate", "w_up", "w_down")]


class vf_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("layers", C.POINTER(vf_layer_w))]


class vf_accept_params(C.Structure):
    _fields_ = [("mode", C.c_int32), ("temperature", C.c_float), ("q_dev", C.c_void_p),
                ("u_dev", C.c_void_p)]


class vf_reuse_pool(C.Structure):
    _fields_ = [("tokens", C.c_int32 * VF_MAX_DRAFTS)] + \
               [(n, C.c_int32) for n in ("len", "age", "max_age", "cap")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2510_15312_amd.build)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sig = {
        "vf_last_error": (C.c_char_p, []),
        "vf_model_packed_bytes": (sz, [C.POINTER(vf_config)]),
        "vf_model_create": (C.c_int, [C.POINTER(vf_config), C.POINTER(vf_weights), vp, sz, vp, C.POINTER(vp)]),
        "vf_model_destroy": (C.c_int, [vp]),
        "vf_seq_state_bytes": (sz, [vp]),
        "vf_kv_bytes": (sz, [vp, C.c_int, C.c_int]),
        "vf_seq_create": (C.c_int, [vp, vp, sz, C.c_int, C.c_int, C.c_int, vp, vp, vp, C.POINTER(vp)]),
        "vf_seq_destroy": (C.c_int, [vp]),
        "vf_seq_set_len": (C.c_int, [vp, C.c_int, vp]),
        "vf_seq_set_pending": (C.c_int, [vp, i32, vp]),
        "vf_seq_get_state": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32), vp]),
        "vf_seq_note_len": (C.c_int, [vp, C.c_int]),
        "vf_kv_read": (C.c_int, [vp, vp, C.c_int, C.c_int, C.c_int, vp, vp, vp]),
        "vf_kv_write": (C.c_int, [vp, vp, C.c_int, C.c_int, C.c_int, vp, vp, vp]),
        "vf_prefill_chunk": (C.c_int, [vp, vp, vp, C.c_int, C.c_int, vp, C.c_int, vp, C.c_float, vp]),
        "vf_verify": (C.c_int, [vp, C.POINTER(vp), C.c_int, vp, C.POINTER(i32), vp, vp]),
        "vf_accept": (C.c_int, [vp, C.POINTER(vp), C.c_int, vp, C.POINTER(i32), C.POINTER(vf_accept_params),
                                vp, vp, vp, vp, vp]),
        "vf_accept_static": (C.c_int, [vp, C.POINTER(vp), C.c_int, vp, C.POINTER(i32), C.POINTER(vf_accept_params),
                                       vp, vp, vp, vp, vp]),
        "vf_set_option": (C.c_int, [vp, C.c_int, C.c_int]),
        "vf_profile": (C.c_int, [vp, C.c_int]),
        "vf_stream_read": (C.c_int, [vp, C.POINTER(sz), vp]),
        "vf_profile_read": (C.c_int, [vp, C.POINTER(C.c_float), C.POINTER(i32)]),
        "vf_draft_suffix_match": (C.c_int, [C.POINTER(i32), C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(i32)]),
        "vf_prefill_chunk_topk": (C.c_int, [vp, vp, vp, C.c_int, C.c_int, vp, vp, C.c_int, vp, C.c_float, vp]),
        "vf_verify_tree": (C.c_int, [vp, C.POINTER(vp), C.c_int, vp, C.POINTER(i32), C.POINTER(i32), vp, vp]),
        "vf_accept_tree": (C.c_int, [vp, C.POINTER(vp), C.c_int, vp, C.POINTER(i32), C.POINTER(i32),
                                     C.POINTER(vf_accept_params), vp, vp, vp, vp, vp, vp]),
        "vf_reuse_select": (C.c_int, [C.c_int, vp, C.POINTER(i32), vp, vp, vp, vp]),
        "vf_reuse_pool_init": (C.c_int, [C.POINTER(vf_reuse_pool), C.c_int, C.c_int]),
        "vf_reuse_pool_update": (C.c_int, [C.POINTER(vf_reuse_pool), C.POINTER(i32), C.c_int, C.c_int, C.c_int]),
        "vf_reuse_pool_extend": (C.c_int, [C.POINTER(vf_reuse_pool), C.POINTER(i32), C.c_int]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


def _check(rc):
    if rc != VF_OK:
        raise VfError(rc, lib.vf_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Model:
    """Handle of a packed model; keeps the device buffer it lives in alive."""

    def __init__(self, handle, cfg, buf):
        self.handle, self.cfg, self.buf = handle, cfg, buf

    def __del__(self):
        if getattr(self, "handle", None):
            lib.vf_model_destroy(self.handle)
            self.handle = None


class Seq:
    """Handle of a sequence; keeps its KV memory, block table and state alive."""

    def __init__(self, handle, model, kv, state, block_table, capacity):
        self.handle, self.model, self.kv, self.state = handle, model, kv, state
        self.block_table, self.capacity = block_table, capacity

    def __del__(self):
        if getattr(self, "handle", None):
            lib.vf_seq_destroy(self.handle)
            self.handle = None


def make_config(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype, rope_theta,
                rms_eps, max_rows, max_positions, qkv_bias=False, tie_embeddings=True):
    return vf_config(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                     VF_BF16 if dtype in ("bf16", VF_BF16) else VF_F32, rope_theta, rms_eps,
                     int(tie_embeddings), int(qkv_bias), max_rows, max_positions)


def vf_model_packed_bytes(cfg):
    n = lib.vf_model_packed_bytes(C.byref(cfg))
    if n == 0:
        raise VfError(VF_ERR_ARG, lib.vf_last_error().decode())
    return n


def vf_model_create(cfg, weights, device="cuda:0"):
    """weights: dict like workloads.make_weights but of torch DEVICE tensors (matrices in the
    model dtype, vectors float32)."""
    layers = (vf_layer_w * cfg.n_layers)()
    for l, lw in enumerate(weights["layers"]):
        for name, _ in vf_layer_w._fields_:
            setattr(layers[l], name, lw[name].data_ptr() if lw.get(name) is not None else None)
    lm = weights.get("lm_head")
    w = vf_weights(weights["embed"].data_ptr(), lm.data_ptr() if lm is not None else None,
                   weights["final_norm"].data_ptr(), layers)
    nbytes = vf_model_packed_bytes(cfg)
    buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
    out = C.c_void_p()
    _check(lib.vf_model_create(C.byref(cfg), C.byref(w), _ptr(buf), nbytes, _stream(), C.byref(out)))
    return Model(out, cfg, buf)


def vf_kv_bytes(model, page_tokens, n):
    b = lib.vf_kv_bytes(model.handle, page_tokens, n)
    if b == 0:
        raise VfError(VF_ERR_ARG, lib.vf_last_error().decode())
    return b


def vf_seq_create(model, capacity, pool=None, block_table=None, device="cuda:0"):
    """Contiguous cache (pool None: allocated here) or paged (pool = uint8 tensor of
    vf_kv_bytes(model, 64, n_pages), block_table = int32 device tensor)."""
    state = torch.empty(lib.vf_seq_state_bytes(model.handle), dtype=torch.uint8, device=device)
    out = C.c_void_p()
    if pool is None:
        kv = torch.empty(vf_kv_bytes(model, 0, capacity), dtype=torch.uint8, device=device)
        rc = lib.vf_seq_create(model.handle, _ptr(kv), kv.numel(), 0, 0, capacity, None, _ptr(state),
                               _stream(), C.byref(out))
    else:
        kv = pool
        es = 2 if model.cfg.dtype == VF_BF16 else 4
        page_bytes = model.cfg.n_layers * 2 * model.cfg.n_kv_heads * 64 * model.cfg.head_dim * es
        rc = lib.vf_seq_create(model.handle, _ptr(kv), kv.numel(), 64, kv.numel() // page_bytes, capacity,
                               _ptr(block_table), _ptr(state), _stream(), C.byref(out))
    _check(rc)
    return Seq(out, model, kv, state, block_table, capacity)


def vf_seq_set_len(seq, n):
    _check(lib.vf_seq_set_len(seq.handle, n, _stream()))


def vf_seq_set_pending(seq, token):
    _check(lib.vf_seq_set_pending(seq.handle, token, _stream()))


def vf_seq_get_state(seq):
    a, b = C.c_int32(), C.c_int32()
    _check(lib.vf_seq_get_state(seq.handle, C.byref(a), C.byref(b), _stream()))
    return a.value, b.value


def vf_seq_note_len(seq, n):
    """Host only: tightens the host-side bound of the length to the true length n."""
    _check(lib.vf_seq_note_len(seq.handle, int(n)))


def vf_kv_read(model, seq, layer, t0, n):
    shape = (n, model.cfg.n_kv_heads, model.cfg.head_dim)
    k = torch.empty(shape, dtype=torch.float32, device=seq.state.device)
    v = torch.empty(shape, dtype=torch.float32, device=seq.state.device)
    _check(lib.vf_kv_read(model.handle, seq.handle, layer, t0, n, _ptr(k), _ptr(v), _stream()))
    return k, v


def vf_kv_write(model, seq, layer, t0, k, v):
    """k, v: float32 device tensors [n, n_kv_heads, head_dim]."""
    _check(lib.vf_kv_write(model.handle, seq.handle, layer, t0, k.shape[0], _ptr(k), _ptr(v), _stream()))


def vf_prefill_chunk(model, seq, tokens, logits_mode=0, logits_out=None, sample_first=False, u=None,
                     temperature=0.0):
    """tokens: int32 device tensor [n]."""
    _check(lib.vf_prefill_chunk(model.handle, seq.handle, _ptr(tokens), tokens.numel(), logits_mode,
                                _ptr(logits_out), int(sample_first), _ptr(u), temperature, _stream()))


def _batch(seqs, row_off):
    hs = (C.c_void_p * len(seqs))(*[s.handle for s in seqs])
    ro = (C.c_int32 * len(row_off))(*[int(r) for r in row_off])
    return hs, ro


def vf_verify(model, seqs, tokens, row_off, logits_out=None):
    """tokens: int32 device tensor [total_rows]; row_off: host ints [n_seqs + 1]."""
    hs, ro = _batch(seqs, row_off)
    _check(lib.vf_verify(model.handle, hs, len(seqs), _ptr(tokens), ro, _ptr(logits_out), _stream()))


def vf_accept(model, seqs, tokens, row_off, params, n_accept, out_tokens, y, logits=None):
    """params: list of (mode, temperature, q tensor or None, u tensor or None) per sequence;
    n_accept int32[n_seqs], out_tokens int32[total_rows], y int32[total_rows]: device tensors."""
    hs, ro = _batch(seqs, row_off)
    ps = (vf_accept_params * len(seqs))()
    for i, (mode, temp, q, u) in enumerate(params):
        ps[i] = vf_accept_params(mode, temp, q.data_ptr() if q is not None else None,
                                 u.data_ptr() if u is not None else None)
    _check(lib.vf_accept(model.handle, hs, len(seqs), _ptr(tokens), ro, ps, _ptr(logits), _ptr(n_accept),
                         _ptr(out_tokens), _ptr(y), _stream()))


def vf_accept_static(model, seqs, tokens, row_off, params, n_accept, out_tokens, y, logits=None):
    """vf_accept with the library's static device scratch; arguments as vf_accept."""
    hs, ro = _batch(seqs, row_off)
    ps = (vf_accept_params * len(seqs))()
    for i, (mode, temp, q, u) in enumerate(params):
        ps[i] = vf_accept_params(mode, temp, q.data_ptr() if q is not None else None,
                                 u.data_ptr() if u is not None else None)
    _check(lib.vf_accept_static(model.handle, hs, len(seqs), _ptr(tokens), ro, ps, _ptr(logits), _ptr(n_accept),
                                _ptr(out_tokens), _ptr(y), _stream()))


def vf_prefill_chunk_topk(model, seq, tokens, top_k, topk_logit, topk_id, sample_first=False, u=None,
                          temperature=0.0):
    """tokens int32[n] (device); topk_logit float32[n, top_k], topk_id int32[n, top_k]: device tensors."""
    _check(lib.vf_prefill_chunk_topk(model.handle, seq.handle, _ptr(tokens), tokens.numel(), int(top_k),
                                     _ptr(topk_logit), _ptr(topk_id), int(bool(sample_first)), _ptr(u),
                                     float(temperature), _stream()))


def vf_verify_tree(model, seqs, tokens, row_off, parents, logits_out=None):
    """As vf_verify; parents: host ints [total_rows], -1 for each sequence's first row, else the
    parent's row within the sequence."""
    hs, ro = _batch(seqs, row_off)
    par = (C.c_int32 * len(parents))(*[int(p) for p in parents])
    _check(lib.vf_verify_tree(model.handle, hs, len(seqs), _ptr(tokens), ro, par, _ptr(logits_out), _stream()))


def vf_accept_tree(model, seqs, tokens, row_off, parents, params, n_accept, out_tokens, y, path, logits=None):
    """As vf_accept, plus path int32[total_rows] (device): the rows of the accepted path."""
    hs, ro = _batch(seqs, row_off)
    par = (C.c_int32 * len(parents))(*[int(p) for p in parents])
    ps = (vf_accept_params * len(seqs))()
    for i, (mode, temp, q, u) in enumerate(params):
        ps[i] = vf_accept_params(mode, temp, q.data_ptr() if q is not None else None,
                                 u.data_ptr() if u is not None else None)
    _check(lib.vf_accept_tree(model.handle, hs, len(seqs), _ptr(tokens), ro, par, ps, _ptr(logits), _ptr(n_accept),
                              _ptr(out_tokens), _ptr(y), _ptr(path), _stream()))


def vf_draft_suffix_match(history, k, max_suffix, min_suffix=1):
    """history: host ints; returns the list of drafts (possibly empty)."""
    n = len(history)
    arr = (C.c_int32 * max(1, n))(*[int(t) for t in history])
    out = (C.c_int32 * VF_MAX_DRAFTS)()
    got = lib.vf_draft_suffix_match(arr, n, int(max_suffix), int(min_suffix), int(k), out)
    if got < 0:
        _check(got)
    return list(out[:got])


def vf_reuse_select(tokens, row_off, y, n_accept, seg):
    """tokens, y int32[total_rows], n_accept int32[n_seqs], seg int32[2 * n_seqs]: device tensors."""
    ro = (C.c_int32 * len(row_off))(*[int(r) for r in row_off])
    _check(lib.vf_reuse_select(len(row_off) - 1, _ptr(tokens), ro, _ptr(y), _ptr(n_accept), _ptr(seg), _stream()))


def vf_reuse_pool_init(max_age, cap=VF_MAX_DRAFTS):
    pool = vf_reuse_pool()
    _check(lib.vf_reuse_pool_init(C.byref(pool), int(max_age), int(cap)))
    return pool


def vf_reuse_pool_update(pool, drafts, seg_start, seg_len):
    """drafts: host ints, the drafts of the step the segment was found in."""
    arr = (C.c_int32 * max(1, len(drafts)))(*[int(t) for t in drafts])
    _check(lib.vf_reuse_pool_update(C.byref(pool), arr, len(drafts), int(seg_start), int(seg_len)))


def vf_reuse_pool_extend(pool, fresh):
    """Returns the drafts of the next step: the fresh ones, then the held segment if it fits."""
    arr = (C.c_int32 * VF_MAX_DRAFTS)(*[int(t) for t in fresh])
    n = lib.vf_reuse_pool_extend(C.byref(pool), arr, len(fresh))
    if n < 0:
        _check(n)
    return list(arr[:n])


def vf_profile(model, enable):
    _check(lib.vf_profile(model.handle, int(enable)))


def vf_profile_read(model):
    """{site: (total ms, launch groups)} since the last read."""
    ms = (C.c_float * len(SITES))()
    cnt = (C.c_int32 * len(SITES))()
    _check(lib.vf_profile_read(model.handle, ms, cnt))
    return {s: (ms[i], cnt[i]) for i, s in enumerate(SITES)}


def vf_stream_read(model):
    """Launches the read-every-weight yardstick kernel; returns the bytes it reads."""
    n = C.c_size_t(0)
    _check(lib.vf_stream_read(model.handle, C.byref(n), _stream()))
    return n.value


def vf_set_option(model, option, value):
    _check(lib.vf_set_option(model.handle, option, int(value)))
