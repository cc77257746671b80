// Host side of the C ABI: argument checking, memory carving, and the order of kernel launches
// for prefill, verify and accept.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <new>

#include "vf_internal.h"

static thread_local char g_err[512] = "";

int vf_fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char *vf_last_error(void) { return g_err; }

namespace {

struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(char *b) : base(b) {}
    void *take(size_t bytes) {
        off = (off + 255) & ~(size_t)255;
        void *p = base ? base + off : nullptr;
        off += bytes;
        return p;
    }
};

int check_config(const vf_config *c) {
    if (!c) return vf_fail(VF_ERR_ARG, "config is NULL");
    if (c->n_layers < 1 || c->d_model < 32 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 32 ||
        c->vocab < 16 || c->max_rows < 1 || c->max_positions < 1)
        return vf_fail(VF_ERR_ARG, "config: non-positive dimension");
    if (c->dtype != VF_F32 && c->dtype != VF_BF16) return vf_fail(VF_ERR_ARG, "config: dtype %d", c->dtype);
    if (c->n_q_heads % c->n_kv_heads) return vf_fail(VF_ERR_ARG, "config: n_q_heads %% n_kv_heads != 0");
    if (c->head_dim != 64 && c->head_dim != 128)
        return vf_fail(VF_ERR_UNSUPPORTED, "head_dim %d (built for 64 and 128)", c->head_dim);
    if (c->d_model % 32 || c->d_ffn % 32 || (c->n_q_heads * c->head_dim) % 32 || c->vocab % 16)
        return vf_fail(VF_ERR_UNSUPPORTED, "d_model, d_ffn, n_q_heads*head_dim must be multiples of 32, vocab of 16");
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return vf_fail(VF_ERR_ARG, "config: rope_theta / rms_eps");
    if (c->max_rows > 4096) return vf_fail(VF_ERR_UNSUPPORTED, "max_rows %d > 4096", c->max_rows);
    return VF_OK;
}

// Lays the model out in `base` (NULL: only measures).  Returns total bytes.
size_t carve_model(vf_model *m, char *base) {
    const vf_config &c = m->cfg;
    const size_t es = m->es;
    const size_t d = c.d_model, F = c.d_ffn, V = c.vocab, hd = c.head_dim;
    const size_t nq = (size_t)c.n_q_heads * hd, nkv = (size_t)c.n_kv_heads * hd;
    const size_t R = ((size_t)c.max_rows + 15) / 16 * 16;
    Carver cv(base);
    m->embed = cv.take(V * d * es);
    m->lm_head = c.tie_embeddings ? m->embed : cv.take(V * d * es);
    m->final_norm = (float *)cv.take(d * 4);
    for (int l = 0; l < c.n_layers; ++l) {
        LayerPacked lp;
        lp.wqkv = cv.take((nq + 2 * nkv) * d * es);
        lp.wo = cv.take(d * nq * es);
        lp.wgu = cv.take(2 * F * d * es);
        lp.wd = cv.take(d * F * es);
        lp.attn_norm = (float *)cv.take(d * 4);
        lp.ffn_norm = (float *)cv.take(d * 4);
        lp.bqkv = (float *)cv.take((nq + 2 * nkv) * 4);
        if (m->layers) m->layers[l] = lp;
    }
    m->rope_cos = (float *)cv.take((size_t)c.max_positions * (hd / 2) * 4);
    m->rope_sin = (float *)cv.take((size_t)c.max_positions * (hd / 2) * 4);
    const size_t xw = d > nq ? d : nq;
    m->h = (float *)cv.take(R * d * 4);
    m->x = cv.take(R * xw * es);
    m->q = cv.take(R * nq * es);
    m->o = cv.take(R * nq * es);
    m->a = cv.take(R * F * es);
    size_t widest = 2 * F;
    if (nq + 2 * nkv > widest) widest = nq + 2 * nkv;
    m->part_floats = R * widest * 2;  // room for two partials of the widest layer GEMM
    m->part_floats = std::max(m->part_floats, vf_fused_part_floats(c));  // and for the persistent kernel's K splits
    m->part = (float *)cv.take(m->part_floats * 4);
    {
        // general path: 16 slices per row of max_rows; few-row path: up to 48 rows, one slice per 128 keys
        size_t recs = R * c.n_q_heads * 16;
        const size_t few = (size_t)48 * c.n_q_heads * (((size_t)c.max_positions + 127) / 128);
        if (few > recs) recs = few;
        m->attn_part_floats = recs * (hd + 4);
        m->attn_part = (float *)cv.take(recs * (hd + 4) * 4);
    }
    m->logits = (float *)cv.take(R * V * 4);
    m->stat_max = (float *)cv.take(R * VF_STAT_CHUNKS * 4);
    m->stat_idx = (int32_t *)cv.take(R * VF_STAT_CHUNKS * 4);
    m->stat_sum = (double *)cv.take(R * VF_STAT_CHUNKS * 8);
    m->draw = (DrawDesc *)cv.take(sizeof(DrawDesc) * VF_MAX_BATCH);
    m->draw_sums = (double *)cv.take((size_t)VF_MAX_BATCH * VF_STAT_CHUNKS * 8);
    m->scratch_i32 = (int32_t *)cv.take(64 * 4);
    m->ss = (float *)cv.take((d / 16) * 64 * 4);
    m->counters = (int32_t *)cv.take(VF_N_COUNTERS * 4);
    m->topk_cand_v = (float *)cv.take((size_t)R * vf_topk_max_slices(c) * VF_TOPK_MAX * 4);
    m->topk_cand_i = (int32_t *)cv.take((size_t)R * vf_topk_max_slices(c) * VF_TOPK_MAX * 4);
    m->tree_anc = (tree_mask_t *)cv.take((size_t)R * 8);
    m->tree_depth = (int32_t *)cv.take((size_t)R * 4);
    m->fz_ws = (char *)cv.take(vf_fused_workspace_bytes(c));
    return (cv.off + 255) & ~(size_t)255;
}

SeqDesc describe(const vf_seq *s, int row0, int nrows) {
    SeqDesc d;
    d.kv = s->kv;
    d.block_table = s->block_table;
    d.state = s->state;
    d.n_pages = s->n_pages;
    d.capacity = s->capacity;
    d.row0 = row0;
    d.nrows = nrows;
    d.len_ub = s->len_ub;
    d.pad = 0;
    return d;
}

// One pass of the decoder stack over the rows of `b`; leaves the residual stream in m->h with
// the last down-projection still in (part, nparts) form: *tail_parts tells the caller how many
// partial sums the final norm must add.
int run_layers(vf_model *m, const Batch &b, const int32_t *tokens, int *tail_parts, hipStream_t st,
               bool tree = false) {
    const vf_config &c = m->cfg;
    const int rows = b.total_rows, R = rows;  // partials are laid out with ld = rows of this call
    const int d = c.d_model, F = c.d_ffn, nq = c.n_q_heads * c.head_dim, nkv = c.n_kv_heads * c.head_dim;
    int rc;
    if ((rc = vf_launch_embed(m, b, tokens, st))) return rc;
    int nparts = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerPacked &lp = m->layers[l];
        { ProfScope ps(m, VF_SITE_SMALL, st);
          if ((rc = vf_launch_norm(m, lp.attn_norm, m->x, m->part, nparts, rows, R, st))) return rc; }
        GemmPlan p = vf_gemm_plan(m, nq + 2 * nkv, d, rows, 0);
        { ProfScope ps(m, VF_SITE_QKV, st);
          if ((rc = vf_launch_gemm(m, lp.wqkv, m->x, m->part, nq + 2 * nkv, d, rows, 0, rows, R, p, st))) return rc; }
        { ProfScope ps(m, VF_SITE_SMALL, st);
          if ((rc = vf_launch_qkv_finish(m, b, l, m->part, p.ks, R, tree ? m->tree_depth : nullptr, st))) return rc; }
        { ProfScope ps(m, VF_SITE_ATTN, st);
          if ((rc = vf_launch_attention(m, b, l, tree ? m->tree_anc : nullptr, st))) return rc; }
        p = vf_gemm_plan(m, d, nq, rows, 0);
        { ProfScope ps(m, VF_SITE_O, st);
          if ((rc = vf_launch_gemm(m, lp.wo, m->o, m->part, d, nq, rows, 0, rows, R, p, st))) return rc; }
        { ProfScope ps(m, VF_SITE_SMALL, st);
          if ((rc = vf_launch_norm(m, lp.ffn_norm, m->x, m->part, p.ks, rows, R, st))) return rc; }
        // many rows: one K range per workgroup, and the activation function is the GEMM's epilogue
        p = vf_gemm_plan(m, 2 * F, d, rows, 0);
        if (p.tnb) {
            p = vf_gemm_plan(m, 2 * F, d, rows, 1);
            p.swiglu = 1;
        }
        { ProfScope ps(m, VF_SITE_GATEUP, st);
          if ((rc = vf_launch_gemm(m, lp.wgu, m->x, p.swiglu ? (float *)m->a : m->part, 2 * F, d, rows, 0, rows, R, p,
                                   st))) return rc; }
        if (!p.swiglu) {
            ProfScope ps(m, VF_SITE_SMALL, st);
            if ((rc = vf_launch_swiglu(m, m->part, p.ks, rows, R, st))) return rc;
        }
        p = vf_gemm_plan(m, d, F, rows, 0);
        { ProfScope ps(m, VF_SITE_DOWN, st);
          if ((rc = vf_launch_gemm(m, lp.wd, m->a, m->part, d, F, rows, 0, rows, R, p, st))) return rc; }
        nparts = p.ks;
    }
    *tail_parts = nparts;
    return VF_OK;
}

// Final norm + output head for rows [row_lo, row_hi) -> out[(row - row_lo), vocab].
int run_head(vf_model *m, int rows, int tail_parts, int row_lo, int row_hi, float *out, hipStream_t st) {
    const vf_config &c = m->cfg;
    int rc;
    { ProfScope ps(m, VF_SITE_SMALL, st);
      if ((rc = vf_launch_norm(m, m->final_norm, m->x, m->part, tail_parts, rows, rows, st))) return rc; }
    GemmPlan p = vf_gemm_plan(m, c.vocab, c.d_model, rows, 1);
    ProfScope ps(m, VF_SITE_HEAD, st);
    // with ks == 1 the "partial" [ld_rows][V] is the logits matrix itself: shift the base so
    // that row_lo lands on out[0]
    float *base = out - (size_t)row_lo * c.vocab;
    return vf_launch_gemm(m, m->lm_head, m->x, base, c.vocab, c.d_model, rows, row_lo, row_hi, rows, p, st);
}

}  // namespace

extern "C" {

size_t vf_model_packed_bytes(const vf_config *cfg) {
    if (check_config(cfg) != VF_OK) return 0;
    vf_model tmp;
    memset(&tmp, 0, sizeof tmp);
    tmp.cfg = *cfg;
    tmp.es = cfg->dtype == VF_BF16 ? 2 : 4;
    return carve_model(&tmp, nullptr);
}

int vf_model_create(const vf_config *cfg, const vf_weights *w, void *packed_dev, size_t packed_bytes,
                    void *stream, vf_model **out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w || !packed_dev || !out || !w->layers || !w->embed || !w->final_norm)
        return vf_fail(VF_ERR_ARG, "vf_model_create: NULL argument");
    if (!cfg->tie_embeddings && !w->lm_head) return vf_fail(VF_ERR_ARG, "lm_head is NULL but embeddings are not tied");
    if ((uintptr_t)packed_dev & 255) return vf_fail(VF_ERR_ARG, "packed_dev must be 256-byte aligned");
    for (int l = 0; l < cfg->n_layers; ++l) {
        const vf_layer_w &lw = w->layers[l];
        if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.ffn_norm || !lw.w_gate || !lw.w_up ||
            !lw.w_down)
            return vf_fail(VF_ERR_ARG, "layer %d: NULL weight", l);
        if (cfg->qkv_bias && (!lw.bq || !lw.bk || !lw.bv)) return vf_fail(VF_ERR_ARG, "layer %d: NULL bias", l);
    }
    vf_model *m = new (std::nothrow) vf_model;
    if (!m) return vf_fail(VF_ERR_ARG, "out of host memory");
    memset(m, 0, sizeof *m);
    m->cfg = *cfg;
    m->es = cfg->dtype == VF_BF16 ? 2 : 4;
    m->fast_path = 1;
    m->persistent = 1;
    m->prof = new std::vector<vf_model::ProfRec>();
    m->prof_pool = new std::vector<hipEvent_t>();
    m->layers = new (std::nothrow) LayerPacked[cfg->n_layers];
    if (!m->layers) { delete m->prof; delete m->prof_pool; delete m; return vf_fail(VF_ERR_ARG, "out of host memory"); }
    const size_t need = carve_model(m, (char *)packed_dev);
    if (packed_bytes < need) {
        delete[] m->layers; delete m->prof; delete m->prof_pool; delete m;
        return vf_fail(VF_ERR_ARG, "packed buffer too small: %zu < %zu", packed_bytes, need);
    }
    m->base = (char *)packed_dev;
    m->bytes = need;
    hipStream_t st = (hipStream_t)stream;
    const vf_config &c = m->cfg;
    const int d = c.d_model, F = c.d_ffn, hd = c.head_dim, nq = c.n_q_heads * hd, nkv = c.n_kv_heads * hd;
    auto fail = [&](int code) { delete[] m->layers; delete m->prof; delete m->prof_pool; delete m; return code; };
#define TRY(x) do { int rc_ = (x); if (rc_) return fail(rc_); } while (0)
#define TRYHIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) return fail(vf_fail(VF_ERR_HIP, "%s: %s", #x, hipGetErrorString(e_))); } while (0)
    TRY(vf_launch_pack(m, w->embed, m->embed, c.vocab, d, 0, 1, 0, st));
    if (!c.tie_embeddings) TRY(vf_launch_pack(m, w->lm_head, m->lm_head, c.vocab, d, 0, 1, 0, st));
    TRYHIP(hipMemcpyAsync(m->final_norm, w->final_norm, (size_t)d * 4, hipMemcpyDeviceToDevice, st));
    for (int l = 0; l < c.n_layers; ++l) {
        const vf_layer_w &lw = w->layers[l];
        LayerPacked &lp = m->layers[l];
        TRY(vf_launch_pack(m, lw.wq, lp.wqkv, nq, d, 0, 1, hd, st));
        TRY(vf_launch_pack(m, lw.wk, lp.wqkv, nkv, d, nq / 16, 1, hd, st));
        TRY(vf_launch_pack(m, lw.wv, lp.wqkv, nkv, d, (nq + nkv) / 16, 1, 0, st));
        TRY(vf_launch_pack(m, lw.wo, lp.wo, d, nq, 0, 1, 0, st));
        TRY(vf_launch_pack(m, lw.w_gate, lp.wgu, F, d, 0, 2, 0, st));
        TRY(vf_launch_pack(m, lw.w_up, lp.wgu, F, d, 1, 2, 0, st));
        TRY(vf_launch_pack(m, lw.w_down, lp.wd, d, F, 0, 1, 0, st));
        TRYHIP(hipMemcpyAsync(lp.attn_norm, lw.attn_norm, (size_t)d * 4, hipMemcpyDeviceToDevice, st));
        TRYHIP(hipMemcpyAsync(lp.ffn_norm, lw.ffn_norm, (size_t)d * 4, hipMemcpyDeviceToDevice, st));
        if (c.qkv_bias) {
            TRY(vf_launch_pack_vec((const float *)lw.bq, lp.bqkv, nq, hd, st));
            TRY(vf_launch_pack_vec((const float *)lw.bk, lp.bqkv + nq, nkv, hd, st));
            TRY(vf_launch_pack_vec((const float *)lw.bv, lp.bqkv + nq + nkv, nkv, 0, st));
        }
    }
    TRY(vf_launch_rope_table(m, st));
    // activation buffers start at zero so that padding rows of a 16-row block are finite
    TRYHIP(hipMemsetAsync(m->h, 0, (size_t)((char *)m->base + m->bytes - (char *)m->h), st));
    if (c.dtype == VF_BF16) TRY(vf_fused_init(m, m->fz_ws, st));
    TRY(vf_accept_static_init());  // device address of the static acceptance scratch on this GPU
#undef TRY
#undef TRYHIP
    *out = m;
    return VF_OK;
}

int vf_model_destroy(vf_model *m) {
    if (!m) return vf_fail(VF_ERR_ARG, "vf_model_destroy: NULL");
    if (m->prof) {
        for (auto &r : *m->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (auto e : *m->prof_pool) (void)hipEventDestroy(e);
        delete m->prof;
        delete m->prof_pool;
    }
    delete[] m->layers;
    delete m;
    return VF_OK;
}

size_t vf_seq_state_bytes(const vf_model *m) { return m ? 16 : 0; }

size_t vf_kv_bytes(const vf_model *m, int page_tokens, int n) {
    if (!m || n < 1 || (page_tokens != 0 && page_tokens != VF_TILE)) {
        vf_fail(VF_ERR_ARG, "vf_kv_bytes: bad argument");
        return 0;
    }
    const size_t pages = page_tokens ? (size_t)n : ((size_t)n + VF_TILE - 1) / VF_TILE;
    const vf_config &c = m->cfg;
    return pages * c.n_layers * 2 * c.n_kv_heads * VF_TILE * c.head_dim * m->es;
}

int vf_seq_create(vf_model *m, void *kv_dev, size_t kv_bytes, int page_tokens, int pool_pages,
                  int capacity_tokens, const int32_t *block_table_dev, void *state_dev, void *stream,
                  vf_seq **out) {
    if (!m || !kv_dev || !state_dev || !out) return vf_fail(VF_ERR_ARG, "vf_seq_create: NULL argument");
    if (capacity_tokens < 1 || capacity_tokens > m->cfg.max_positions)
        return vf_fail(VF_ERR_ARG, "capacity_tokens %d outside 1..max_positions (%d)", capacity_tokens,
                       m->cfg.max_positions);
    int n_pages;
    if (page_tokens == 0) {
        if (block_table_dev) return vf_fail(VF_ERR_ARG, "contiguous cache takes no block table");
        n_pages = (capacity_tokens + VF_TILE - 1) / VF_TILE;
    } else if (page_tokens == VF_TILE) {
        if (!block_table_dev) return vf_fail(VF_ERR_ARG, "paged cache needs a block table");
        if (pool_pages < (capacity_tokens + VF_TILE - 1) / VF_TILE)
            return vf_fail(VF_ERR_ARG, "pool of %d pages cannot hold %d tokens", pool_pages, capacity_tokens);
        n_pages = pool_pages;
    } else {
        return vf_fail(VF_ERR_UNSUPPORTED, "page_tokens %d (0 or %d)", page_tokens, VF_TILE);
    }
    const size_t need = vf_kv_bytes(m, page_tokens, page_tokens ? n_pages : capacity_tokens);
    if (kv_bytes < need) return vf_fail(VF_ERR_ARG, "kv buffer too small: %zu < %zu", kv_bytes, need);
    vf_seq *s = new (std::nothrow) vf_seq;
    if (!s) return vf_fail(VF_ERR_ARG, "out of host memory");
    s->m = m;
    s->kv = (char *)kv_dev;
    s->block_table = block_table_dev;
    s->state = (int32_t *)state_dev;
    s->n_pages = n_pages;
    s->capacity = capacity_tokens;
    s->paged = page_tokens != 0;
    s->len_ub = 0;
    hipStream_t st = (hipStream_t)stream;
    int rc = vf_launch_state_set(s->state, 0, 0, st);
    if (!rc) rc = vf_launch_state_set(s->state, 1, 0, st);
    if (rc) { delete s; return rc; }
    *out = s;
    return VF_OK;
}

int vf_seq_destroy(vf_seq *s) {
    if (!s) return vf_fail(VF_ERR_ARG, "vf_seq_destroy: NULL");
    delete s;
    return VF_OK;
}

int vf_seq_set_len(vf_seq *s, int len, void *stream) {
    if (!s) return vf_fail(VF_ERR_ARG, "vf_seq_set_len: NULL");
    if (len < 0 || len > s->capacity) return vf_fail(VF_ERR_ARG, "len %d outside 0..%d", len, s->capacity);
    int rc = vf_launch_state_set(s->state, 0, len, (hipStream_t)stream);
    if (rc) return rc;
    s->len_ub = len;
    return VF_OK;
}

int vf_seq_set_pending(vf_seq *s, int32_t token, void *stream) {
    if (!s) return vf_fail(VF_ERR_ARG, "vf_seq_set_pending: NULL");
    if (token < 0 || token >= s->m->cfg.vocab) return vf_fail(VF_ERR_ARG, "token %d outside the vocabulary", token);
    return vf_launch_state_set(s->state, 1, token, (hipStream_t)stream);
}

int vf_seq_get_state(vf_seq *s, int32_t *len_host, int32_t *pending_host, void *stream) {
    if (!s) return vf_fail(VF_ERR_ARG, "vf_seq_get_state: NULL");
    int32_t tmp[2];
    VF_HIP(hipMemcpyAsync(tmp, s->state, sizeof tmp, hipMemcpyDeviceToHost, (hipStream_t)stream));
    VF_HIP(hipStreamSynchronize((hipStream_t)stream));
    if (tmp[0] >= 0 && tmp[0] <= s->capacity) s->len_ub = tmp[0];
    if (len_host) *len_host = tmp[0];
    if (pending_host) *pending_host = tmp[1];
    return vf_fused_check(s->m);
}

int vf_seq_note_len(vf_seq *s, int len) {
    if (!s) return vf_fail(VF_ERR_ARG, "vf_seq_note_len: NULL");
    if (len < 0 || len > s->capacity) return vf_fail(VF_ERR_ARG, "len %d outside 0..%d", len, s->capacity);
    s->len_ub = len;
    return VF_OK;
}

int vf_kv_read(vf_model *m, vf_seq *s, int layer, int t0, int n, float *k_out_dev, float *v_out_dev,
               void *stream) {
    if (!m || !s || !k_out_dev || !v_out_dev) return vf_fail(VF_ERR_ARG, "vf_kv_read: NULL argument");
    if (layer < 0 || layer >= m->cfg.n_layers || t0 < 0 || n < 0 || t0 + n > s->capacity)
        return vf_fail(VF_ERR_ARG, "vf_kv_read: range outside the cache");
    return vf_launch_kv_read(m, describe(s, 0, 0), layer, t0, n, k_out_dev, v_out_dev, (hipStream_t)stream);
}

int vf_kv_write(vf_model *m, vf_seq *s, int layer, int t0, int n, const float *k_in_dev, const float *v_in_dev,
                void *stream) {
    if (!m || !s || !k_in_dev || !v_in_dev) return vf_fail(VF_ERR_ARG, "vf_kv_write: NULL argument");
    if (s->m != m) return vf_fail(VF_ERR_ARG, "sequence belongs to another model");
    if (layer < 0 || layer >= m->cfg.n_layers || t0 < 0 || n < 0 || t0 + n > s->capacity)
        return vf_fail(VF_ERR_ARG, "vf_kv_write: range outside the cache");
    return vf_launch_kv_write(m, describe(s, 0, 0), layer, t0, n, k_in_dev, v_in_dev, (hipStream_t)stream);
}

int vf_prefill_chunk(vf_model *m, vf_seq *s, const int32_t *tokens_dev, int n_tokens, int logits_mode,
                     float *logits_out_dev, int sample_first, const float *u_dev, float temperature,
                     void *stream) {
    if (!m || !s || !tokens_dev) return vf_fail(VF_ERR_ARG, "vf_prefill_chunk: NULL argument");
    if (s->m != m) return vf_fail(VF_ERR_ARG, "sequence belongs to another model");
    if (n_tokens < 1) return vf_fail(VF_ERR_ARG, "n_tokens %d < 1", n_tokens);
    if (n_tokens > m->cfg.max_rows) return vf_fail(VF_ERR_CAP, "n_tokens %d > max_rows %d", n_tokens, m->cfg.max_rows);
    if (logits_mode < 0 || logits_mode > 2) return vf_fail(VF_ERR_ARG, "logits_mode %d", logits_mode);
    if (logits_mode && !logits_out_dev) return vf_fail(VF_ERR_ARG, "logits_out_dev is NULL");
    if (sample_first && temperature < 0.f) return vf_fail(VF_ERR_ARG, "temperature < 0");
    if (sample_first && temperature > 0.f && !u_dev) return vf_fail(VF_ERR_ARG, "u_dev is NULL");
    if (s->len_ub + n_tokens > s->capacity)
        return vf_fail(VF_ERR_CAP, "KV cache: %d + %d > capacity %d", s->len_ub, n_tokens, s->capacity);
    hipStream_t st = (hipStream_t)stream;
    Batch b;
    b.n_seqs = 1;
    b.total_rows = n_tokens;
    b.s[0] = describe(s, 0, n_tokens);
    int tail = 0, rc;
    if ((rc = run_layers(m, b, tokens_dev, &tail, st))) return rc;
    const float *last_row = nullptr;
    if (logits_mode == 2) {
        if ((rc = run_head(m, n_tokens, tail, 0, n_tokens, logits_out_dev, st))) return rc;
        last_row = logits_out_dev + (size_t)(n_tokens - 1) * m->cfg.vocab;
    } else if (logits_mode == 1 || sample_first) {
        float *dst = logits_mode == 1 ? logits_out_dev : m->logits;
        if ((rc = run_head(m, n_tokens, tail, n_tokens - 1, n_tokens, dst, st))) return rc;
        last_row = dst;
    }
    if (sample_first)
        if ((rc = vf_launch_first_token(m, b.s[0], last_row, u_dev, temperature, st))) return rc;
    if ((rc = vf_launch_state_add(s->state, 0, n_tokens, st))) return rc;
    s->len_ub += n_tokens;
    return VF_OK;
}

int vf_prefill_chunk_topk(vf_model *m, vf_seq *s, const int32_t *tokens_dev, int n_tokens, int top_k,
                          float *topk_logit_dev, int32_t *topk_id_dev, int sample_first, const float *u_dev,
                          float temperature, void *stream) {
    if (!m || !s || !tokens_dev || !topk_logit_dev || !topk_id_dev)
        return vf_fail(VF_ERR_ARG, "vf_prefill_chunk_topk: NULL argument");
    if (s->m != m) return vf_fail(VF_ERR_ARG, "sequence belongs to another model");
    if (n_tokens < 1) return vf_fail(VF_ERR_ARG, "n_tokens %d < 1", n_tokens);
    if (n_tokens > m->cfg.max_rows) return vf_fail(VF_ERR_CAP, "n_tokens %d > max_rows %d", n_tokens, m->cfg.max_rows);
    if (top_k < 1 || top_k > VF_TOPK_MAX || top_k > m->cfg.vocab)
        return vf_fail(VF_ERR_ARG, "top_k %d outside 1..%d", top_k, VF_TOPK_MAX);
    if (sample_first && temperature < 0.f) return vf_fail(VF_ERR_ARG, "temperature < 0");
    if (sample_first && temperature > 0.f && !u_dev) return vf_fail(VF_ERR_ARG, "u_dev is NULL");
    if (s->len_ub + n_tokens > s->capacity)
        return vf_fail(VF_ERR_CAP, "KV cache: %d + %d > capacity %d", s->len_ub, n_tokens, s->capacity);
    hipStream_t st = (hipStream_t)stream;
    const vf_config &c = m->cfg;
    Batch b;
    b.n_seqs = 1;
    b.total_rows = n_tokens;
    b.s[0] = describe(s, 0, n_tokens);
    int tail = 0, rc;
    if ((rc = run_layers(m, b, tokens_dev, &tail, st))) return rc;
    { ProfScope ps(m, VF_SITE_SMALL, st);
      if ((rc = vf_launch_norm(m, m->final_norm, m->x, m->part, tail, n_tokens, n_tokens, st))) return rc; }
    GemmPlan p = vf_gemm_plan(m, c.vocab, c.d_model, n_tokens, 1);
    const float *last_row;
    if (p.tnb) {
        // many rows: the candidates leave the GEMM's epilogue, one list per (row, column tile)
        const int n_tiles = (c.vocab / 16 + p.tnb - 1) / p.tnb;
        p.topk = top_k;
        p.topk_ids = m->topk_cand_i;
        { ProfScope ps(m, VF_SITE_HEAD, st);
          if ((rc = vf_launch_gemm(m, m->lm_head, m->x, m->topk_cand_v, c.vocab, c.d_model, n_tokens, 0, n_tokens,
                                   n_tokens, p, st))) return rc; }
        if ((rc = vf_launch_topk_merge(m, n_tokens, n_tiles, top_k, topk_logit_dev, topk_id_dev, st))) return rc;
        if (sample_first) {  // the last row's logits in full, for the draw of the first token
            GemmPlan p1 = vf_gemm_plan(m, c.vocab, c.d_model, n_tokens, 1);
            ProfScope ps(m, VF_SITE_HEAD, st);
            if ((rc = vf_launch_gemm(m, m->lm_head, m->x, m->logits - (size_t)(n_tokens - 1) * c.vocab, c.vocab,
                                     c.d_model, n_tokens, n_tokens - 1, n_tokens, n_tokens, p1, st))) return rc;
        }
        last_row = m->logits;
    } else {
        { ProfScope ps(m, VF_SITE_HEAD, st);
          if ((rc = vf_launch_gemm(m, m->lm_head, m->x, m->logits, c.vocab, c.d_model, n_tokens, 0, n_tokens, n_tokens,
                                   p, st))) return rc; }
        if ((rc = vf_launch_topk_slices(m, m->logits, n_tokens, top_k, st))) return rc;
        if ((rc = vf_launch_topk_merge(m, n_tokens, VF_STAT_CHUNKS, top_k, topk_logit_dev, topk_id_dev, st))) return rc;
        last_row = m->logits + (size_t)(n_tokens - 1) * c.vocab;
    }
    if (sample_first)
        if ((rc = vf_launch_first_token(m, b.s[0], last_row, u_dev, temperature, st))) return rc;
    if ((rc = vf_launch_state_add(s->state, 0, n_tokens, st))) return rc;
    s->len_ub += n_tokens;
    return VF_OK;
}

static int build_batch(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *row_off, Batch *b,
                       const char *who) {
    if (!m || !seqs || !row_off) return vf_fail(VF_ERR_ARG, "%s: NULL argument", who);
    if (n_seqs < 1 || n_seqs > VF_MAX_BATCH) return vf_fail(VF_ERR_ARG, "%s: n_seqs %d outside 1..%d", who, n_seqs, VF_MAX_BATCH);
    if (row_off[0] != 0) return vf_fail(VF_ERR_ARG, "%s: row_off[0] != 0", who);
    b->n_seqs = n_seqs;
    for (int i = 0; i < n_seqs; ++i) {
        if (!seqs[i]) return vf_fail(VF_ERR_ARG, "%s: seqs[%d] is NULL", who, i);
        if (seqs[i]->m != m) return vf_fail(VF_ERR_ARG, "%s: seqs[%d] belongs to another model", who, i);
        for (int j = 0; j < i; ++j)
            if (seqs[j] == seqs[i]) return vf_fail(VF_ERR_ARG, "%s: seqs[%d] repeats seqs[%d]", who, i, j);
        const int rows = row_off[i + 1] - row_off[i];
        if (rows < 1 || rows > VF_MAX_DRAFTS + 1)
            return vf_fail(VF_ERR_ARG, "%s: sequence %d has %d rows (1..%d)", who, i, rows, VF_MAX_DRAFTS + 1);
        b->s[i] = describe(seqs[i], row_off[i], rows);
    }
    b->total_rows = row_off[n_seqs];
    if (b->total_rows > m->cfg.max_rows)
        return vf_fail(VF_ERR_CAP, "%s: %d rows > max_rows %d", who, b->total_rows, m->cfg.max_rows);
    return VF_OK;
}

// parent_host (one entry per row of the call): -1 for the first row of a sequence, else the row,
// counted within the sequence, of the parent node, which must come earlier.
static int build_tree(const Batch &b, const int32_t *parent_host, TreeDesc *tree, const char *who) {
    if (!parent_host) return vf_fail(VF_ERR_ARG, "%s: parent_host is NULL", who);
    memset(tree, 0, sizeof(*tree));
    for (int i = 0; i < b.n_seqs; ++i)
        for (int r = 0; r < b.s[i].nrows; ++r) {
            const int p = parent_host[b.s[i].row0 + r];
            if (r == 0 ? p != -1 : (p < 0 || p >= r))
                return vf_fail(VF_ERR_ARG, "%s: sequence %d row %d has parent %d", who, i, r, p);
            tree->parent[i][r] = (int8_t)p;
        }
    return VF_OK;
}

static int verify_impl(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                       const int32_t *row_off_host, const int32_t *parent_host, bool tree, float *logits_out_dev,
                       void *stream, const char *who) {
    Batch b;
    int rc = build_batch(m, seqs, n_seqs, row_off_host, &b, who);
    if (rc) return rc;
    if (!tokens_dev) return vf_fail(VF_ERR_ARG, "%s: tokens_dev is NULL", who);
    for (int i = 0; i < n_seqs; ++i)
        if (seqs[i]->len_ub + b.s[i].nrows > seqs[i]->capacity)
            return vf_fail(VF_ERR_CAP, "%s: sequence %d: %d + %d > capacity %d", who, i, seqs[i]->len_ub,
                           b.s[i].nrows, seqs[i]->capacity);
    hipStream_t st = (hipStream_t)stream;
    if (tree) {
        TreeDesc td;
        if ((rc = build_tree(b, parent_host, &td, who))) return rc;
        if (m->cfg.head_dim != 64 && m->cfg.head_dim != 128)
            return vf_fail(VF_ERR_UNSUPPORTED, "%s: head_dim %d (built for 64 and 128)", who, m->cfg.head_dim);
        if ((rc = vf_launch_tree_prep(m, b, td, st))) return rc;
    }
    float *dst = logits_out_dev ? logits_out_dev : m->logits;
    if (m->fast_path && m->persistent && vf_fused_ok(m, b)) {
        if ((rc = vf_run_fused(m, b, tokens_dev, dst, tree, st))) return rc;
    } else if (!tree && m->fast_path && vf_fast_path_ok(m, b.total_rows)) {
        if ((rc = vf_run_fast(m, b, tokens_dev, dst, st))) return rc;
    } else {
        int tail = 0;
        if ((rc = run_layers(m, b, tokens_dev, &tail, st, tree))) return rc;
        if ((rc = run_head(m, b.total_rows, tail, 0, b.total_rows, dst, st))) return rc;
    }
    m->last_logits = dst;
    m->last_rows = b.total_rows;
    return VF_OK;
}

int vf_verify(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
              const int32_t *row_off_host, float *logits_out_dev, void *stream) {
    return verify_impl(m, seqs, n_seqs, tokens_dev, row_off_host, nullptr, false, logits_out_dev, stream, "vf_verify");
}

int vf_verify_tree(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                   const int32_t *row_off_host, const int32_t *parent_host, float *logits_out_dev, void *stream) {
    return verify_impl(m, seqs, n_seqs, tokens_dev, row_off_host, parent_host, true, logits_out_dev, stream,
                       "vf_verify_tree");
}

static int accept_impl(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                       const int32_t *row_off_host, const int32_t *parent_host, bool tree, bool static_scratch,
                       const vf_accept_params *params_host, const float *logits_dev, int32_t *n_accept_dev,
                       int32_t *out_tokens_dev, int32_t *y_dev, int32_t *path_dev, void *stream, const char *who) {
    Batch b;
    int rc = build_batch(m, seqs, n_seqs, row_off_host, &b, who);
    if (rc) return rc;
    if (!tokens_dev || !params_host || !n_accept_dev || !out_tokens_dev || !y_dev || (tree && !path_dev))
        return vf_fail(VF_ERR_ARG, "%s: NULL argument", who);
    const float *logits = logits_dev ? logits_dev : m->last_logits;
    if (!logits) return vf_fail(VF_ERR_ARG, "%s: no logits (run the verify first or pass logits_dev)", who);
    if (!logits_dev && m->last_rows != b.total_rows)
        return vf_fail(VF_ERR_ARG, "%s: %d rows but the last verify had %d", who, b.total_rows, m->last_rows);
    TreeDesc td;
    if (tree && (rc = build_tree(b, parent_host, &td, who))) return rc;
    AcceptBatch ab;
    for (int i = 0; i < n_seqs; ++i) {
        const vf_accept_params &p = params_host[i];
        if (p.mode != VF_GREEDY && p.mode != VF_STOCHASTIC) return vf_fail(VF_ERR_ARG, "%s: mode %d", who, p.mode);
        if (p.mode == VF_STOCHASTIC) {
            if (!(p.temperature > 0.f)) return vf_fail(VF_ERR_ARG, "%s: temperature must be > 0", who);
            if (!p.u_dev) return vf_fail(VF_ERR_ARG, "%s: u_dev is NULL", who);
            if (tree && p.q_dev)
                return vf_fail(VF_ERR_UNSUPPORTED, "%s: tree drafts take a deterministic drafter (q_dev NULL)", who);
        }
        if (seqs[i]->len_ub + b.s[i].nrows > seqs[i]->capacity)
            return vf_fail(VF_ERR_CAP, "%s: sequence %d would exceed its capacity", who, i);
        ab.a[i].q = p.q_dev;
        ab.a[i].u = p.u_dev;
        ab.a[i].temperature = p.mode == VF_STOCHASTIC ? p.temperature : 1.f;
        ab.a[i].mode = p.mode;
    }
    {
        ProfScope ps(m, VF_SITE_ACCEPT, (hipStream_t)stream);
        if (tree) {
            if ((rc = vf_launch_accept_tree(m, b, ab, td, tokens_dev, logits, n_accept_dev, out_tokens_dev, y_dev,
                                            path_dev, (hipStream_t)stream)))
                return rc;
            if ((rc = vf_launch_kv_compact(m, b, n_accept_dev, path_dev, (hipStream_t)stream))) return rc;
        } else if (static_scratch) {
            if ((rc = vf_launch_accept_static(m, b, ab, tokens_dev, logits, n_accept_dev, out_tokens_dev, y_dev,
                                              (hipStream_t)stream)))
                return rc;
        } else if ((rc = vf_launch_accept(m, b, ab, tokens_dev, logits, n_accept_dev, out_tokens_dev, y_dev,
                                          (hipStream_t)stream))) {
            return rc;
        }
    }
    for (int i = 0; i < n_seqs; ++i) seqs[i]->len_ub += b.s[i].nrows;
    return VF_OK;
}

int vf_accept(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
              const int32_t *row_off_host, const vf_accept_params *params_host, const float *logits_dev,
              int32_t *n_accept_dev, int32_t *out_tokens_dev, int32_t *y_dev, void *stream) {
    return accept_impl(m, seqs, n_seqs, tokens_dev, row_off_host, nullptr, false, false, params_host, logits_dev,
                       n_accept_dev, out_tokens_dev, y_dev, nullptr, stream, "vf_accept");
}

int vf_accept_static(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                     const int32_t *row_off_host, const vf_accept_params *params_host, const float *logits_dev,
                     int32_t *n_accept_dev, int32_t *out_tokens_dev, int32_t *y_dev, void *stream) {
    return accept_impl(m, seqs, n_seqs, tokens_dev, row_off_host, nullptr, false, true, params_host, logits_dev,
                       n_accept_dev, out_tokens_dev, y_dev, nullptr, stream, "vf_accept_static");
}

int vf_accept_tree(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                   const int32_t *row_off_host, const int32_t *parent_host, const vf_accept_params *params_host,
                   const float *logits_dev, int32_t *n_accept_dev, int32_t *out_tokens_dev, int32_t *y_dev,
                   int32_t *path_dev, void *stream) {
    return accept_impl(m, seqs, n_seqs, tokens_dev, row_off_host, parent_host, true, false, params_host, logits_dev,
                       n_accept_dev, out_tokens_dev, y_dev, path_dev, stream, "vf_accept_tree");
}

int vf_set_option(vf_model *m, int option, int value) {
    if (!m) return vf_fail(VF_ERR_ARG, "vf_set_option: NULL");
    if (option == VF_OPT_FAST_PATH) { m->fast_path = value != 0; return VF_OK; }
    if (option == VF_OPT_PERSISTENT) { m->persistent = value != 0; return VF_OK; }
    return vf_fail(VF_ERR_ARG, "vf_set_option: unknown option %d", option);
}

int vf_stream_read(vf_model *m, size_t *bytes_host, void *stream) {
    if (!m || !bytes_host) return vf_fail(VF_ERR_ARG, "vf_stream_read: NULL argument");
    return vf_launch_stream_read(m, bytes_host, (hipStream_t)stream);
}

int vf_profile(vf_model *m, int enable) {
    if (!m) return vf_fail(VF_ERR_ARG, "vf_profile: NULL");
    m->prof_on = enable != 0;
    return VF_OK;
}

int vf_profile_read(vf_model *m, float *ms_host, int32_t *count_host) {
    if (!m || !ms_host || !count_host) return vf_fail(VF_ERR_ARG, "vf_profile_read: NULL argument");
    for (int i = 0; i < VF_N_SITES; ++i) { ms_host[i] = 0.f; count_host[i] = 0; }
    for (auto &r : *m->prof) {
        VF_HIP(hipEventSynchronize(r.b));
        float ms = 0.f;
        VF_HIP(hipEventElapsedTime(&ms, r.a, r.b));
        ms_host[r.site] += ms;
        count_host[r.site] += 1;
        m->prof_pool->push_back(r.a);
        m->prof_pool->push_back(r.b);
    }
    m->prof->clear();
    return vf_fused_check(m);
}

}  // extern "C"
