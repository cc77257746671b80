// Causal grouped-query attention of the call's rows over the KV cache, split over the keys
// (decode-style): each workgroup handles the query rows of one kv head for one slice of the
// keys and writes (max, sum, weighted V) partials; a second kernel merges the slices by
// log-sum-exp.  Row r of a sequence sits at position len + r and sees keys 0..len + r
// (the verify rows [T, x_1..x_k] of paper Sec. 4.3; a prefill chunk of Sec. 4.1 is the same with
// more rows).
#include "vf_internal.h"

namespace {

constexpr int ATT_THREADS = 128;  // query items (row, head-in-group) per workgroup
constexpr int ATT_TK = 32;        // keys staged in LDS at a time

template <typename T, int HD>
__global__ __launch_bounds__(ATT_THREADS) void attn_partial_kernel(
    Batch b, int layer, const T *__restrict__ q, float *__restrict__ part, int hq, int hkv, int n_splits,
    int chunk, float scale, const tree_mask_t *__restrict__ anc) {
    __shared__ float ks[ATT_TK][HD];
    __shared__ float vs[ATT_TK][HD];
    const int group = hq / hkv;
    const int seq = blockIdx.z / hkv, kvh = blockIdx.z % hkv;
    const SeqDesc &s = b.s[seq];
    const int n_items = s.nrows * group;
    const int item0 = blockIdx.x * ATT_THREADS;
    if (item0 >= n_items) return;
    const int len = s.state[0];
    const int item = item0 + threadIdx.x;
    const bool valid = item < n_items;
    const int r = valid ? item / group : 0, jg = valid ? item % group : 0;
    const int head = kvh * group + jg;
    const int row = s.row0 + r;
    const int last_key = len + r;  // inclusive
    // tree-structured drafts: of the call's own rows (keys len..) only the ancestors are visible
    const tree_mask_t visible_rows = anc && valid ? anc[row] : ~(tree_mask_t)0;
    const int r_max = min(s.nrows - 1, (item0 + ATT_THREADS - 1) / group);
    const int split = blockIdx.y;
    const int k_begin = split * chunk;
    const int k_end = min(k_begin + chunk, min(len + r_max + 1, s.capacity));

    float qv[HD], o[HD];
#pragma unroll
    for (int d = 0; d < HD; ++d) {
        qv[d] = valid ? to_f32(q[((size_t)row * hq + head) * HD + d]) * scale : 0.f;
        o[d] = 0.f;
    }
    float mx = -INFINITY, l = 0.f;
    const T *kv = reinterpret_cast<const T *>(s.kv);

    for (int t0 = k_begin; t0 < k_end; t0 += ATT_TK) {
        const int nt = min(ATT_TK, k_end - t0);
        __syncthreads();
        const int page = kv_page(s, t0), tin0 = t0 % VF_TILE;  // a 32-key tile never straddles a 64 tile
        for (int i = threadIdx.x; i < nt * HD; i += ATT_THREADS) {
            int t = i / HD, d = i % HD;
            ks[t][d] = to_f32(kv[kv_k_index(layer, s.n_pages, page, hkv, kvh, tin0 + t, d, HD)]);
        }
        for (int i = threadIdx.x; i < nt * HD; i += ATT_THREADS) {
            int d = i / nt, t = i % nt;
            vs[t][d] = to_f32(kv[kv_v_index(layer, s.n_pages, page, hkv, kvh, tin0 + t, d, HD)]);
        }
        __syncthreads();
        if (!valid) continue;
        for (int t = 0; t < nt; ++t) {
            if (t0 + t > last_key) break;
            if (anc && t0 + t >= len && !((visible_rows >> (t0 + t - len)) & 1)) continue;
            float sc = 0.f;
#pragma unroll
            for (int d = 0; d < HD; ++d) sc = fmaf(qv[d], ks[t][d], sc);
            if (sc > mx) {
                const float corr = expf(mx - sc);
                l *= corr;
#pragma unroll
                for (int d = 0; d < HD; ++d) o[d] *= corr;
                mx = sc;
            }
            const float p = expf(sc - mx);
            l += p;
#pragma unroll
            for (int d = 0; d < HD; ++d) o[d] = fmaf(p, vs[t][d], o[d]);
        }
    }
    if (!valid) return;
    float *out = part + (((size_t)row * hq + head) * n_splits + split) * (HD + 2);
    out[0] = mx;
    out[1] = l;
#pragma unroll
    for (int d = 0; d < HD; ++d) out[2 + d] = o[d];
}

template <typename T, int HD>
__global__ __launch_bounds__(HD) void attn_combine_kernel(const float *__restrict__ part, T *__restrict__ o,
                                                          int hq, int n_splits, int ncb) {
    const int row = blockIdx.x / hq, head = blockIdx.x % hq, d = threadIdx.x;
    const float *p = part + ((size_t)row * hq + head) * n_splits * (HD + 2);
    float M = -INFINITY;
    for (int s = 0; s < n_splits; ++s) M = fmaxf(M, p[s * (HD + 2)]);
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float w = expf(p[s * (HD + 2)] - M);
        L += p[s * (HD + 2) + 1] * w;
        acc += p[s * (HD + 2) + 2 + d] * w;
    }
    o[act_index<T>(row, head * HD + d, hq * HD, ncb)] = from_f32<T>(acc / L);
}

template <typename T, int HD>
int launch(const vf_model *m, const Batch &b, int layer, const tree_mask_t *anc, hipStream_t st) {
    const vf_config &c = m->cfg;
    const int group = c.n_q_heads / c.n_kv_heads;
    int max_items = 0, max_keys = 0;
    for (int i = 0; i < b.n_seqs; ++i) {
        max_items = max(max_items, b.s[i].nrows * group);
        max_keys = max(max_keys, b.s[i].len_ub + b.s[i].nrows);
    }
    const int tiles = (max_items + ATT_THREADS - 1) / ATT_THREADS;
    const int wgs = tiles * c.n_kv_heads * b.n_seqs;
    int n_splits = (512 + wgs - 1) / wgs;
    n_splits = min(n_splits, (max_keys + VF_TILE - 1) / VF_TILE);
    const int room = ((c.max_rows + 15) / 16 * 16) * 16 / b.total_rows;  // partial buffer: 16 per row of max_rows
    n_splits = max(1, min(n_splits, min(room, 64)));
    int chunk = (max_keys + n_splits - 1) / n_splits;
    chunk = (chunk + VF_TILE - 1) / VF_TILE * VF_TILE;
    const float scale = 1.0f / sqrtf((float)HD);
    hipLaunchKernelGGL((attn_partial_kernel<T, HD>), dim3(tiles, n_splits, b.n_seqs * c.n_kv_heads),
                       dim3(ATT_THREADS), 0, st, b, layer, (const T *)m->q, m->attn_part, c.n_q_heads,
                       c.n_kv_heads, n_splits, chunk, scale, anc);
    VF_LAUNCH_CHECK("attn_partial");
    const int ncb = (b.total_rows + 15) >> 4;
    hipLaunchKernelGGL((attn_combine_kernel<T, HD>), dim3(b.total_rows * c.n_q_heads), dim3(HD), 0, st,
                       m->attn_part, (T *)m->o, c.n_q_heads, n_splits, ncb);
    VF_LAUNCH_CHECK("attn_combine");
    return VF_OK;
}

}  // namespace

int vf_launch_attention(const vf_model *m, const Batch &b, int layer, const tree_mask_t *anc, hipStream_t st) {
    const vf_config &c = m->cfg;
    if (c.dtype == VF_BF16) {
        if (m->fast_path && !anc) return vf_launch_attention_rows(m, b, layer, st);  // MFMA kernel
        if (c.head_dim == 64) return launch<bf16_t, 64>(m, b, layer, anc, st);
        if (c.head_dim == 128) return launch<bf16_t, 128>(m, b, layer, anc, st);
    } else {
        if (c.head_dim == 64) return launch<float, 64>(m, b, layer, anc, st);
        if (c.head_dim == 128) return launch<float, 128>(m, b, layer, anc, st);
    }
    return vf_fail(VF_ERR_UNSUPPORTED, "head_dim %d (built for 64 and 128)", c.head_dim);
}
