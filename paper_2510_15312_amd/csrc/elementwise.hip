// Small kernels around the GEMMs: weight re-packing, rotary tables, embedding gather,
// residual + RMSNorm, the QKV epilogue (bias, rotary embedding, KV append), SwiGLU, and the
// device-side sequence state.  Each adds the split-K partial sums of the GEMM before it in a
// fixed order.
#include "vf_internal.h"

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
namespace {

// ---- model creation -----------------------------------------------------------------------------

// Row-major bf16 [n_rows, K] -> 16x32 fragments; source n-block nb lands at dst block
// dst_nb0 + nb * dst_nb_stride (interleaving gate and up, concatenating q, k, v).
// perm_hd > 0: within every head of perm_hd rows, packed row 2i is source row i and packed row 2i+1
// is source row i + perm_hd/2, so that the two elements of a rotary pair are neighbours.
__device__ inline int pack_src_row(int n, int perm_hd) {
    if (perm_hd <= 0) return n;
    const int head = n / perm_hd, p = n % perm_hd;
    return head * perm_hd + (p >> 1) + (p & 1) * (perm_hd >> 1);
}

__global__ void pack_bf16_kernel(const uint16_t *__restrict__ src, uint4 *__restrict__ dst, int n_rows,
                                 int K, int dst_nb0, int dst_nb_stride, int perm_hd) {
    const int KB = K >> 5;
    size_t total = (size_t)(n_rows >> 4) * KB * 64;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        int lane = (int)(i & 63);
        size_t f = i >> 6;
        int kb = (int)(f % KB), nb = (int)(f / KB);
        int n = pack_src_row(nb * 16 + (lane & 15), perm_hd), k = kb * 32 + (lane >> 4) * 8;
        uint4 v = *reinterpret_cast<const uint4 *>(src + (size_t)n * K + k);
        int dnb = dst_nb0 + nb * dst_nb_stride;
        dst[((size_t)dnb * KB + kb) * 64 + lane] = v;
    }
}

// float32 model: same block re-ordering on plain row-major rows.
__global__ void pack_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, int n_rows, int K,
                                int dst_nb0, int dst_nb_stride, int perm_hd) {
    size_t total = (size_t)n_rows * K;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        int n = (int)(i / K), k = (int)(i % K);
        int dn = (dst_nb0 + (n >> 4) * dst_nb_stride) * 16 + (n & 15);
        dst[(size_t)dn * K + k] = src[(size_t)pack_src_row(n, perm_hd) * K + k];
    }
}

// cos/sin of pos * theta^(-2i/hd), evaluated in float64 and stored as float32.
__global__ void rope_table_kernel(float *__restrict__ cosv, float *__restrict__ sinv, int max_pos, int half,
                                  double theta) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= max_pos * half) return;
    int pos = i / half, j = i % half;
    double inv = pow(theta, -2.0 * (double)j / (double)(2 * half));
    double ang = (double)pos * inv;
    cosv[i] = (float)cos(ang);
    sinv[i] = (float)sin(ang);
}

// ---- forward pass helpers -----------------------------------------------------------------------

template <typename T>
__global__ void embed_kernel(const T *__restrict__ E, const int32_t *__restrict__ tokens, Batch b,
                             float *__restrict__ h, int d, int vocab) {
    const int row = blockIdx.x;
    int tok = tokens[row];
    if (tok == VF_PENDING) tok = b.s[find_seq(b, row)].state[1];
    if (tok < 0 || tok >= vocab) tok = 0;
    for (int k = threadIdx.x; k < d; k += blockDim.x) h[(size_t)row * d + k] = to_f32(E[w_index<T>(tok, k, d)]);
}

__device__ inline float block_sum(float v, float *red) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < nw; ++i) s += red[i];
    __syncthreads();
    return s;
}

// h[row] += sum of partials (if any); x[row] = T(rmsnorm(h[row]) * gain) in activation layout.
template <typename T>
__global__ __launch_bounds__(256) void norm_kernel(float *__restrict__ h, const float *__restrict__ part,
                                                   int nparts, int ld_rows, const float *__restrict__ gain,
                                                   T *__restrict__ x, int d, int ncb, float eps) {
    __shared__ float red[4];
    const int row = blockIdx.x;
    float ss = 0.f;
    for (int k = threadIdx.x; k < d; k += 256) {
        float v = h[(size_t)row * d + k];
        for (int p = 0; p < nparts; ++p) v += part[((size_t)p * ld_rows + row) * d + k];
        if (nparts) h[(size_t)row * d + k] = v;
        ss += v * v;
    }
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    for (int k = threadIdx.x; k < d; k += 256)
        x[act_index<T>(row, k, d, ncb)] = from_f32<T>(h[(size_t)row * d + k] * inv * gain[k]);
}

// The same for bf16 activations with d a multiple of 8: a thread owns runs of eight consecutive
// elements (one 16-byte piece of an activation fragment), keeps them in registers between the
// sum of squares and the scaling, and stores the piece whole.
template <int VPT>
__global__ __launch_bounds__(256) void norm_bf16_vec_kernel(float *__restrict__ h, const float *__restrict__ part,
                                                            int nparts, int ld_rows, const float *__restrict__ gain,
                                                            u32x4_t *__restrict__ x, int d, int ncb, float eps) {
    __shared__ float red[4];
    const int row = blockIdx.x;
    float v[VPT][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int k0 = (threadIdx.x + i * 256) * 8;
        if (k0 < d) {
            float *hp = h + (size_t)row * d + k0;
            const float4 a = *reinterpret_cast<const float4 *>(hp), b = *reinterpret_cast<const float4 *>(hp + 4);
            v[i][0] = a.x; v[i][1] = a.y; v[i][2] = a.z; v[i][3] = a.w;
            v[i][4] = b.x; v[i][5] = b.y; v[i][6] = b.z; v[i][7] = b.w;
            for (int p = 0; p < nparts; ++p) {
                const float *pp = part + ((size_t)p * ld_rows + row) * d + k0;
                const float4 c = *reinterpret_cast<const float4 *>(pp), e = *reinterpret_cast<const float4 *>(pp + 4);
                v[i][0] += c.x; v[i][1] += c.y; v[i][2] += c.z; v[i][3] += c.w;
                v[i][4] += e.x; v[i][5] += e.y; v[i][6] += e.z; v[i][7] += e.w;
            }
            if (nparts) {
                *reinterpret_cast<float4 *>(hp) = float4{v[i][0], v[i][1], v[i][2], v[i][3]};
                *reinterpret_cast<float4 *>(hp + 4) = float4{v[i][4], v[i][5], v[i][6], v[i][7]};
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[i][j] = 0.f;
        }
    }
    // the sum runs over k in the order of the scalar kernel's threads only up to rounding; both
    // are sums of d squares in float32
#pragma unroll
    for (int i = 0; i < VPT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += v[i][j] * v[i][j];
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int k0 = (threadIdx.x + i * 256) * 8;
        if (k0 >= d) continue;
        const float4 ga = *reinterpret_cast<const float4 *>(gain + k0), gb = *reinterpret_cast<const float4 *>(gain + k0 + 4);
        const float gv[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
        u32x4_t out;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bf16_t lo = (bf16_t)(v[i][2 * j] * inv * gv[2 * j]), hi = (bf16_t)(v[i][2 * j + 1] * inv * gv[2 * j + 1]);
            out[j] = (unsigned)__builtin_bit_cast(unsigned short, lo) | ((unsigned)__builtin_bit_cast(unsigned short, hi) << 16);
        }
        const int kb = k0 >> 5, lane = (((k0 >> 3) & 3) << 4) | (row & 15);
        x[((size_t)kb * ncb + (row >> 4)) * 64 + lane] = out;
    }
}

// QKV epilogue: one thread per (row, head, rotary pair).  Heads 0..Hq-1 are q, then Hkv k heads,
// then Hkv v heads (v is not rotated).  Pair = elements (i, i + hd/2) of a head; the packed
// q and k weight rows (and biases) hold a pair in neighbouring columns 2i, 2i+1.
template <typename T>
__global__ void qkv_finish_kernel(const float *__restrict__ part, int nparts, int ld_rows, Batch b, int layer,
                                  const float *__restrict__ bias, const float *__restrict__ cosv,
                                  const float *__restrict__ sinv, T *__restrict__ q, int hq, int hkv, int hd,
                                  const int32_t *__restrict__ depth) {
    const int half = hd >> 1;
    const int heads = hq + 2 * hkv;
    const int per_row = heads * half;
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= b.total_rows * per_row) return;
    const int row = idx / per_row, rem = idx % per_row;
    const int head = rem / half, i = rem % half;
    const int N = heads * hd;
    const bool rot = head < hq + hkv;
    const int n0 = rot ? head * hd + 2 * i : head * hd + i, n1 = rot ? n0 + 1 : n0 + half;
    float v0 = 0.f, v1 = 0.f;
    for (int p = 0; p < nparts; ++p) {
        const float *pr = part + ((size_t)p * ld_rows + row) * N;
        v0 += pr[n0];
        v1 += pr[n1];
    }
    if (bias) { v0 += bias[n0]; v1 += bias[n1]; }
    const SeqDesc &s = b.s[find_seq(b, row)];
    // the rotary angle is that of the token's position; the cache row is the call's row (the two
    // differ for tree-structured drafts, where a node stands at the position of its depth)
    const int slot = s.state[0] + (row - s.row0);
    const int pos = depth ? s.state[0] + depth[row] : slot;
    if (slot < 0 || slot >= s.capacity) return;
    if (rot) {
        const float c = cosv[(size_t)pos * half + i], sn = sinv[(size_t)pos * half + i];
        const float r0 = v0 * c - v1 * sn, r1 = v1 * c + v0 * sn;
        v0 = r0; v1 = r1;
    }
    if (head < hq) {
        T *qr = q + ((size_t)row * hq + head) * hd;
        qr[i] = from_f32<T>(v0);
        qr[i + half] = from_f32<T>(v1);
        return;
    }
    T *kv = reinterpret_cast<T *>(s.kv);
    const int page = kv_page(s, slot), tin = slot % VF_TILE;
    if (head < hq + hkv) {
        const int kh = head - hq;
        kv[kv_k_index(layer, s.n_pages, page, hkv, kh, tin, i, hd)] = from_f32<T>(v0);
        kv[kv_k_index(layer, s.n_pages, page, hkv, kh, tin, i + half, hd)] = from_f32<T>(v1);
    } else {
        const int vh = head - hq - hkv;
        kv[kv_v_index(layer, s.n_pages, page, hkv, vh, tin, i, hd)] = from_f32<T>(v0);
        kv[kv_v_index(layer, s.n_pages, page, hkv, vh, tin, i + half, hd)] = from_f32<T>(v1);
    }
}

// a[row, f] = T(silu(gate) * up); the gate/up GEMM output interleaves 16-wide blocks: block 2j is
// gate rows 16j.., block 2j+1 the matching up rows.
template <typename T>
__global__ void swiglu_kernel(const float *__restrict__ part, int nparts, int ld_rows, T *__restrict__ a,
                              int rows, int F, int ncb) {
    size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (idx >= (size_t)rows * F) return;
    const int row = (int)(idx / F), f = (int)(idx % F);
    const int ng = ((f >> 4) * 2) * 16 + (f & 15), nu = ng + 16;
    float g = 0.f, u = 0.f;
    for (int p = 0; p < nparts; ++p) {
        const float *pr = part + ((size_t)p * ld_rows + row) * (2 * (size_t)F);
        g += pr[ng];
        u += pr[nu];
    }
    const float sg = g / (1.0f + expf(-g));
    a[act_index<T>(row, f, F, ncb)] = from_f32<T>(sg * u);
}

__global__ void reduce_rows_kernel(const float *__restrict__ part, int nparts, int ld_rows, int N, int row_lo,
                                   int nrows, float *__restrict__ out, int out_ld) {
    size_t idx = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    if (idx >= (size_t)nrows * N) return;
    const int r = (int)(idx / N), n = (int)(idx % N);
    float v = 0.f;
    for (int p = 0; p < nparts; ++p) v += part[((size_t)p * ld_rows + row_lo + r) * N + n];
    out[(size_t)r * out_ld + n] = v;
}

__global__ void state_set_kernel(int32_t *state, int idx, int32_t value) { state[idx] = value; }
__global__ void state_add_kernel(int32_t *state, int idx, int32_t delta) { state[idx] += delta; }

template <typename T>
__global__ void kv_read_kernel(SeqDesc s, int layer, int t0, int n, int hkv, int hd, float *__restrict__ k_out,
                               float *__restrict__ v_out) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * hkv * hd) return;
    const int r = idx / (hkv * hd), head = (idx / hd) % hkv, d = idx % hd;
    const int t = t0 + r;
    const T *kv = reinterpret_cast<const T *>(s.kv);
    const int page = kv_page(s, t), tin = t % VF_TILE;
    k_out[idx] = to_f32(kv[kv_k_index(layer, s.n_pages, page, hkv, head, tin, d, hd)]);
    v_out[idx] = to_f32(kv[kv_v_index(layer, s.n_pages, page, hkv, head, tin, d, hd)]);
}

template <typename T>
__global__ void kv_write_kernel(SeqDesc s, int layer, int t0, int n, int hkv, int hd, const float *__restrict__ k_in,
                                const float *__restrict__ v_in) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * hkv * hd) return;
    const int r = idx / (hkv * hd), head = (idx / hd) % hkv, d = idx % hd;
    const int t = t0 + r;
    T *kv = reinterpret_cast<T *>(s.kv);
    const int page = kv_page(s, t), tin = t % VF_TILE;
    kv[kv_k_index(layer, s.n_pages, page, hkv, head, tin, d, hd)] = from_f32<T>(k_in[idx]);
    kv[kv_v_index(layer, s.n_pages, page, hkv, head, tin, d, hd)] = from_f32<T>(v_in[idx]);
}

inline int nblocks(size_t n, int bs) { return (int)((n + bs - 1) / bs); }

__global__ void pack_vec_kernel(const float *__restrict__ src, float *__restrict__ dst, int n, int perm_hd) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[pack_src_row(i, perm_hd)];
}

// Tree-structured drafts: lane r of the sequence's wavefront walks from row r to the root and
// collects the ancestor mask (bit j = row j lies on the path, r itself included) and the depth.
// The host has checked 0 <= parent < r, so the walk ends after at most r steps.
__global__ __launch_bounds__(64) void tree_prep_kernel(Batch b, TreeDesc tree, tree_mask_t *__restrict__ anc,
                                                       int32_t *__restrict__ depth) {
    const SeqDesc &s = b.s[blockIdx.x];
    const int r = threadIdx.x;
    if (r >= s.nrows) return;
    tree_mask_t mask = 0;
    int d = 0;
    for (int a = r, steps = 0; a >= 0 && steps <= VF_MAX_DRAFTS; ++steps) {
        mask |= (tree_mask_t)1 << a;
        const int p = a > 0 ? tree.parent[blockIdx.x][a] : -1;
        if (p >= 0) ++d;
        a = p;
    }
    anc[s.row0 + r] = mask;
    depth[s.row0 + r] = d;
}

// After a tree verify: cache rows of the accepted path go to len_old + 1 .. len_old + a in path
// order (row len_old, the root, stays).  Path rows increase and path[j] >= j, so a destination row
// j can be the source only of an earlier step (path[j'] = j with j' < j).  One thread per (layer,
// kv head, element) copies its element for j = 1, 2, ... in turn: it has read row path[j'] before
// it overwrites that row at step j.
template <typename T>
__global__ void kv_compact_kernel(Batch b, const int32_t *__restrict__ n_accept, const int32_t *__restrict__ path,
                                  int n_layers, int hkv, int hd) {
    const SeqDesc &s = b.s[blockIdx.y];
    const int a = n_accept[blockIdx.y];
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_layers * hkv * hd || a <= 0 || a >= s.nrows) return;
    const int layer = idx / (hkv * hd), head = (idx / hd) % hkv, d = idx % hd;
    const int len_old = s.state[0] - 1 - a;  // the acceptance kernels have already advanced the length
    T *kv = reinterpret_cast<T *>(s.kv);
    for (int j = 1; j <= a; ++j) {
        const int r = path[s.row0 + j];
        if (r == j || r < j || r >= s.nrows) continue;
        const int src = len_old + r, dst = len_old + j;
        if (src >= s.capacity) continue;
        const int ps = kv_page(s, src), pd = kv_page(s, dst);
        kv[kv_k_index(layer, s.n_pages, pd, hkv, head, dst % VF_TILE, d, hd)] =
            kv[kv_k_index(layer, s.n_pages, ps, hkv, head, src % VF_TILE, d, hd)];
        kv[kv_v_index(layer, s.n_pages, pd, hkv, head, dst % VF_TILE, d, hd)] =
            kv[kv_v_index(layer, s.n_pages, ps, hkv, head, src % VF_TILE, d, hd)];
    }
}

}  // namespace

int vf_launch_pack_vec(const float *src, float *dst, int n, int perm_hd, hipStream_t st) {
    hipLaunchKernelGGL(pack_vec_kernel, dim3((n + 255) / 256), dim3(256), 0, st, src, dst, n, perm_hd);
    VF_LAUNCH_CHECK("pack_vec");
    return VF_OK;
}

namespace {
inline int nblocks2(size_t n, int bs) { return (int)((n + bs - 1) / bs); }
}

int vf_launch_pack(const vf_model *m, const void *src, void *dst, int n_rows, int K, int dst_nb0,
                   int dst_nb_stride, int perm_hd, hipStream_t st) {
    if (m->cfg.dtype == VF_BF16) {
        size_t total = (size_t)(n_rows >> 4) * (K >> 5) * 64;
        int grid = (int)((total + 255) / 256 < 65535 ? (total + 255) / 256 : 65535);
        hipLaunchKernelGGL(pack_bf16_kernel, dim3(grid), dim3(256), 0, st, (const uint16_t *)src, (uint4 *)dst,
                           n_rows, K, dst_nb0, dst_nb_stride, perm_hd);
    } else {
        size_t total = (size_t)n_rows * K;
        int grid = (int)((total + 255) / 256 < 65535 ? (total + 255) / 256 : 65535);
        hipLaunchKernelGGL(pack_f32_kernel, dim3(grid), dim3(256), 0, st, (const float *)src, (float *)dst,
                           n_rows, K, dst_nb0, dst_nb_stride, perm_hd);
    }
    VF_LAUNCH_CHECK("pack");
    return VF_OK;
}

int vf_launch_rope_table(const vf_model *m, hipStream_t st) {
    const int half = m->cfg.head_dim / 2, n = m->cfg.max_positions * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3(nblocks(n, 256)), dim3(256), 0, st, m->rope_cos, m->rope_sin,
                       m->cfg.max_positions, half, (double)m->cfg.rope_theta);
    VF_LAUNCH_CHECK("rope_table");
    return VF_OK;
}

int vf_launch_embed(const vf_model *m, const Batch &b, const int32_t *tokens, hipStream_t st) {
    if (m->cfg.dtype == VF_BF16)
        hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(b.total_rows), dim3(256), 0, st, (const bf16_t *)m->embed,
                           tokens, b, m->h, m->cfg.d_model, m->cfg.vocab);
    else
        hipLaunchKernelGGL(embed_kernel<float>, dim3(b.total_rows), dim3(256), 0, st, (const float *)m->embed,
                           tokens, b, m->h, m->cfg.d_model, m->cfg.vocab);
    VF_LAUNCH_CHECK("embed");
    return VF_OK;
}

int vf_launch_norm(const vf_model *m, const float *gain, void *x_out, const float *part, int nparts, int rows,
                   int ld_rows, hipStream_t st) {
    const int ncb = (rows + 15) >> 4;
    const int d = m->cfg.d_model;
    if (m->cfg.dtype == VF_BF16 && d % 8 == 0 && d <= 2048)
        hipLaunchKernelGGL(norm_bf16_vec_kernel<1>, dim3(rows), dim3(256), 0, st, m->h, part, nparts, ld_rows, gain,
                           (u32x4_t *)x_out, d, ncb, m->cfg.rms_eps);
    else if (m->cfg.dtype == VF_BF16 && d % 8 == 0 && d <= 4096)
        hipLaunchKernelGGL(norm_bf16_vec_kernel<2>, dim3(rows), dim3(256), 0, st, m->h, part, nparts, ld_rows, gain,
                           (u32x4_t *)x_out, d, ncb, m->cfg.rms_eps);
    else if (m->cfg.dtype == VF_BF16)
        hipLaunchKernelGGL(norm_kernel<bf16_t>, dim3(rows), dim3(256), 0, st, m->h, part, nparts, ld_rows, gain,
                           (bf16_t *)x_out, m->cfg.d_model, ncb, m->cfg.rms_eps);
    else
        hipLaunchKernelGGL(norm_kernel<float>, dim3(rows), dim3(256), 0, st, m->h, part, nparts, ld_rows, gain,
                           (float *)x_out, m->cfg.d_model, ncb, m->cfg.rms_eps);
    VF_LAUNCH_CHECK("norm");
    return VF_OK;
}

int vf_launch_qkv_finish(const vf_model *m, const Batch &b, int layer, const float *part, int nparts,
                         int ld_rows, const int32_t *depth, hipStream_t st) {
    const vf_config &c = m->cfg;
    const int total = b.total_rows * (c.n_q_heads + 2 * c.n_kv_heads) * (c.head_dim / 2);
    const float *bias = c.qkv_bias ? m->layers[layer].bqkv : nullptr;
    if (c.dtype == VF_BF16)
        hipLaunchKernelGGL(qkv_finish_kernel<bf16_t>, dim3(nblocks(total, 256)), dim3(256), 0, st, part, nparts,
                           ld_rows, b, layer, bias, m->rope_cos, m->rope_sin, (bf16_t *)m->q, c.n_q_heads,
                           c.n_kv_heads, c.head_dim, depth);
    else
        hipLaunchKernelGGL(qkv_finish_kernel<float>, dim3(nblocks(total, 256)), dim3(256), 0, st, part, nparts,
                           ld_rows, b, layer, bias, m->rope_cos, m->rope_sin, (float *)m->q, c.n_q_heads,
                           c.n_kv_heads, c.head_dim, depth);
    VF_LAUNCH_CHECK("qkv_finish");
    return VF_OK;
}

int vf_launch_swiglu(const vf_model *m, const float *part, int nparts, int rows, int ld_rows, hipStream_t st) {
    const int F = m->cfg.d_ffn, ncb = (rows + 15) >> 4;
    const size_t total = (size_t)rows * F;
    if (m->cfg.dtype == VF_BF16)
        hipLaunchKernelGGL(swiglu_kernel<bf16_t>, dim3(nblocks(total, 256)), dim3(256), 0, st, part, nparts,
                           ld_rows, (bf16_t *)m->a, rows, F, ncb);
    else
        hipLaunchKernelGGL(swiglu_kernel<float>, dim3(nblocks(total, 256)), dim3(256), 0, st, part, nparts,
                           ld_rows, (float *)m->a, rows, F, ncb);
    VF_LAUNCH_CHECK("swiglu");
    return VF_OK;
}

int vf_launch_reduce_rows(const vf_model *, const float *part, int nparts, int N, int row_lo, int row_hi,
                          int ld_rows, float *out, int out_ld, hipStream_t st) {
    const int nrows = row_hi - row_lo;
    if (nrows <= 0) return VF_OK;
    hipLaunchKernelGGL(reduce_rows_kernel, dim3(nblocks((size_t)nrows * N, 256)), dim3(256), 0, st, part, nparts,
                       ld_rows, N, row_lo, nrows, out, out_ld);
    VF_LAUNCH_CHECK("reduce_rows");
    return VF_OK;
}

int vf_launch_state_set(int32_t *state, int idx, int32_t value, hipStream_t st) {
    hipLaunchKernelGGL(state_set_kernel, dim3(1), dim3(1), 0, st, state, idx, value);
    VF_LAUNCH_CHECK("state_set");
    return VF_OK;
}
int vf_launch_state_add(int32_t *state, int idx, int32_t delta, hipStream_t st) {
    hipLaunchKernelGGL(state_add_kernel, dim3(1), dim3(1), 0, st, state, idx, delta);
    VF_LAUNCH_CHECK("state_add");
    return VF_OK;
}

namespace {
// Every thread streams 16-byte pieces at a stride of the whole grid; the xor of what it read goes to a
// word nobody reads unless it is a magic value (so the loads cannot be dropped).
__global__ __launch_bounds__(512) void stream_read_kernel(const u32x4_t *__restrict__ p, size_t n, int32_t *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 7 * stride < n; i += 8 * stride) {
        u32x4_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(p + i + j * stride);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
    for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(p + i);
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) *sink = 1;
}
}  // namespace

int vf_launch_stream_read(const vf_model *m, size_t *bytes, hipStream_t st) {
    // the packed weights sit at the start of the model's buffer, up to the rotary tables
    const size_t n = ((const char *)m->rope_cos - (const char *)m->base) / 16;
    hipLaunchKernelGGL(stream_read_kernel, dim3(1024), dim3(512), 0, st, (const u32x4_t *)m->base, n, m->scratch_i32 + 63);
    VF_LAUNCH_CHECK("stream_read");
    *bytes = n * 16;
    return VF_OK;
}

int vf_launch_kv_write(const vf_model *m, const SeqDesc &s, int layer, int t0, int n, const float *k_in,
                       const float *v_in, hipStream_t st) {
    const vf_config &c = m->cfg;
    const int total = n * c.n_kv_heads * c.head_dim;
    if (total <= 0) return VF_OK;
    if (c.dtype == VF_BF16)
        hipLaunchKernelGGL(kv_write_kernel<bf16_t>, dim3(nblocks(total, 256)), dim3(256), 0, st, s, layer, t0, n,
                           c.n_kv_heads, c.head_dim, k_in, v_in);
    else
        hipLaunchKernelGGL(kv_write_kernel<float>, dim3(nblocks(total, 256)), dim3(256), 0, st, s, layer, t0, n,
                           c.n_kv_heads, c.head_dim, k_in, v_in);
    VF_LAUNCH_CHECK("kv_write");
    return VF_OK;
}

int vf_launch_kv_read(const vf_model *m, const SeqDesc &s, int layer, int t0, int n, float *k_out, float *v_out,
                      hipStream_t st) {
    const vf_config &c = m->cfg;
    const int total = n * c.n_kv_heads * c.head_dim;
    if (total <= 0) return VF_OK;
    if (c.dtype == VF_BF16)
        hipLaunchKernelGGL(kv_read_kernel<bf16_t>, dim3(nblocks(total, 256)), dim3(256), 0, st, s, layer, t0, n,
                           c.n_kv_heads, c.head_dim, k_out, v_out);
    else
        hipLaunchKernelGGL(kv_read_kernel<float>, dim3(nblocks(total, 256)), dim3(256), 0, st, s, layer, t0, n,
                           c.n_kv_heads, c.head_dim, k_out, v_out);
    VF_LAUNCH_CHECK("kv_read");
    return VF_OK;
}

int vf_launch_tree_prep(const vf_model *m, const Batch &b, const TreeDesc &tree, hipStream_t st) {
    hipLaunchKernelGGL(tree_prep_kernel, dim3(b.n_seqs), dim3(64), 0, st, b, tree, m->tree_anc, m->tree_depth);
    VF_LAUNCH_CHECK("tree_prep");
    return VF_OK;
}

int vf_launch_kv_compact(const vf_model *m, const Batch &b, const int32_t *n_accept, const int32_t *path,
                         hipStream_t st) {
    const vf_config &c = m->cfg;
    const int total = c.n_layers * c.n_kv_heads * c.head_dim;
    if (c.dtype == VF_BF16)
        hipLaunchKernelGGL(kv_compact_kernel<bf16_t>, dim3(nblocks(total, 256), b.n_seqs), dim3(256), 0, st, b,
                           n_accept, path, c.n_layers, c.n_kv_heads, c.head_dim);
    else
        hipLaunchKernelGGL(kv_compact_kernel<float>, dim3(nblocks(total, 256), b.n_seqs), dim3(256), 0, st, b,
                           n_accept, path, c.n_layers, c.n_kv_heads, c.head_dim);
    VF_LAUNCH_CHECK("kv_compact");
    return VF_OK;
}
