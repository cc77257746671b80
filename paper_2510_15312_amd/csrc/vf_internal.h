// Internal declarations shared by the translation units of libvf.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "vf.h"

#include <string.h>
#include <vector>

#define VF_TILE 64            // tokens per KV tile / page
#define VF_ATTN_SPLIT_MAX 128 // most key slices one query row can have
#define VF_STAT_CHUNKS 64     // vocabulary chunks of the row-statistics pass (one per lane)

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// ---- per-call description of the batch, passed to kernels by value --------------------------
struct SeqDesc {
    char *kv;                   // KV pool base
    const int32_t *block_table; // NULL: page id = tile index
    int32_t *state;             // [0] = length, [1] = pending token
    int32_t n_pages;            // pages in the pool (contiguous: tiles of this sequence)
    int32_t capacity;           // tokens this sequence may hold
    int32_t row0, nrows;        // its rows inside the call
    int32_t len_ub;             // host upper bound of the length before this call
    int32_t pad;
};
struct Batch {
    int32_t n_seqs, total_rows;
    SeqDesc s[VF_MAX_BATCH];
};

// Tree-structured drafts: parent row (within the sequence) of every row; -1 for row 0.
struct TreeDesc {
    int8_t parent[VF_MAX_BATCH][VF_MAX_DRAFTS + 1];
};
typedef unsigned long long tree_mask_t;  // bit j: row j of the sequence is an ancestor of (or is) this row

struct AcceptDesc {
    const float *q;             // [k, V] or NULL
    const float *u;             // [2*(k+1)]
    float temperature;
    int32_t mode;
};
struct AcceptBatch {
    AcceptDesc a[VF_MAX_BATCH];
};
// what the decide kernel leaves for the replacement / bonus draw of one sequence
struct DrawDesc {
    double zmax, S, u, t;       // row maximum, softmax normaliser, uniform, temperature
    const float *q;             // draft distribution row or NULL
    int32_t row, x_excl, active, acc;
    int32_t n_excl;             // tree verification: tokens of the refused children of the deciding node
    int32_t excl[VF_MAX_DRAFTS];
};

// ---- model / sequence host structs ------------------------------------------------------------
struct LayerPacked {
    void *wqkv, *wo, *wgu, *wd; // packed matrices
    float *attn_norm, *ffn_norm, *bqkv;
};

struct vf_model {
    vf_config cfg;
    int es;                     // bytes per element of the model dtype
    char *base;
    size_t bytes;
    LayerPacked *layers;        // host array
    void *embed, *lm_head;
    float *final_norm, *rope_cos, *rope_sin;
    // workspace
    float *h;                   // residual stream [R, d]
    void *x;                    // GEMM input (activation layout) [R, max(d, Hq*hd)]
    void *q;                    // [R, Hq*hd] row-major
    void *o;                    // attention output (activation layout) [R, Hq*hd]
    void *a;                    // SwiGLU product (activation layout) [R, F]
    float *part;                // split-K partial sums
    size_t part_floats;
    float *attn_part;           // [R*Hq, 16, hd+4]
    size_t attn_part_floats;
    float *logits;              // [R, V]
    float *stat_max;            // [R, VF_STAT_CHUNKS]
    int32_t *stat_idx;          // [R, VF_STAT_CHUNKS]
    double *stat_sum;           // [R, VF_STAT_CHUNKS]
    DrawDesc *draw;             // [VF_MAX_BATCH]
    double *draw_sums;          // [VF_MAX_BATCH, VF_STAT_CHUNKS]
    int32_t *scratch_i32;       // [64]
    float *ss;                  // per-16-column sums of squares of h rows, [d/16][64]
    int32_t *counters;          // split-K arrival counters, [VF_N_COUNTERS], zero between kernels
    float *topk_cand_v;         // top-k candidates per (row, vocabulary slice), [R, slices, VF_TOPK_MAX]
    int32_t *topk_cand_i;
    tree_mask_t *tree_anc;      // tree verify: ancestor mask of every row of the call, [R]
    int32_t *tree_depth;        // tree verify: depth of every row, [R]
    int fast_path;              // option: use the few-row kernels when they apply
    int persistent;             // option: use the persistent whole-pass kernel when it applies
    // persistent kernel: single-assignment activation buffers, barrier counters, layer table
    float *fz_h, *fz_ss, *fz_att;
    void *fz_q, *fz_o, *fz_a, *fz_layers;
    unsigned *fz_bar;
    char *fz_ws;                // their workspace
    unsigned fz_epoch;          // value the barrier's root counter has after all launches so far
    const float *last_logits;   // where the last verify left its logits
    int last_rows;
    // measurement hook
    struct ProfRec { int site; hipEvent_t a, b; };
    bool prof_on;
    std::vector<ProfRec> *prof;       // recorded, not yet read
    std::vector<hipEvent_t> *prof_pool;  // events free for reuse
};

struct vf_seq {
    vf_model *m;
    char *kv;
    const int32_t *block_table;
    int32_t *state;
    int n_pages, capacity, paged;
    int len_ub;                 // host upper bound of the device-side length
};

#define VF_N_COUNTERS 8192

// ---- error handling ----------------------------------------------------------------------------
int vf_fail(int code, const char *fmt, ...);
#define VF_HIP(call)                                                                       \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess) return vf_fail(VF_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)
#define VF_LAUNCH_CHECK(name)                                                              \
    do {                                                                                   \
        hipError_t e_ = hipGetLastError();                                                 \
        if (e_ != hipSuccess) return vf_fail(VF_ERR_HIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// Brackets a launch group with two events when profiling is on.
struct ProfScope {
    vf_model *m;
    hipStream_t st;
    hipEvent_t b = nullptr;
    ProfScope(vf_model *m_, int site, hipStream_t st_) : m(m_), st(st_) {
        if (!m->prof_on) return;
        hipEvent_t ev[2];
        for (int i = 0; i < 2; ++i) {
            if (!m->prof_pool->empty()) { ev[i] = m->prof_pool->back(); m->prof_pool->pop_back(); }
            else if (hipEventCreate(&ev[i]) != hipSuccess) { if (i) m->prof_pool->push_back(ev[0]); return; }
        }
        (void)hipEventRecord(ev[0], st);
        m->prof->push_back({site, ev[0], ev[1]});
        b = ev[1];
    }
    ~ProfScope() { if (b) (void)hipEventRecord(b, st); }
};

// ---- layouts ------------------------------------------------------------------------------------
// Packed bf16 matrix W[N, K]: 16x32 fragments in MFMA A-operand order.  Fragment (nb, kb) holds
// rows 16*nb.. and columns 32*kb..; lane l of a wavefront owns row (l & 15), columns
// 8*(l >> 4) .. +8: eight consecutive bf16 = 16 bytes.  Fragments of one nb are contiguous in kb.
__host__ __device__ inline size_t wfrag_index(int n, int k, int K) {
    int nb = n >> 4, kb = k >> 5;
    int lane = (((k >> 3) & 3) << 4) | (n & 15);
    return (((size_t)nb * (K >> 5) + kb) * 64 + lane) * 8 + (k & 7);
}
// bf16 activations X[rows, K] in MFMA B-operand order: fragment (kb, cb) holds rows 16*cb.. and
// columns 32*kb..; ncb = number of 16-row blocks.  float32 activations are plain row-major.
__host__ __device__ inline size_t xfrag_index(int row, int k, int ncb) {
    int cb = row >> 4, kb = k >> 5;
    int lane = (((k >> 3) & 3) << 4) | (row & 15);
    return (((size_t)kb * ncb + cb) * 64 + lane) * 8 + (k & 7);
}
template <typename T> __device__ inline size_t act_index(int row, int k, int K, int ncb);
template <> __device__ inline size_t act_index<float>(int row, int k, int K, int) { return (size_t)row * K + k; }
template <> __device__ inline size_t act_index<bf16_t>(int row, int k, int, int ncb) { return xfrag_index(row, k, ncb); }

template <typename T> __device__ inline size_t w_index(int n, int k, int K);
template <> __device__ inline size_t w_index<float>(int n, int k, int K) { return (size_t)n * K + k; }
template <> __device__ inline size_t w_index<bf16_t>(int n, int k, int K) { return wfrag_index(n, k, K); }

// KV pool: per layer and 64-token page, the K blocks of the kv heads, then their V blocks, 64 * hd
// elements each, stored in the order the attention MFMAs read them, so that a wavefront's load of one
// operand fragment is one contiguous kilobyte (lane l reads 16 bytes at 16 * l):
//   K: [32-key tile][16-key half h][32-wide depth block kd][g4][l15][8]   key  = 8 * (l15 >> 2) + (l15 & 3) + 4 * h
//                                                                         d    = 32 * kd + 8 * g4 + j
//   V: [32-key tile][16-wide depth block db][g4][l15][8]                  key  = 8 * g4 + j,  d = 16 * db + l15
// (lane = 16 * g4 + l15; a K row's eight-element groups and a V row's eight-key groups stay contiguous).
__host__ __device__ inline size_t kv_k_index(int layer, int n_pages, int page, int hkv, int head, int tin,
                                              int d, int hd) {
    const int key = tin % 32, h = (key % 8) / 4, l15 = (key / 8) * 4 + key % 4;
    const int frag = ((tin / 32) * 2 + h) * (hd / 32) + d / 32;
    return (((size_t)layer * n_pages + page) * 2 * hkv + head) * VF_TILE * hd +
           (size_t)((frag * 4 + (d % 32) / 8) * 16 + l15) * 8 + d % 8;
}
__host__ __device__ inline size_t kv_v_index(int layer, int n_pages, int page, int hkv, int head, int tin,
                                              int d, int hd) {
    const int key = tin % 32;
    const int frag = (tin / 32) * (hd / 16) + d / 16;
    return (((size_t)layer * n_pages + page) * 2 * hkv + hkv + head) * VF_TILE * hd +
           (size_t)((frag * 4 + key / 8) * 16 + d % 16) * 8 + key % 8;
}
__device__ inline int kv_page(const SeqDesc &s, int t) {
    int tile = t / VF_TILE;
    return s.block_table ? s.block_table[tile] : tile;
}

__device__ inline float to_f32(float v) { return v; }
__device__ inline float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ inline T from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // round-to-nearest-even

// Kernels that keep MFMA accumulators live across a loop ask for at least two wavefronts per SIMD:
// within that register budget (256 per lane) the compiler places accumulators in ordinary vector
// registers and updates them in place; with the whole file at its disposal it moves them to and
// from accumulation registers around every MFMA.
#define VF_MFMA_KERNEL __attribute__((amdgpu_waves_per_eu(2)))

// Workgroup barrier for data exchanged through LDS only.  Unlike __syncthreads() it does not wait
// for this wavefront's global loads in flight, only for its LDS operations; the empty asm
// statements keep the compiler from moving memory accesses across it.
__device__ __forceinline__ void lds_sync() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ inline int find_seq(const Batch &b, int row) {
    int i = 0;
    while (i + 1 < b.n_seqs && row >= b.s[i + 1].row0) ++i;
    return i;
}

// ---- launchers (defined next to their kernels) --------------------------------------------------
struct GemmPlan {
    int ks;        // K splits (partials)
    int nbw;       // n-blocks per wavefront
    int tnb;       // > 0: many-row kernel with this many weight blocks per workgroup
    int swiglu;    // many-row kernel only: write bf16(silu(gate) * up) in activation layout, not partials
    int topk;      // many-row kernel only, > 0: write this many top candidates per (row, column tile), not partials
    int32_t *topk_ids;  // their ids (the values go where the partials would)
};
GemmPlan vf_gemm_plan(const vf_model *m, int N, int K, int rows, int force_single);
// Y partials [ks][R][N] (R = ld_rows) for rows [row_lo, row_hi) of X.
int vf_launch_gemm(const vf_model *m, const void *W, const void *X, float *part, int N, int K,
                   int rows_total, int row_lo, int row_hi, int ld_rows, GemmPlan plan, hipStream_t st);

int vf_launch_pack(const vf_model *m, const void *src, void *dst, int n_rows, int K, int dst_nb0,
                   int dst_nb_stride, int perm_hd, hipStream_t st);
int vf_launch_pack_vec(const float *src, float *dst, int n, int perm_hd, hipStream_t st);
int vf_launch_rope_table(const vf_model *m, hipStream_t st);
int vf_launch_embed(const vf_model *m, const Batch &b, const int32_t *tokens, hipStream_t st);
int vf_launch_norm(const vf_model *m, const float *gain, void *x_out, const float *part, int nparts,
                   int rows, int ld_rows, hipStream_t st);
// depth != NULL (tree verify): row r stands at position len + depth[row], not len + r
int vf_launch_qkv_finish(const vf_model *m, const Batch &b, int layer, const float *part, int nparts,
                         int ld_rows, const int32_t *depth, hipStream_t st);
// ancestor masks and depths of every row of the call from the parent table, into the model workspace
int vf_launch_tree_prep(const vf_model *m, const Batch &b, const TreeDesc &tree, hipStream_t st);
// moves the K/V rows of the accepted path (path[row0 + j], j = 1..n_accept) to the positions right
// after the old length; runs after the acceptance kernels have committed the new length
int vf_launch_kv_compact(const vf_model *m, const Batch &b, const int32_t *n_accept, const int32_t *path,
                         hipStream_t st);
int vf_launch_accept_tree(const vf_model *m, const Batch &b, const AcceptBatch &ab, const TreeDesc &tree,
                          const int32_t *tokens, const float *logits, int32_t *n_accept, int32_t *out_tokens,
                          int32_t *y, int32_t *path, hipStream_t st);
int vf_launch_swiglu(const vf_model *m, const float *part, int nparts, int rows, int ld_rows, hipStream_t st);
int vf_launch_reduce_rows(const vf_model *m, const float *part, int nparts, int N, int row_lo, int row_hi,
                          int ld_rows, float *out, int out_ld, hipStream_t st);
// anc != NULL: rows of the call see, among the call's rows, only those in their ancestor mask
int vf_launch_attention(const vf_model *m, const Batch &b, int layer, const tree_mask_t *anc, hipStream_t st);
int vf_launch_state_set(int32_t *state, int idx, int32_t value, hipStream_t st);
int vf_launch_state_add(int32_t *state, int idx, int32_t delta, hipStream_t st);
int vf_launch_kv_read(const vf_model *m, const SeqDesc &s, int layer, int t0, int n, float *k_out,
                      float *v_out, hipStream_t st);
int vf_launch_stream_read(const vf_model *m, size_t *bytes, hipStream_t st);
int vf_launch_kv_write(const vf_model *m, const SeqDesc &s, int layer, int t0, int n, const float *k_in,
                       const float *v_in, hipStream_t st);
int vf_launch_accept(const vf_model *m, const Batch &b, const AcceptBatch &ab, const int32_t *tokens,
                     const float *logits, int32_t *n_accept, int32_t *out_tokens, int32_t *y,
                     hipStream_t st);
int vf_launch_accept_static(const vf_model *m, const Batch &b, const AcceptBatch &ab, const int32_t *tokens,
                            const float *logits, int32_t *n_accept, int32_t *out_tokens, int32_t *y,
                            hipStream_t st);
int vf_accept_static_init();
int vf_launch_attention_rows(const vf_model *m, const Batch &b, int layer, hipStream_t st);
bool vf_fast_path_ok(const vf_model *m, int total_rows);
int vf_run_fast(vf_model *m, const Batch &b, const int32_t *tokens, float *logits_out, hipStream_t st);
size_t vf_fused_workspace_bytes(const vf_config &c);
int vf_fused_init(vf_model *m, char *ws, hipStream_t st);
bool vf_fused_ok(const vf_model *m, const Batch &b);
// tree: rows take position and visibility from the model's tree_depth / tree_anc tables
int vf_run_fused(vf_model *m, const Batch &b, const int32_t *tokens, float *logits_out, bool tree, hipStream_t st);
int vf_fused_check(vf_model *m);
size_t vf_fused_part_floats(const vf_config &c);
// per-row top-k of logits: candidates per vocabulary slice into the model's candidate buffers, then the merge
int vf_launch_topk_slices(const vf_model *m, const float *logits, int rows, int K, hipStream_t st);
int vf_launch_topk_merge(const vf_model *m, int rows, int n_slices, int K, float *out_v, int32_t *out_i,
                         hipStream_t st);
// most (row, slice) candidate lists a row can have: slices of the slice kernel or column tiles of the GEMM
inline int vf_topk_max_slices(const vf_config &c) {
    const int tiles = (c.vocab / 16 + 3) / 4;  // narrow GEMM tile: four 16-column blocks
    return tiles > VF_STAT_CHUNKS ? tiles : VF_STAT_CHUNKS;
}
int vf_launch_first_token(const vf_model *m, const SeqDesc &s, const float *logits_row, const float *u,
                          float temperature, hipStream_t st);
