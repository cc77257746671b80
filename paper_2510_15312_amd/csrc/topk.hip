// Top successors of every prefill position (paper Sec. 4.2, workflow step "Sample"): the k largest
// logits of each row, equal logits by rising id.  Two stages: candidates per (row, slice of the
// vocabulary), then a merge per row.  The candidates come either from this file's slice kernel
// (logits in memory) or straight from the output-head GEMM's epilogue (gemm.hip), which then never
// writes the logits.
#include "vf_internal.h"

namespace {

struct Cand {
    float v;
    int i;
};
// a comes before b in the result order
__device__ inline bool before(Cand a, Cand b) { return a.v > b.v || (a.v == b.v && a.i < b.i); }

__device__ inline Cand block_first(Cand mine, Cand *red) {
    for (int off = 32; off > 0; off >>= 1) {
        const Cand o{__shfl_xor(mine.v, off, 64), __shfl_xor(mine.i, off, 64)};
        if (before(o, mine)) mine = o;
    }
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();  // red may still be read from the round before
    if ((threadIdx.x & 63) == 0) red[wave] = mine;
    __syncthreads();
    Cand best = red[0];
    for (int w = 1; w < nw; ++w)
        if (before(red[w], best)) best = red[w];
    return best;
}

// K rounds; in each, every thread looks through its share for the first element (in result order)
// that comes after the one chosen in the round before.  Ids are unique, so the order is strict and
// nothing needs to be marked.  An exhausted slice yields (-inf, -1).
template <typename Load>
__device__ inline void select_k(int n, int K, Load load, float *out_v, int32_t *out_i, Cand *red) {
    Cand prev{INFINITY, -1};
    for (int r = 0; r < K; ++r) {
        Cand best{-INFINITY, 0x7fffffff};
        for (int j = threadIdx.x; j < n; j += blockDim.x) {
            const Cand c = load(j);
            if (c.i >= 0 && before(prev, c) && before(c, best)) best = c;
        }
        best = block_first(best, red);
        if (best.i == 0x7fffffff) best = Cand{-INFINITY, -1};
        if (threadIdx.x == 0) {
            out_v[r] = best.v;
            out_i[r] = best.i;
        }
        if (best.i < 0) {  // nothing left: the same for every thread
            for (int q = r + 1; q < K; ++q)
                if (threadIdx.x == 0) {
                    out_v[q] = -INFINITY;
                    out_i[q] = -1;
                }
            return;
        }
        prev = best;
    }
}

__global__ __launch_bounds__(256) void topk_slice_kernel(const float *__restrict__ logits, int V, int n_slices, int K,
                                                         float *__restrict__ cand_v, int32_t *__restrict__ cand_i) {
    __shared__ Cand red[4];
    const int row = blockIdx.y, sl = blockIdx.x;
    const int per = (V + n_slices - 1) / n_slices;
    const int v0 = min(V, sl * per), v1 = min(V, v0 + per);
    const float *z = logits + (size_t)row * V;
    const size_t o = ((size_t)row * n_slices + sl) * K;
    select_k(v1 - v0, K, [&](int j) { return Cand{z[v0 + j], v0 + j}; }, cand_v + o, cand_i + o, red);
}

__global__ __launch_bounds__(256) void topk_merge_kernel(const float *__restrict__ cand_v,
                                                         const int32_t *__restrict__ cand_i, int n_cand, int K,
                                                         float *__restrict__ out_v, int32_t *__restrict__ out_i) {
    __shared__ Cand red[4];
    const int row = blockIdx.x;
    const float *cv = cand_v + (size_t)row * n_cand;
    const int32_t *ci = cand_i + (size_t)row * n_cand;
    select_k(n_cand, K, [&](int j) { return Cand{cv[j], ci[j]}; }, out_v + (size_t)row * K, out_i + (size_t)row * K, red);
}

}  // namespace

int vf_launch_topk_slices(const vf_model *m, const float *logits, int rows, int K, hipStream_t st) {
    hipLaunchKernelGGL(topk_slice_kernel, dim3(VF_STAT_CHUNKS, rows), dim3(256), 0, st, logits, m->cfg.vocab,
                       VF_STAT_CHUNKS, K, m->topk_cand_v, m->topk_cand_i);
    VF_LAUNCH_CHECK("topk_slice");
    return VF_OK;
}

int vf_launch_topk_merge(const vf_model *m, int rows, int n_slices, int K, float *out_v, int32_t *out_i,
                         hipStream_t st) {
    hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(256), 0, st, m->topk_cand_v, m->topk_cand_i, n_slices * K,
                       K, out_v, out_i);
    VF_LAUNCH_CHECK("topk_merge");
    return VF_OK;
}
