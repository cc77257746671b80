// Acceptance on the device (paper Sec. 3 "any tokens after the first mismatch are discarded",
// Sec. 4.3 "accepted prefix x_1..x_{e-1}, y_e"), greedy and stochastic, and the commit of the
// sequence state (length, pending token) without a host round trip.
//
// Pass 1 (row_stats): per (row, vocabulary chunk) the maximum logit, its lowest index and, for
// stochastic rows, sum exp((z - chunk max)/T) in float64.
// Pass 2 (finalize): one workgroup per sequence merges the chunks in a fixed order, walks the
// drafts, and if needed draws the replacement / bonus token by inverse CDF over the
// vocabulary in id order, all in float64.
#include "vf_internal.h"

namespace {

constexpr int FIN_THREADS = 1024;

struct MaxIdx {
    float v;
    int i;
};
__device__ inline MaxIdx better(MaxIdx a, MaxIdx b) {
    if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
    return a;
}

__global__ __launch_bounds__(256) void row_stats_kernel(const float *__restrict__ logits, int V, int n_chunks,
                                                        Batch b, AcceptBatch ab, float *__restrict__ smax,
                                                        int32_t *__restrict__ sidx, double *__restrict__ ssum) {
    __shared__ MaxIdx rm[4];
    __shared__ double rs[4];
    const int row = blockIdx.y, chunk = blockIdx.x;
    const int per = (V + n_chunks - 1) / n_chunks;
    const int v0 = chunk * per, v1 = min(V, v0 + per);
    const float *z = logits + (size_t)row * V;
    MaxIdx best{-INFINITY, 0x7fffffff};
    for (int v = v0 + threadIdx.x; v < v1; v += 256) best = better(best, MaxIdx{z[v], v});
    for (int off = 32; off > 0; off >>= 1) {
        MaxIdx o{__shfl_xor(best.v, off, 64), __shfl_xor(best.i, off, 64)};
        best = better(best, o);
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) rm[wave] = best;
    __syncthreads();
    best = better(better(rm[0], rm[1]), better(rm[2], rm[3]));
    const AcceptDesc &a = ab.a[find_seq(b, row)];
    double sum = 0.0;
    if (a.mode == VF_STOCHASTIC && v0 < v1) {
        const double t = (double)a.temperature, cm = (double)best.v;
        for (int v = v0 + threadIdx.x; v < v1; v += 256) sum += exp(((double)z[v] - cm) / t);
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
        if ((threadIdx.x & 63) == 0) rs[wave] = sum;
        __syncthreads();
        sum = ((rs[0] + rs[1]) + rs[2]) + rs[3];
    }
    if (threadIdx.x == 0) {
        const size_t o = (size_t)row * n_chunks + chunk;
        smax[o] = best.v;
        sidx[o] = best.i;
        ssum[o] = sum;
    }
}

// Inverse-CDF draw over the vocabulary in id order, by the whole workgroup.
//   weight(v) = max(0, p_v - q_v)   (q given)          p_v = exp((z_v - zmax)/t) / S
//             = p_v with p_x = 0    (one-hot drafter, x = excluded id)
//             = p_v                 (bonus / first token: q == NULL and x < 0)
// If every weight is zero the draw is from p.  Returns the smallest id whose running sum
// exceeds u * total (same value in every thread).
__device__ int draw_token(const float *__restrict__ z, int V, double zmax, double t, double S,
                          const float *__restrict__ q, int x, double u, double *seg, int *result) {
    const int per = (V + FIN_THREADS - 1) / FIN_THREADS;
    const int v0 = min(V, (int)threadIdx.x * per), v1 = min(V, v0 + per);
    for (int pass = 0; pass < 2; ++pass) {
        const bool plain = pass == 1;
        auto weight = [&](int v) -> double {
            double p = exp(((double)z[v] - zmax) / t) / S;
            if (plain) return p;
            if (q) return fmax(p - (double)q[v], 0.0);
            return v == x ? 0.0 : p;
        };
        double local = 0.0;
        for (int v = v0; v < v1; ++v) local += weight(v);
        __syncthreads();
        seg[threadIdx.x] = local;
        if (threadIdx.x == 0) *result = 0x7fffffff;
        __syncthreads();
        // exclusive prefix of the segment sums, in segment order (every thread the same way)
        double before = 0.0, total = 0.0;
        for (int j = 0; j < FIN_THREADS; ++j) {
            if (j == (int)threadIdx.x) before = total;
            total += seg[j];
        }
        if (total == 0.0 && !plain) continue;
        const double target = u * total;
        if (before <= target) {
            double run = before;
            for (int v = v0; v < v1; ++v) {
                run += weight(v);
                if (run > target) {
                    atomicMin(result, v);
                    break;
                }
            }
        }
        __syncthreads();
        int w = *result;
        if (w == 0x7fffffff) w = V - 1;  // rounding left the running sum at or below the target
        __syncthreads();
        return w;
    }
    return V - 1;
}

__global__ __launch_bounds__(FIN_THREADS) void accept_finalize_kernel(
    const float *__restrict__ logits, int V, int n_chunks, Batch b, AcceptBatch ab,
    const int32_t *__restrict__ tokens, const float *__restrict__ smax, const int32_t *__restrict__ sidx,
    const double *__restrict__ ssum, int32_t *__restrict__ n_accept, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ y) {
    __shared__ double seg[FIN_THREADS];
    __shared__ double row_S[VF_MAX_DRAFTS + 1];
    __shared__ float row_max[VF_MAX_DRAFTS + 1];
    __shared__ int row_arg[VF_MAX_DRAFTS + 1];
    __shared__ int sh_a, sh_result;
    const SeqDesc &s = b.s[blockIdx.x];
    const AcceptDesc &a = ab.a[blockIdx.x];
    const int m = s.nrows, k = m - 1;
    const double t = (double)a.temperature;
    if ((int)threadIdx.x < m) {
        const size_t o = (size_t)(s.row0 + threadIdx.x) * n_chunks;
        MaxIdx best{-INFINITY, 0x7fffffff};
        for (int c = 0; c < n_chunks; ++c) best = better(best, MaxIdx{smax[o + c], sidx[o + c]});
        double S = 0.0;
        if (a.mode == VF_STOCHASTIC)
            for (int c = 0; c < n_chunks; ++c)
                if (ssum[o + c] != 0.0) S += ssum[o + c] * exp(((double)smax[o + c] - (double)best.v) / t);
        row_S[threadIdx.x] = S;
        row_max[threadIdx.x] = best.v;
        row_arg[threadIdx.x] = best.i;
        y[s.row0 + threadIdx.x] = best.i;
    }
    __syncthreads();
    const int32_t *drafts = tokens + s.row0 + 1;
    if (threadIdx.x == 0) {
        int acc = 0;
        if (a.mode == VF_GREEDY) {
            while (acc < k && drafts[acc] == row_arg[acc]) ++acc;
        } else {
            for (; acc < k; ++acc) {
                const int x = drafts[acc];
                if (x < 0 || x >= V) break;
                const float *z = logits + (size_t)(s.row0 + acc) * V;
                const double px = exp(((double)z[x] - (double)row_max[acc]) / t) / row_S[acc];
                const double qx = a.q ? (double)a.q[(size_t)acc * V + x] : 1.0;
                if (!((double)a.u[acc] * qx < px)) break;
            }
        }
        sh_a = acc;
    }
    __syncthreads();
    const int acc = sh_a;
    int emitted;
    if (a.mode == VF_GREEDY) {
        emitted = row_arg[acc];
    } else {
        const float *z = logits + (size_t)(s.row0 + acc) * V;
        const float *q = (acc < k && a.q) ? a.q + (size_t)acc * V : nullptr;
        const int x = (acc < k && !a.q) ? drafts[acc] : -1;
        emitted = draw_token(z, V, (double)row_max[acc], t, row_S[acc], q, x, (double)a.u[m + acc], seg,
                             &sh_result);
    }
    if ((int)threadIdx.x < m) {
        int v = -1;
        if ((int)threadIdx.x < acc) v = drafts[threadIdx.x];
        else if ((int)threadIdx.x == acc) v = emitted;
        out_tokens[s.row0 + threadIdx.x] = v;
    }
    if (threadIdx.x == 0) {
        n_accept[blockIdx.x] = acc;
        s.state[0] += 1 + acc;
        s.state[1] = emitted;
    }
}

// First generated token from one row of logits: arg-max (temperature 0) or a draw from
// softmax(z / temperature); written to the sequence's pending token.
__global__ __launch_bounds__(FIN_THREADS) void first_token_kernel(const float *__restrict__ z, int V,
                                                                  const float *__restrict__ u, float temperature,
                                                                  int32_t *__restrict__ state) {
    __shared__ double seg[FIN_THREADS];
    __shared__ MaxIdx rm[FIN_THREADS / 64];
    __shared__ int sh_result;
    MaxIdx best{-INFINITY, 0x7fffffff};
    for (int v = threadIdx.x; v < V; v += FIN_THREADS) best = better(best, MaxIdx{z[v], v});
    for (int off = 32; off > 0; off >>= 1) {
        MaxIdx o{__shfl_xor(best.v, off, 64), __shfl_xor(best.i, off, 64)};
        best = better(best, o);
    }
    if ((threadIdx.x & 63) == 0) rm[threadIdx.x >> 6] = best;
    __syncthreads();
    best = rm[0];
    for (int i = 1; i < FIN_THREADS / 64; ++i) best = better(best, rm[i]);
    int tok = best.i;
    if (temperature > 0.f) {
        const double t = (double)temperature;
        double local = 0.0;
        for (int v = threadIdx.x; v < V; v += FIN_THREADS) local += exp(((double)z[v] - (double)best.v) / t);
        __syncthreads();
        seg[threadIdx.x] = local;
        __syncthreads();
        double S = 0.0;
        for (int j = 0; j < FIN_THREADS; ++j) S += seg[j];
        tok = draw_token(z, V, (double)best.v, t, S, nullptr, -1, (double)u[0], seg, &sh_result);
    }
    if (threadIdx.x == 0) state[1] = tok;
}

}  // namespace

int vf_launch_accept(const vf_model *m, const Batch &b, const AcceptBatch &ab, const int32_t *tokens,
                     const float *logits, int32_t *n_accept, int32_t *out_tokens, int32_t *y, hipStream_t st) {
    const int V = m->cfg.vocab;
    hipLaunchKernelGGL(row_stats_kernel, dim3(m->n_chunks, b.total_rows), dim3(256), 0, st, logits, V,
                       m->n_chunks, b, ab, m->stat_max, m->stat_idx, m->stat_sum);
    VF_LAUNCH_CHECK("row_stats");
    hipLaunchKernelGGL(accept_finalize_kernel, dim3(b.n_seqs), dim3(FIN_THREADS), 0, st, logits, V, m->n_chunks,
                       b, ab, tokens, m->stat_max, m->stat_idx, m->stat_sum, n_accept, out_tokens, y);
    VF_LAUNCH_CHECK("accept_finalize");
    return VF_OK;
}

int vf_launch_first_token(const vf_model *m, const SeqDesc &s, const float *logits_row, const float *u,
                          float temperature, hipStream_t st) {
    hipLaunchKernelGGL(first_token_kernel, dim3(1), dim3(FIN_THREADS), 0, st, logits_row, m->cfg.vocab, u,
                       temperature, s.state);
    VF_LAUNCH_CHECK("first_token");
    return VF_OK;
}
