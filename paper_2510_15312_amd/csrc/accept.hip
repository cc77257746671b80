// Acceptance on the device (paper Sec. 3: drafts from the first mismatch on are dropped; Sec. 4.3:
// the accepted prefix x_1..x_{e-1} followed by y_e), greedy and stochastic, and the commit of the
// sequence state (length, pending token) without a host round trip.
//
//   row_stats : per (row, vocabulary chunk): maximum logit, its lowest index and, for stochastic
//               rows, sum exp((z - chunk max)/T) in float64.
//   decide    : one workgroup per sequence merges the chunks in a fixed order (arg-max y of every
//               row, softmax normaliser), walks the drafts and fixes the accepted count a.  Greedy
//               sequences are finished here.
//   draw_sums : stochastic only: per vocabulary chunk the float64 sum of the weights the
//               replacement (or bonus) token is drawn from at row a.
//   emit      : inverse CDF in id order: finds the chunk, then the id inside it; commits the state.
#include "vf_internal.h"

namespace {

// Where the kernels below keep what they hand to one another: per (row, vocabulary chunk) statistics,
// one draw descriptor per sequence, and the per-chunk weight sums of the draw.
struct AcceptScratch {
    float *smax;        // [rows, VF_STAT_CHUNKS]
    int32_t *sidx;      // [rows, VF_STAT_CHUNKS]
    double *ssum;       // [rows, VF_STAT_CHUNKS]
    DrawDesc *draw;     // [VF_MAX_BATCH]
    double *draw_sums;  // [VF_MAX_BATCH, VF_STAT_CHUNKS]
};

// Scratch of vf_accept_static: the same buffers for up to VF_ACCEPT_STATIC_MAX_ROWS rows, in device
// memory that belongs to the loaded library (one copy per GPU, held until the process ends) instead of
// the model workspace.  The name is only a host-side handle: the device address is asked for once per
// device (static_scratch) and that pointer is what the launches get.
constexpr size_t SS_SMAX = 0;
constexpr size_t SS_SIDX = SS_SMAX + (size_t)VF_ACCEPT_STATIC_MAX_ROWS * VF_STAT_CHUNKS * 4;
constexpr size_t SS_SSUM = SS_SIDX + (size_t)VF_ACCEPT_STATIC_MAX_ROWS * VF_STAT_CHUNKS * 4;
constexpr size_t SS_DRAW = SS_SSUM + (size_t)VF_ACCEPT_STATIC_MAX_ROWS * VF_STAT_CHUNKS * 8;
constexpr size_t SS_DSUM = (SS_DRAW + sizeof(DrawDesc) * VF_MAX_BATCH + 255) / 256 * 256;
constexpr size_t SS_BYTES = SS_DSUM + (size_t)VF_MAX_BATCH * VF_STAT_CHUNKS * 8;
static __device__ __align__(256) unsigned char scratch[SS_BYTES];

constexpr int SS_MAX_DEVICES = 64;
unsigned char *g_scratch_ptr[SS_MAX_DEVICES];  // device address of `scratch` on every GPU seen so far

// Device address of the static scratch on the current device; resolved on the first call per device.
int static_scratch(AcceptScratch *out) {
    int dev = 0;
    VF_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= SS_MAX_DEVICES) return vf_fail(VF_ERR_UNSUPPORTED, "device ordinal %d", dev);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        VF_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return vf_fail(VF_ERR_HIP, "hipGetSymbolAddress returned no address");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    unsigned char *base = g_scratch_ptr[dev];
    out->smax = reinterpret_cast<float *>(base + SS_SMAX);
    out->sidx = reinterpret_cast<int32_t *>(base + SS_SIDX);
    out->ssum = reinterpret_cast<double *>(base + SS_SSUM);
    out->draw = reinterpret_cast<DrawDesc *>(base + SS_DRAW);
    out->draw_sums = reinterpret_cast<double *>(base + SS_DSUM);
    return VF_OK;
}

AcceptScratch model_scratch(const vf_model *m) {
    return AcceptScratch{m->stat_max, m->stat_idx, m->stat_sum, m->draw, m->draw_sums};
}

struct MaxIdx {
    float v;
    int i;
};
__device__ inline MaxIdx better(MaxIdx a, MaxIdx b) {
    if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
    return a;
}
__device__ inline MaxIdx wave_best(MaxIdx best) {
    for (int off = 32; off > 0; off >>= 1) {
        MaxIdx o{__shfl_xor(best.v, off, 64), __shfl_xor(best.i, off, 64)};
        best = better(best, o);
    }
    return best;
}
__device__ inline double wave_sum(double s) {
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    return s;
}

__global__ __launch_bounds__(256) void row_stats_kernel(const float *__restrict__ logits, int V, Batch b,
                                                        AcceptBatch ab, float *__restrict__ smax,
                                                        int32_t *__restrict__ sidx, double *__restrict__ ssum) {
    __shared__ MaxIdx rm[4];
    __shared__ double rs[4];
    const int row = blockIdx.y, chunk = blockIdx.x;
    const int per = (V + VF_STAT_CHUNKS - 1) / VF_STAT_CHUNKS;
    const int v0 = min(V, chunk * per), v1 = min(V, v0 + per);
    const float *z = logits + (size_t)row * V;
    MaxIdx best{-INFINITY, 0x7fffffff};
    for (int v = v0 + threadIdx.x; v < v1; v += 256) best = better(best, MaxIdx{z[v], v});
    best = wave_best(best);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) rm[wave] = best;
    __syncthreads();
    best = better(better(rm[0], rm[1]), better(rm[2], rm[3]));
    const AcceptDesc &a = ab.a[find_seq(b, row)];
    double sum = 0.0;
    if (a.mode == VF_STOCHASTIC && v0 < v1) {
        const double t = (double)a.temperature, cm = (double)best.v;
        for (int v = v0 + threadIdx.x; v < v1; v += 256) sum += exp(((double)z[v] - cm) / t);
        sum = wave_sum(sum);
        if ((threadIdx.x & 63) == 0) rs[wave] = sum;
        __syncthreads();
        sum = ((rs[0] + rs[1]) + rs[2]) + rs[3];
    }
    if (threadIdx.x == 0) {
        const size_t o = (size_t)row * VF_STAT_CHUNKS + chunk;
        smax[o] = best.v;
        sidx[o] = best.i;
        ssum[o] = sum;
    }
}

// commit_len == 0: only the pending token is written (first token after prefill).
__global__ __launch_bounds__(256) void accept_decide_kernel(
    const float *__restrict__ logits, int V, Batch b, AcceptBatch ab, const int32_t *__restrict__ tokens,
    const float *__restrict__ smax, const int32_t *__restrict__ sidx, const double *__restrict__ ssum,
    int32_t *__restrict__ n_accept, int32_t *__restrict__ out_tokens, int32_t *__restrict__ y,
    DrawDesc *__restrict__ draw, int commit_len) {
    __shared__ double row_S[VF_MAX_DRAFTS + 1];
    __shared__ float row_max[VF_MAX_DRAFTS + 1];
    __shared__ int row_arg[VF_MAX_DRAFTS + 1];
    __shared__ int ok[VF_MAX_DRAFTS + 1];
    const SeqDesc &s = b.s[blockIdx.x];
    const AcceptDesc &a = ab.a[blockIdx.x];
    const int m = s.nrows, k = m - 1;
    const double t = (double)a.temperature;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < m; r += 4) {
        const size_t o = (size_t)(s.row0 + r) * VF_STAT_CHUNKS + lane;  // one chunk per lane
        const MaxIdx mine{smax[o], sidx[o]};
        const MaxIdx best = wave_best(mine);
        double S = 0.0;
        if (a.mode == VF_STOCHASTIC) {
            const double sm = ssum[o];
            S = wave_sum(sm != 0.0 ? sm * exp(((double)mine.v - (double)best.v) / t) : 0.0);
        }
        if (lane == 0) {
            row_S[r] = S;
            row_max[r] = best.v;
            row_arg[r] = best.i;
            y[s.row0 + r] = best.i;
        }
    }
    __syncthreads();
    const int32_t *drafts = tokens + s.row0 + 1;
    if ((int)threadIdx.x < k) {
        const int i = threadIdx.x, x = drafts[i];
        int good;
        if (a.mode == VF_GREEDY) {
            good = x == row_arg[i];
        } else if (x < 0 || x >= V) {
            good = 0;
        } else {
            const float *z = logits + (size_t)(s.row0 + i) * V;
            const double px = exp(((double)z[x] - (double)row_max[i]) / t) / row_S[i];
            const double qx = a.q ? (double)a.q[(size_t)i * V + x] : 1.0;
            good = (double)a.u[i] * qx < px;
        }
        ok[i] = good;
    }
    __syncthreads();
    int acc = 0;
    while (acc < k && ok[acc]) ++acc;
    if ((int)threadIdx.x < m) {
        int v = -1;
        if ((int)threadIdx.x < acc) v = drafts[threadIdx.x];
        else if ((int)threadIdx.x == acc && a.mode == VF_GREEDY) v = row_arg[acc];
        out_tokens[s.row0 + threadIdx.x] = v;
    }
    if (threadIdx.x == 0) {
        n_accept[blockIdx.x] = acc;
        DrawDesc d;
        d.zmax = (double)row_max[acc];
        d.S = row_S[acc];
        d.active = a.mode == VF_STOCHASTIC;
        d.acc = acc;
        d.row = s.row0 + acc;
        d.q = (acc < k && a.q) ? a.q + (size_t)acc * V : nullptr;
        d.x_excl = (acc < k && !a.q) ? drafts[acc] : -1;
        d.n_excl = 0;
        d.u = d.active ? (double)a.u[m + acc] : 0.0;
        d.t = t;
        draw[blockIdx.x] = d;
        if (a.mode == VF_GREEDY) {
            if (commit_len) s.state[0] += 1 + acc;
            s.state[1] = row_arg[acc];
        }
    }
}

// Tree-structured drafts: the same row statistics, then one thread walks down from the root.
// Greedy: move to the first child (in row order) whose token is the arg-max at the current node.
// Stochastic, deterministic drafter: the children are tried in row order against the residual of
// the node's target distribution p: child with token x is kept when u * (1 - struck mass) < r(x),
// r(x) = p(x) unless an earlier refused sibling carried the same token; a refused child's token is
// struck.  The walk ends at the node none of whose children is kept; the token emitted there is the
// arg-max (greedy) or a draw from the residual (emit kernel, via the exclusion list).
__global__ __launch_bounds__(256) void accept_tree_decide_kernel(
    const float *__restrict__ logits, int V, Batch b, AcceptBatch ab, TreeDesc tree,
    const int32_t *__restrict__ tokens, const float *__restrict__ smax, const int32_t *__restrict__ sidx,
    const double *__restrict__ ssum, int32_t *__restrict__ n_accept, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ y, int32_t *__restrict__ path_out, DrawDesc *__restrict__ draw) {
    __shared__ double row_S[VF_MAX_DRAFTS + 1];
    __shared__ float row_max[VF_MAX_DRAFTS + 1];
    __shared__ int row_arg[VF_MAX_DRAFTS + 1];
    __shared__ double px[VF_MAX_DRAFTS + 1];   // p of the parent node at this node's token
    __shared__ int path[VF_MAX_DRAFTS + 1];
    const SeqDesc &s = b.s[blockIdx.x];
    const AcceptDesc &a = ab.a[blockIdx.x];
    const int8_t *par = tree.parent[blockIdx.x];
    const int m = s.nrows;
    const double t = (double)a.temperature;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < m; r += 4) {
        const size_t o = (size_t)(s.row0 + r) * VF_STAT_CHUNKS + lane;  // one chunk per lane
        const MaxIdx mine{smax[o], sidx[o]};
        const MaxIdx best = wave_best(mine);
        double S = 0.0;
        if (a.mode == VF_STOCHASTIC) {
            const double sm = ssum[o];
            S = wave_sum(sm != 0.0 ? sm * exp(((double)mine.v - (double)best.v) / t) : 0.0);
        }
        if (lane == 0) {
            row_S[r] = S;
            row_max[r] = best.v;
            row_arg[r] = best.i;
            y[s.row0 + r] = best.i;
        }
    }
    __syncthreads();
    const int c = threadIdx.x;
    if (c >= 1 && c < m) {
        double v = 0.0;
        const int x = tokens[s.row0 + c], pr = par[c];
        if (a.mode == VF_STOCHASTIC && x >= 0 && x < V)
            v = exp(((double)logits[(size_t)(s.row0 + pr) * V + x] - (double)row_max[pr]) / t) / row_S[pr];
        px[c] = v;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    DrawDesc &d = draw[blockIdx.x];
    int acc = 0, cur = 0, n_excl = 0;
    path[0] = 0;
    while (true) {
        int kept = -1;
        n_excl = 0;
        double struck = 0.0;
        for (int ch = cur + 1; ch < m; ++ch) {
            if (par[ch] != cur) continue;
            const int x = tokens[s.row0 + ch];
            if (a.mode == VF_GREEDY) {
                if (x == row_arg[cur]) { kept = ch; break; }
                continue;
            }
            bool dup = false;
            for (int i = 0; i < n_excl; ++i) dup = dup || d.excl[i] == x;
            const double rx = dup ? 0.0 : px[ch];
            if ((double)a.u[ch - 1] * (1.0 - struck) < rx) { kept = ch; break; }
            if (!dup && x >= 0 && x < V) {
                d.excl[n_excl++] = x;
                struck += px[ch];
            }
        }
        if (kept < 0) break;
        path[++acc] = kept;
        cur = kept;
    }
    for (int j = 0; j < m; ++j) {
        int v = -1;
        if (j < acc) v = tokens[s.row0 + path[j + 1]];
        else if (j == acc && a.mode == VF_GREEDY) v = row_arg[cur];
        out_tokens[s.row0 + j] = v;
        path_out[s.row0 + j] = j <= acc ? path[j] : -1;
    }
    n_accept[blockIdx.x] = acc;
    d.zmax = (double)row_max[cur];
    d.S = row_S[cur];
    d.active = a.mode == VF_STOCHASTIC;
    d.acc = acc;
    d.row = s.row0 + cur;
    d.q = nullptr;
    d.x_excl = -1;
    d.n_excl = n_excl;
    d.u = d.active ? (double)a.u[m + cur] : 0.0;
    d.t = t;
    if (a.mode == VF_GREEDY) {
        s.state[0] += 1 + acc;
        s.state[1] = row_arg[cur];
    }
}

// weight of id v in the draw at the deciding row:
//   max(0, p_v - q_v)  (dense draft distribution),  p_v with p_x = 0  (one-hot drafter; for a tree
//   every refused child's token x),
//   p_v  (bonus token / first token / every residual weight zero),  p_v = exp((z_v - zmax)/T) / S.
__device__ inline double draw_weight(const float *__restrict__ z, const DrawDesc &d, int v, bool plain) {
    const double p = exp(((double)z[v] - d.zmax) / d.t) / d.S;
    if (plain) return p;
    if (d.q) return fmax(p - (double)d.q[v], 0.0);
    if (v == d.x_excl) return 0.0;
    for (int i = 0; i < d.n_excl; ++i)
        if (v == d.excl[i]) return 0.0;
    return p;
}

__device__ inline double chunk_weight_sum(const float *__restrict__ z, const DrawDesc &d, int v0, int v1,
                                          bool plain, double *rs) {
    double sum = 0.0;
    for (int v = v0 + threadIdx.x; v < v1; v += 256) sum += draw_weight(z, d, v, plain);
    sum = wave_sum(sum);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) rs[threadIdx.x >> 6] = sum;
    __syncthreads();
    return ((rs[0] + rs[1]) + rs[2]) + rs[3];
}

__global__ __launch_bounds__(256) void draw_sums_kernel(const float *__restrict__ logits, int V,
                                                        const DrawDesc *__restrict__ draw,
                                                        double *__restrict__ wsum) {
    __shared__ double rs[4];
    const DrawDesc &d = draw[blockIdx.y];
    if (!d.active) return;
    const int per = (V + VF_STAT_CHUNKS - 1) / VF_STAT_CHUNKS;
    const int v0 = min(V, (int)blockIdx.x * per), v1 = min(V, v0 + per);
    const double sum = chunk_weight_sum(logits + (size_t)d.row * V, d, v0, v1, false, rs);
    if (threadIdx.x == 0) wsum[blockIdx.y * VF_STAT_CHUNKS + blockIdx.x] = sum;
}

__global__ __launch_bounds__(256) void accept_emit_kernel(const float *__restrict__ logits, int V, Batch b,
                                                          const DrawDesc *__restrict__ draw,
                                                          const double *__restrict__ wsum,
                                                          int32_t *__restrict__ out_tokens, int commit_len) {
    __shared__ double cs[VF_STAT_CHUNKS];
    __shared__ double seg[256];
    __shared__ double rs[4];
    __shared__ int result;
    const DrawDesc &d = draw[blockIdx.x];
    if (!d.active) return;
    const SeqDesc &s = b.s[blockIdx.x];
    const float *z = logits + (size_t)d.row * V;
    const int per = (V + VF_STAT_CHUNKS - 1) / VF_STAT_CHUNKS;
    if (threadIdx.x < VF_STAT_CHUNKS) cs[threadIdx.x] = wsum[blockIdx.x * VF_STAT_CHUNKS + threadIdx.x];
    __syncthreads();
    double total = 0.0;
    for (int c = 0; c < VF_STAT_CHUNKS; ++c) total += cs[c];
    bool plain = false;
    if (total == 0.0) {
        // every residual weight is zero: draw from p itself (sums recomputed here; rare)
        plain = true;
        for (int c = 0; c < VF_STAT_CHUNKS; ++c) {
            const int v0 = min(V, c * per), v1 = min(V, v0 + per);
            const double sum = chunk_weight_sum(z, d, v0, v1, true, rs);
            if (threadIdx.x == 0) cs[c] = sum;
        }
        __syncthreads();
        total = 0.0;
        for (int c = 0; c < VF_STAT_CHUNKS; ++c) total += cs[c];
    }
    const double target = d.u * total;
    // first chunk whose inclusive prefix exceeds the target
    int cstar = VF_STAT_CHUNKS - 1;
    double before_chunk = 0.0;
    {
        double run = 0.0;
        for (int c = 0; c < VF_STAT_CHUNKS; ++c) {
            if (run + cs[c] > target) { cstar = c; before_chunk = run; break; }
            run += cs[c];
            if (c == VF_STAT_CHUNKS - 1) before_chunk = run - cs[c];
        }
    }
    const int v0 = min(V, cstar * per), v1 = min(V, v0 + per);
    const int per_t = (v1 - v0 + 255) / 256;
    const int a0 = min(v1, v0 + (int)threadIdx.x * per_t), a1 = min(v1, a0 + per_t);
    double local = 0.0;
    for (int v = a0; v < a1; ++v) local += draw_weight(z, d, v, plain);
    seg[threadIdx.x] = local;
    if (threadIdx.x == 0) result = 0x7fffffff;
    __syncthreads();
    double before = before_chunk;
    for (int j = 0; j < (int)threadIdx.x; ++j) before += seg[j];
    if (before <= target) {
        double run = before;
        for (int v = a0; v < a1; ++v) {
            run += draw_weight(z, d, v, plain);
            if (run > target) { atomicMin(&result, v); break; }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int w = result;
        if (w == 0x7fffffff) {
            // rounding left the running sum at the target: the draw is the last id of positive weight
            // at or before the end of the chosen chunk (never an id the rule gives no weight)
            w = -1;
            for (int v = v1 - 1; v >= 0 && w < 0; --v)
                if (draw_weight(z, d, v, plain) > 0.0) w = v;
            if (w < 0) w = max(v0, v1 - 1);
        }
        out_tokens[s.row0 + d.acc] = w;
        if (commit_len) s.state[0] += 1 + d.acc;
        s.state[1] = w;
    }
}

int launch_all(const vf_model *m, const AcceptScratch &sc, const Batch &b, const AcceptBatch &ab,
               const int32_t *tokens, const float *logits, int32_t *n_accept, int32_t *out_tokens, int32_t *y,
               int commit_len, hipStream_t st) {
    const int V = m->cfg.vocab;
    hipLaunchKernelGGL(row_stats_kernel, dim3(VF_STAT_CHUNKS, b.total_rows), dim3(256), 0, st, logits, V, b, ab,
                       sc.smax, sc.sidx, sc.ssum);
    VF_LAUNCH_CHECK("row_stats");
    hipLaunchKernelGGL(accept_decide_kernel, dim3(b.n_seqs), dim3(256), 0, st, logits, V, b, ab, tokens,
                       sc.smax, sc.sidx, sc.ssum, n_accept, out_tokens, y, sc.draw, commit_len);
    VF_LAUNCH_CHECK("accept_decide");
    bool any = false;
    for (int i = 0; i < b.n_seqs; ++i) any = any || ab.a[i].mode == VF_STOCHASTIC;
    if (!any) return VF_OK;
    hipLaunchKernelGGL(draw_sums_kernel, dim3(VF_STAT_CHUNKS, b.n_seqs), dim3(256), 0, st, logits, V, sc.draw,
                       sc.draw_sums);
    VF_LAUNCH_CHECK("draw_sums");
    hipLaunchKernelGGL(accept_emit_kernel, dim3(b.n_seqs), dim3(256), 0, st, logits, V, b, sc.draw,
                       sc.draw_sums, out_tokens, commit_len);
    VF_LAUNCH_CHECK("accept_emit");
    return VF_OK;
}

}  // namespace

int vf_launch_accept(const vf_model *m, const Batch &b, const AcceptBatch &ab, const int32_t *tokens,
                     const float *logits, int32_t *n_accept, int32_t *out_tokens, int32_t *y, hipStream_t st) {
    return launch_all(m, model_scratch(m), b, ab, tokens, logits, n_accept, out_tokens, y, 1, st);
}

// The same kernels with the library's static device scratch instead of the model workspace.
int vf_launch_accept_static(const vf_model *m, const Batch &b, const AcceptBatch &ab, const int32_t *tokens,
                            const float *logits, int32_t *n_accept, int32_t *out_tokens, int32_t *y,
                            hipStream_t st) {
    if (b.total_rows > VF_ACCEPT_STATIC_MAX_ROWS)
        return vf_fail(VF_ERR_CAP, "vf_accept_static: %d rows exceed the static scratch (%d rows)", b.total_rows,
                       VF_ACCEPT_STATIC_MAX_ROWS);
    AcceptScratch sc;
    const int rc = static_scratch(&sc);
    if (rc) return rc;
    return launch_all(m, sc, b, ab, tokens, logits, n_accept, out_tokens, y, 1, st);
}

// Resolves the static scratch of the current device ahead of the first vf_accept_static (set-up time).
int vf_accept_static_init() {
    AcceptScratch sc;
    return static_scratch(&sc);
}

int vf_launch_accept_tree(const vf_model *m, const Batch &b, const AcceptBatch &ab, const TreeDesc &tree,
                          const int32_t *tokens, const float *logits, int32_t *n_accept, int32_t *out_tokens,
                          int32_t *y, int32_t *path, hipStream_t st) {
    const int V = m->cfg.vocab;
    hipLaunchKernelGGL(row_stats_kernel, dim3(VF_STAT_CHUNKS, b.total_rows), dim3(256), 0, st, logits, V, b, ab,
                       m->stat_max, m->stat_idx, m->stat_sum);
    VF_LAUNCH_CHECK("row_stats");
    hipLaunchKernelGGL(accept_tree_decide_kernel, dim3(b.n_seqs), dim3(256), 0, st, logits, V, b, ab, tree, tokens,
                       m->stat_max, m->stat_idx, m->stat_sum, n_accept, out_tokens, y, path, m->draw);
    VF_LAUNCH_CHECK("accept_tree_decide");
    bool any = false;
    for (int i = 0; i < b.n_seqs; ++i) any = any || ab.a[i].mode == VF_STOCHASTIC;
    if (!any) return VF_OK;
    hipLaunchKernelGGL(draw_sums_kernel, dim3(VF_STAT_CHUNKS, b.n_seqs), dim3(256), 0, st, logits, V, m->draw,
                       m->draw_sums);
    VF_LAUNCH_CHECK("draw_sums");
    hipLaunchKernelGGL(accept_emit_kernel, dim3(b.n_seqs), dim3(256), 0, st, logits, V, b, m->draw, m->draw_sums,
                       out_tokens, 1);
    VF_LAUNCH_CHECK("accept_emit");
    return VF_OK;
}

// First generated token from one row of logits: arg-max (temperature 0) or a draw from
// softmax(z / temperature): acceptance with no drafts whose "bonus" token becomes the pending
// token; the length is left alone.
int vf_launch_first_token(const vf_model *m, const SeqDesc &s, const float *logits_row, const float *u,
                          float temperature, hipStream_t st) {
    Batch b;
    b.n_seqs = 1;
    b.total_rows = 1;
    b.s[0] = s;
    b.s[0].row0 = 0;
    b.s[0].nrows = 1;
    AcceptBatch ab;
    ab.a[0].q = nullptr;
    ab.a[0].u = u;  // u[m + acc] with m = 1, acc = 0 is u[1]: see the shift below
    ab.a[0].temperature = temperature > 0.f ? temperature : 1.f;
    ab.a[0].mode = temperature > 0.f ? VF_STOCHASTIC : VF_GREEDY;
    if (u) ab.a[0].u = u - 1;  // the draw reads u[1]; the caller's single uniform sits at u[0]
    int32_t *ws = m->scratch_i32;
    return launch_all(m, model_scratch(m), b, ab, ws + 8, logits_row, ws, ws + 16, ws + 24, 0, st);
}
