// Acceptance on the device (paper Sec. 3: drafts from the first mismatch on are dropped; Sec. 4.3:
// the accepted prefix x_1..x_{e-1} followed by y_e), greedy and stochastic, and the commit of the
// sequence state (length, pending token) without a host round trip.
//
//   row statistics : per (row, vocabulary chunk): maximum logit, its lowest index and, for stochastic
//                    rows, sum exp((z - chunk max)/T) in float64.
//   decide         : per sequence the chunks are merged in a fixed order (arg-max y of every row,
//                    softmax normaliser), the drafts are walked and the accepted count a is fixed.
//                    Greedy sequences are finished here.
//   draw sums      : stochastic only: per vocabulary chunk the float64 sum of the weights the
//                    replacement (or bonus) token is drawn from at row a.
//   emit           : inverse CDF in id order: finds the chunk, then the id inside it; commits the state.
// Four short launches in stream order.  Each is a chain of a few dependent trips to memory, so inside
// a kernel everything a thread needs is requested together and kept in registers (the logits of a
// chunk for both passes over them, the weights of the chosen chunk, the drafts' logits and draft
// probabilities ahead of the statistics they are compared with).  Merging them into two launches, the
// workgroup that completes a sequence running the second half, measured slower (52 against 44 us
// per step before this was written): the counter that elects that workgroup costs more trips than
// the kernel boundary it replaces.
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

// exp(x) in float64 for x <= 0 (every use here is exp((z - row maximum) / T)), within one unit in the
// last place of the library routine (checked on the host over 2e7 arguments): x = k ln 2 + r with
// |r| <= ln 2 / 2 (ln 2 in two parts, so r is exact to the last bit), exp(r) by its Taylor polynomial of
// degree 13 (truncation below 4e-18), scaled by 2^k.  About twenty float64 operations; the library
// routine, which also serves arguments this code never has, takes several times as many, and these
// kernels spend their time in it.
__device__ inline double exp_nonpos(double x) {
    if (!(x > -745.2)) return 0.0;  // below the smallest subnormal
    const double kf = rint(x * 1.4426950408889634);
    const double r = fma(kf, -1.90821492927058770002e-10, fma(kf, -6.93147180369123816490e-01, x));
    double p = 1.0 / 6227020800.0;
    p = fma(p, r, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)kf);
}

constexpr int ACC_EL = 16;  // logits a thread holds at a time

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

// Statistics of one (row, vocabulary chunk) by one workgroup of 256 threads.
__device__ inline void row_stats_body(const float *__restrict__ logits, int V, const Batch &b, const AcceptBatch &ab,
                                      int row, int chunk, float *__restrict__ smax, int32_t *__restrict__ sidx,
                                      double *__restrict__ ssum) {
    __shared__ MaxIdx rm[4];
    __shared__ double rs[4];
    const int per = (V + VF_STAT_CHUNKS - 1) / VF_STAT_CHUNKS;
    const int v0 = min(V, chunk * per), v1 = min(V, v0 + per);
    const float *z = logits + (size_t)row * V;
    // A thread's logits (ids v0 + thread, + 256, ...) are requested together and kept in registers
    // for the second pass: one trip to memory instead of one per element.  Chunks too long for that
    // (vocabularies beyond 64 * 256 * ACC_EL ids) take the plain loops.
    const bool held = v1 - v0 <= 256 * ACC_EL;
    float zz[ACC_EL];
    MaxIdx best{-INFINITY, 0x7fffffff};
    if (held) {
#pragma unroll
        for (int i = 0; i < ACC_EL; ++i) {
            const int v = v0 + (int)threadIdx.x + i * 256;
            zz[i] = v < v1 ? z[v] : -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < ACC_EL; ++i) {
            const int v = v0 + (int)threadIdx.x + i * 256;
            if (v < v1) best = better(best, MaxIdx{zz[i], v});
        }
    } else {
        for (int v = v0 + threadIdx.x; v < v1; v += 256) best = better(best, MaxIdx{z[v], v});
    }
    best = wave_best(best);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) rm[wave] = best;
    __syncthreads();
    best = better(better(rm[0], rm[1]), better(rm[2], rm[3]));
    const AcceptDesc &a = ab.a[find_seq(b, row)];
    double sum = 0.0;
    if (a.mode == VF_STOCHASTIC && v0 < v1) {
        const double t = (double)a.temperature, cm = (double)best.v;
        if (held) {
#pragma unroll
            for (int i = 0; i < ACC_EL; ++i)
                if (v0 + (int)threadIdx.x + i * 256 < v1) sum += exp_nonpos(((double)zz[i] - cm) / t);
        } else {
            for (int v = v0 + threadIdx.x; v < v1; v += 256) sum += exp_nonpos(((double)z[v] - cm) / t);
        }
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

__global__ __launch_bounds__(256) void row_stats_kernel(const float *__restrict__ logits, int V, Batch b,
                                                        AcceptBatch ab, float *__restrict__ smax,
                                                        int32_t *__restrict__ sidx, double *__restrict__ ssum) {
    row_stats_body(logits, V, b, ab, blockIdx.y, blockIdx.x, smax, sidx, ssum);
}

// The acceptance decision of sequence `seq` by one workgroup of 256 threads.
// commit_len == 0: only the pending token is written (first token after prefill).
struct DecideInputs {   // thread i < k: draft x_i, its logit in row i, its draft probability (1 for a one-hot drafter), uniform u_i
    int x;
    float zx, qx, u;
};
__device__ inline void decide_body(
    const DecideInputs &di, int V, const Batch &b, const AcceptBatch &ab, int seq, const int32_t *__restrict__ tokens,
    const float *smax, const int32_t *sidx, const double *ssum,
    int32_t *__restrict__ n_accept, int32_t *__restrict__ out_tokens, int32_t *__restrict__ y,
    DrawDesc *__restrict__ draw, int commit_len) {
    __shared__ double row_S[VF_MAX_DRAFTS + 1];
    __shared__ float row_max[VF_MAX_DRAFTS + 1];
    __shared__ int row_arg[VF_MAX_DRAFTS + 1];
    __shared__ int ok[VF_MAX_DRAFTS + 1];
    const SeqDesc &s = b.s[seq];
    const AcceptDesc &a = ab.a[seq];
    const int m = s.nrows, k = m - 1;
    const double t = (double)a.temperature;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // rows wave, wave + 4, ... per wavefront, one chunk per lane; the statistics of all of a
    // wavefront's rows are requested before the first is used
    constexpr int RPW = (VF_MAX_DRAFTS + 1 + 3) / 4;
    float mv[RPW];
    int mi[RPW];
    double ms[RPW];
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int r = min(wave + 4 * j, m - 1);
        const size_t o = (size_t)(s.row0 + r) * VF_STAT_CHUNKS + lane;
        mv[j] = smax[o];
        mi[j] = sidx[o];
        ms[j] = a.mode == VF_STOCHASTIC ? ssum[o] : 0.0;
    }
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int r = wave + 4 * j;
        if (r < m) {
            const MaxIdx mine{mv[j], mi[j]};
            const MaxIdx best = wave_best(mine);
            double S = 0.0;
            if (a.mode == VF_STOCHASTIC)
                S = wave_sum(ms[j] != 0.0 ? ms[j] * exp_nonpos(((double)mine.v - (double)best.v) / t) : 0.0);
            if (lane == 0) {
                row_S[r] = S;
                row_max[r] = best.v;
                row_arg[r] = best.i;
                y[s.row0 + r] = best.i;
            }
        }
    }
    __syncthreads();
    const int32_t *drafts = tokens + s.row0 + 1;
    if ((int)threadIdx.x < k) {
        const int i = threadIdx.x, x = di.x;
        int good;
        if (a.mode == VF_GREEDY) {
            good = x == row_arg[i];
        } else if (x < 0 || x >= V) {
            good = 0;
        } else {
            const double px = exp_nonpos(((double)di.zx - (double)row_max[i]) / t) / row_S[i];
            good = (double)di.u * (double)di.qx < px;
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
        n_accept[seq] = acc;
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
        draw[seq] = d;
        if (a.mode == VF_GREEDY) {
            if (commit_len) s.state[0] += 1 + acc;
            s.state[1] = row_arg[acc];
        }
    }
}

// One workgroup per sequence.
__global__ __launch_bounds__(256) void accept_decide_kernel(
    const float *__restrict__ logits, int V, Batch b, AcceptBatch ab, const int32_t *__restrict__ tokens,
    const float *__restrict__ smax, const int32_t *__restrict__ sidx, const double *__restrict__ ssum,
    int32_t *__restrict__ n_accept, int32_t *__restrict__ out_tokens, int32_t *__restrict__ y,
    DrawDesc *__restrict__ draw, int commit_len) {
    const int seq = blockIdx.x;
    // a draft, its logit, its draft probability and its uniform per thread: requested before the statistics
    DecideInputs di;
    {
        const SeqDesc &sq = b.s[seq];
        const AcceptDesc &aq = ab.a[seq];
        const int k = sq.nrows - 1, i = threadIdx.x;
        di.x = -1;
        di.zx = 0.f;
        di.qx = 1.f;
        di.u = 0.f;
        if (i < k) {
            di.x = tokens[sq.row0 + 1 + i];
            if (aq.mode == VF_STOCHASTIC && di.x >= 0 && di.x < V) {
                di.zx = logits[(size_t)(sq.row0 + i) * V + di.x];
                if (aq.q) di.qx = aq.q[(size_t)i * V + di.x];
                di.u = aq.u[i];
            }
        }
    }
    decide_body(di, V, b, ab, seq, tokens, smax, sidx, ssum, n_accept, out_tokens, y, draw, commit_len);
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
            S = wave_sum(sm != 0.0 ? sm * exp_nonpos(((double)mine.v - (double)best.v) / t) : 0.0);
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
            v = exp_nonpos(((double)logits[(size_t)(s.row0 + pr) * V + x] - (double)row_max[pr]) / t) / row_S[pr];
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
struct DrawParams {       // the scalars of a DrawDesc, read once
    double zmax, S, t;
    const float *q;
    const int32_t *excl;  // the descriptor's exclusion list (left in memory: it is indexed at run time)
    int x_excl, n_excl;
};
__device__ inline DrawParams draw_params(const DrawDesc &d) {
    return DrawParams{d.zmax, d.S, d.t, d.q, d.excl, d.x_excl, d.n_excl};
}
// zv: logit of id v; qv: q[v] when there is a dense draft distribution
__device__ inline double draw_weight(float zv, float qv, const DrawParams &d, int v, bool plain) {
    const double p = exp_nonpos(((double)zv - d.zmax) / d.t) / d.S;
    if (plain) return p;
    if (d.q) return fmax(p - (double)qv, 0.0);
    if (v == d.x_excl) return 0.0;
    for (int i = 0; i < d.n_excl; ++i)
        if (v == d.excl[i]) return 0.0;
    return p;
}

__device__ inline double chunk_weight_sum(const float *__restrict__ z, const DrawParams &d, int v0, int v1,
                                          bool plain, double *rs) {
    double sum = 0.0;
    const bool use_q = d.q && !plain;
    if (v1 - v0 <= 256 * ACC_EL) {
        float zz[ACC_EL], qq[ACC_EL];
#pragma unroll
        for (int i = 0; i < ACC_EL; ++i) {
            const int v = v0 + (int)threadIdx.x + i * 256;
            zz[i] = v < v1 ? z[v] : 0.f;
            qq[i] = (use_q && v < v1) ? d.q[v] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < ACC_EL; ++i) {
            const int v = v0 + (int)threadIdx.x + i * 256;
            if (v < v1) sum += draw_weight(zz[i], qq[i], d, v, plain);
        }
    } else {
        for (int v = v0 + threadIdx.x; v < v1; v += 256) sum += draw_weight(z[v], use_q ? d.q[v] : 0.f, d, v, plain);
    }
    sum = wave_sum(sum);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) rs[threadIdx.x >> 6] = sum;
    __syncthreads();
    return ((rs[0] + rs[1]) + rs[2]) + rs[3];
}

// The draw of sequence `seq` by one workgroup of 256 threads, from the per-chunk weight sums.
__device__ inline void emit_body(const float *__restrict__ logits, int V, const Batch &b, int seq,
                                 const DrawDesc *draw, const double *wsum,
                                 int32_t *__restrict__ out_tokens, int commit_len) {
    __shared__ double cs[VF_STAT_CHUNKS];
    __shared__ double seg[256];
    __shared__ double rs[4];
    __shared__ int result;
    const DrawParams d = draw_params(draw[seq]);
    const int d_row = draw[seq].row, d_acc = draw[seq].acc;
    const double d_u = draw[seq].u;
    const SeqDesc &s = b.s[seq];
    const float *z = logits + (size_t)d_row * V;
    const int per = (V + VF_STAT_CHUNKS - 1) / VF_STAT_CHUNKS;
    if (threadIdx.x < VF_STAT_CHUNKS) cs[threadIdx.x] = wsum[seq * VF_STAT_CHUNKS + threadIdx.x];
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
    const double target = d_u * total;
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
    // the chosen chunk, a run of per_t consecutive ids per thread; a thread's weights are worked out
    // once (values requested together) and kept for the second pass
    const int v0 = min(V, cstar * per), v1 = min(V, v0 + per);
    const int per_t = (v1 - v0 + 255) / 256;
    const int a0 = min(v1, v0 + (int)threadIdx.x * per_t), a1 = min(v1, a0 + per_t);
    const bool held = per_t <= ACC_EL, use_q = d.q && !plain;
    double wt[ACC_EL];
    double local = 0.0;
    if (held) {
        float zz[ACC_EL], qq[ACC_EL];
#pragma unroll
        for (int i = 0; i < ACC_EL; ++i) {
            zz[i] = a0 + i < a1 ? z[a0 + i] : 0.f;
            qq[i] = (use_q && a0 + i < a1) ? d.q[a0 + i] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < ACC_EL; ++i) {
            wt[i] = a0 + i < a1 ? draw_weight(zz[i], qq[i], d, a0 + i, plain) : 0.0;
            if (a0 + i < a1) local += wt[i];
        }
    } else {
        for (int v = a0; v < a1; ++v) local += draw_weight(z[v], use_q ? d.q[v] : 0.f, d, v, plain);
    }
    seg[threadIdx.x] = local;
    if (threadIdx.x == 0) result = 0x7fffffff;
    __syncthreads();
    double before = before_chunk;
    for (int j = 0; j < (int)threadIdx.x; ++j) before += seg[j];
    if (before <= target) {
        double run = before;
        if (held) {
            bool found = false;
#pragma unroll
            for (int i = 0; i < ACC_EL; ++i) {
                if (!found && a0 + i < a1) {
                    run += wt[i];
                    if (run > target) { atomicMin(&result, a0 + i); found = true; }
                }
            }
        } else {
            for (int v = a0; v < a1; ++v) {
                run += draw_weight(z[v], use_q ? d.q[v] : 0.f, d, v, plain);
                if (run > target) { atomicMin(&result, v); break; }
            }
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
                if (draw_weight(z[v], use_q ? d.q[v] : 0.f, d, v, plain) > 0.0) w = v;
            if (w < 0) w = max(v0, v1 - 1);
        }
        out_tokens[s.row0 + d_acc] = w;
        if (commit_len) s.state[0] += 1 + d_acc;
        s.state[1] = w;
    }
}

__global__ __launch_bounds__(256) void draw_sums_kernel(const float *__restrict__ logits, int V,
                                                        const DrawDesc *__restrict__ draw,
                                                        double *__restrict__ wsum) {
    __shared__ double rs[4];
    const int seq = blockIdx.y;
    if (!draw[seq].active) return;
    const DrawParams d = draw_params(draw[seq]);
    const int per = (V + VF_STAT_CHUNKS - 1) / VF_STAT_CHUNKS;
    const int v0 = min(V, (int)blockIdx.x * per), v1 = min(V, v0 + per);
    const double sum = chunk_weight_sum(logits + (size_t)draw[seq].row * V, d, v0, v1, false, rs);
    if (threadIdx.x == 0) wsum[seq * VF_STAT_CHUNKS + blockIdx.x] = sum;
}

__global__ __launch_bounds__(256) void accept_emit_kernel(const float *__restrict__ logits, int V, Batch b,
                                                          const DrawDesc *__restrict__ draw,
                                                          const double *__restrict__ wsum,
                                                          int32_t *__restrict__ out_tokens, int commit_len) {
    if (!draw[blockIdx.x].active) return;
    emit_body(logits, V, b, blockIdx.x, draw, wsum, out_tokens, commit_len);
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
