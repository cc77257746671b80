// Reuse of rejected draft tokens (paper Sec. 4.3, "Reuse strategy", Eq. (reuse)): the device
// kernel that finds the segment to keep, and the host-side pool that holds it between steps.
#include "vf_internal.h"

namespace {

struct RowOffsets { int32_t off[VF_MAX_BATCH + 1]; };

// One wavefront per sequence.  Lane i - 1 compares draft x_i with prediction y_i; the agreeing
// positions after the rejection form a bit mask in which lane 0 looks for the longest run, the
// earliest among equals.  Bit j of the mask is position j + 1.
__global__ __launch_bounds__(64) void reuse_select_kernel(RowOffsets ro, const int32_t *__restrict__ tokens,
                                                          const int32_t *__restrict__ y,
                                                          const int32_t *__restrict__ n_accept,
                                                          int32_t *__restrict__ seg) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int row0 = ro.off[b], n = ro.off[b + 1] - row0 - 1;  // n drafts follow the pending token
    const int a = n_accept[b];
    const int i = lane + 1;                                    // draft index of this lane
    bool eq = false;
    if (i <= n && a < n && i > a + 1) eq = tokens[row0 + i] == y[row0 + i - 1];
    const unsigned long long mask = __ballot(eq);
    if (lane != 0) return;
    int best_start = 0, best_len = 0;
    int j = 0;
    while (j < n) {
        if (!((mask >> j) & 1ull)) { ++j; continue; }
        int len = 0;
        while (j + len < n && ((mask >> (j + len)) & 1ull)) ++len;
        if (len > best_len) { best_len = len; best_start = j + 1; }
        j += len;
    }
    seg[2 * b] = best_start;
    seg[2 * b + 1] = best_len;
}

}  // namespace

int vf_reuse_select(int n_seqs, const int32_t *tokens_dev, const int32_t *row_off_host, const int32_t *y_dev,
                    const int32_t *n_accept_dev, int32_t *seg_dev, void *stream) {
    if (n_seqs < 1 || n_seqs > VF_MAX_BATCH) return vf_fail(VF_ERR_ARG, "vf_reuse_select: n_seqs %d", n_seqs);
    if (!tokens_dev || !row_off_host || !y_dev || !n_accept_dev || !seg_dev)
        return vf_fail(VF_ERR_ARG, "vf_reuse_select: NULL argument");
    RowOffsets ro;
    if (row_off_host[0] != 0) return vf_fail(VF_ERR_ARG, "vf_reuse_select: row_off[0] must be 0");
    for (int b = 0; b <= n_seqs; ++b) {
        ro.off[b] = row_off_host[b];
        if (b > 0) {
            const int rows = row_off_host[b] - row_off_host[b - 1];
            if (rows < 1 || rows > VF_MAX_DRAFTS + 1)
                return vf_fail(VF_ERR_ARG, "vf_reuse_select: sequence %d has %d rows", b - 1, rows);
        }
    }
    hipLaunchKernelGGL(reuse_select_kernel, dim3(n_seqs), dim3(64), 0, (hipStream_t)stream, ro, tokens_dev, y_dev,
                       n_accept_dev, seg_dev);
    VF_LAUNCH_CHECK("reuse_select");
    return VF_OK;
}

// ---- the pool: host memory only ----------------------------------------------------------------

int vf_reuse_pool_init(vf_reuse_pool *p, int max_age, int cap) {
    if (!p) return vf_fail(VF_ERR_ARG, "vf_reuse_pool_init: NULL");
    if (max_age < 0 || cap < 1 || cap > VF_MAX_DRAFTS)
        return vf_fail(VF_ERR_ARG, "vf_reuse_pool_init: max_age %d, cap %d", max_age, cap);
    p->len = 0;
    p->age = 0;
    p->max_age = max_age;
    p->cap = cap;
    return VF_OK;
}

int vf_reuse_pool_update(vf_reuse_pool *p, const int32_t *drafts_host, int n_drafts, int seg_start, int seg_len) {
    if (!p) return vf_fail(VF_ERR_ARG, "vf_reuse_pool_update: NULL");
    if (n_drafts < 0 || n_drafts > VF_MAX_DRAFTS || seg_len < 0 ||
        (seg_len > 0 && (!drafts_host || seg_start < 1 || seg_start + seg_len - 1 > n_drafts)))
        return vf_fail(VF_ERR_ARG, "vf_reuse_pool_update: segment [%d, +%d) of %d drafts", seg_start, seg_len,
                       n_drafts);
    if (p->len > 0 && ++p->age > p->max_age) p->len = p->age = 0;
    if (seg_len > p->len) {
        for (int i = 0; i < seg_len; ++i) p->tokens[i] = drafts_host[seg_start - 1 + i];
        p->len = seg_len;
        p->age = 0;
    }
    return VF_OK;
}

int vf_reuse_pool_extend(vf_reuse_pool *p, int32_t *drafts_host, int n_fresh) {
    if (!p || (!drafts_host && n_fresh > 0)) return vf_fail(VF_ERR_ARG, "vf_reuse_pool_extend: NULL");
    if (n_fresh < 0 || n_fresh > p->cap) return vf_fail(VF_ERR_ARG, "vf_reuse_pool_extend: %d fresh drafts", n_fresh);
    if (p->len == 0) return n_fresh;
    if (n_fresh + p->len > p->cap) {
        p->len = p->age = 0;
        return n_fresh;
    }
    for (int i = 0; i < p->len; ++i) drafts_host[n_fresh + i] = p->tokens[i];
    return n_fresh + p->len;
}
