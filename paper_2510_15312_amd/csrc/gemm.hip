// Weight-streaming GEMM  Y[rows, N] = X[rows, K] * W[N, K]^T  for few rows.
//
// Every linear layer of the verify forward has at most a few dozen activation rows (the
// pending token plus the drafts; paper Sec. 3 and Sec. 4.3), so the step is bound by reading
// each weight byte once from HBM.  The weights are the MFMA A operand, streamed from global
// memory straight into registers as 1 KiB-per-wavefront contiguous fragments; the activations
// are the B operand, staged in LDS once per workgroup and re-used by all its wavefronts.
// Products are accumulated in float32 and written as split-K partial sums [ks][rows][N]; the
// consumer kernels add the partials in a fixed order, which keeps results bit-reproducible.
#include "vf_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int GEMM_WAVES = 4;
constexpr int PREFETCH = 4;   // weight fragments in flight per stream and wavefront

template <int NB> struct Chunk { static constexpr int KC = (NB <= 2) ? 16 : 8; };

__device__ inline u32x4 load_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// NB: 16-row activation blocks handled per pass; NBW: weight n-blocks per wavefront.
template <int NB, int NBW>
__global__ __launch_bounds__(GEMM_WAVES * 64) VF_MFMA_KERNEL void gemm_bf16_kernel(
    const u32x4 *__restrict__ Wp, const u32x4 *__restrict__ Xp, float *__restrict__ part, int N,
    int KB, int ncb, int row_lo, int row_hi, int ld_rows, int kb_per_split) {
    constexpr int KC = Chunk<NB>::KC;
    __shared__ u32x4 xs[KC * NB * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int NBt = N >> 4;
    const int cb0 = (row_lo >> 4) + blockIdx.z * NB;
    const int nb0 = (blockIdx.x * GEMM_WAVES + wave) * NBW;
    const int kb_begin = blockIdx.y * kb_per_split;
    const int kb_end = min(KB, kb_begin + kb_per_split);
    const bool active = nb0 < NBt;

    floatx4 acc[NBW][NB];
#pragma unroll
    for (int i = 0; i < NBW; ++i)
#pragma unroll
        for (int c = 0; c < NB; ++c) acc[i][c] = floatx4{0.f, 0.f, 0.f, 0.f};

    const u32x4 *wp[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
        int nb = min(nb0 + i, NBt - 1);  // out-of-range streams re-read a valid block, never stored
        wp[i] = Wp + (size_t)nb * KB * 64 + lane;
    }
    u32x4 w[PREFETCH][NBW];
    if (active) {
#pragma unroll
        for (int d = 0; d < PREFETCH; ++d)
            if (kb_begin + d < kb_end)
#pragma unroll
                for (int i = 0; i < NBW; ++i) w[d][i] = load_stream(wp[i] + (size_t)(kb_begin + d) * 64);
    }

    for (int kc = kb_begin; kc < kb_end; kc += KC) {
        const int nk = min(KC, kb_end - kc);
        __syncthreads();
        for (int idx = threadIdx.x; idx < nk * NB * 64; idx += GEMM_WAVES * 64) {
            int l = idx & 63, f = idx >> 6;
            int c = f % NB, kbl = f / NB;
            int cb = cb0 + c;
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (cb < ncb) v = Xp[((size_t)(kc + kbl) * ncb + cb) * 64 + l];
            xs[idx] = v;
        }
        __syncthreads();
        if (!active) continue;
#pragma unroll 1
        for (int k0 = 0; k0 < nk; k0 += PREFETCH) {
#pragma unroll
            for (int d = 0; d < PREFETCH; ++d) {
                const int kbl = k0 + d;
                if (kbl < nk) {
                    bf16x8 a[NBW];
#pragma unroll
                    for (int i = 0; i < NBW; ++i) a[i] = __builtin_bit_cast(bf16x8, w[d][i]);
                    const int nxt = kc + kbl + PREFETCH;
                    if (nxt < kb_end)
#pragma unroll
                        for (int i = 0; i < NBW; ++i) w[d][i] = load_stream(wp[i] + (size_t)nxt * 64);
#pragma unroll
                    for (int c = 0; c < NB; ++c) {
                        bf16x8 b = __builtin_bit_cast(bf16x8, xs[(kbl * NB + c) * 64 + lane]);
#pragma unroll
                        for (int i = 0; i < NBW; ++i)
                            acc[i][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b, acc[i][c], 0, 0, 0);
                    }
                }
            }
        }
    }
    if (!active) return;
    // lane holds Y[row = 16*cb + (lane & 15)][n = 16*nb + 4*(lane >> 4) + 0..3]
    float *out = part + (size_t)blockIdx.y * ld_rows * N;
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
        if (nb0 + i >= NBt) break;
#pragma unroll
        for (int c = 0; c < NB; ++c) {
            int row = (cb0 + c) * 16 + (lane & 15);
            if (row >= row_lo && row < row_hi) {
                float *p = out + (size_t)row * N + (nb0 + i) * 16 + (lane >> 4) * 4;
                *reinterpret_cast<floatx4 *>(p) = acc[i][c];
            }
        }
    }
}

// Many rows (a prefill chunk): workgroup tile = 16*MB rows x TNB weight blocks, NW wavefronts
// of 16*MB/NW rows each.  Per K step of KSTEP 32-wide k-blocks the weight and activation fragments
// go through a double-buffered LDS stage, one barrier per step.  What bounds this kernel is the
// number of bytes a compute unit has in flight, so global loads run NSETS steps ahead of the MFMAs
// through NSETS register sets; they are never predicated (addresses past the end are clamped and
// what they fetch is not used), so the wait before a set's LDS stores leaves the other sets' loads
// in flight, and the barrier orders LDS traffic only.
// Measured on the gate/up GEMM of the 1.5B shape (256 x 17920 x 1536, 28 us): with the MFMAs taken out
// it takes 20 us, with the loop's global loads 23 us, with the LDS reads 21 us: three costs of 5 to 8 us
// that two lock-stepped wavefronts per SIMD overlap poorly, over 7 us of launch, first loads and
// epilogue.  128-row tiles (twice the workgroups), deeper register sets, streaming loads, and a loop
// with three LDS buffers in which a step's LDS reads, LDS writes and memory requests are all issued
// ahead of its MFMAs (27 us) left the time where it was: the three costs add up whatever the order of
// issue, which points at the register file's ports rather than at the pipes.
//
// EPI = ROWS_EPI_TOPK (output head, no K split): instead of the logits the kernel writes, per row and
// column tile, the `topk` largest of the tile's TNB * 16 values with their column ids, in falling
// order, equal values by rising id: candidates for the per-row merge (topk.hip).  A lane holds
// TNB * 4 values of a row and the four lanes l, l + 16, l + 32, l + 48 share a row: one round per
// result, in which every lane offers its best remaining value and two shuffles pick the row's.
//
// EPI = ROWS_EPI_SWIGLU (gate/up matrix, no K split): instead of partial sums the kernel writes
// a = bf16(silu(gate) * up) in activation layout.  Weight block 2j holds gate columns 16j.. and
// block 2j+1 the matching up columns, so a pair of accumulators of one lane holds both factors.
// wavefronts per workgroup and register sets of the two tile shapes
#ifndef ROWS_MB_WIDE
#define ROWS_MB_WIDE 16          // 16-row blocks of the wide tile
#endif
#ifndef ROWS_NW_WIDE
#define ROWS_NW_WIDE 8
#endif
#ifndef ROWS_KSTEP_WIDE
#define ROWS_KSTEP_WIDE 2
#endif
#ifndef ROWS_SETS_WIDE
#define ROWS_SETS_WIDE 2
#endif
#ifndef ROWS_NW_NARROW
#define ROWS_NW_NARROW 4
#endif
#ifndef ROWS_SETS_NARROW
#define ROWS_SETS_NARROW 2
#endif
constexpr int ROWS_EPI_PARTIAL = 0, ROWS_EPI_SWIGLU = 1, ROWS_EPI_TOPK = 2;
template <int TNB, int MB, int KSTEP, int NW, int NSETS, int EPI>
__global__ __launch_bounds__(NW * 64) VF_MFMA_KERNEL
void gemm_rows_kernel(const u32x4 *__restrict__ Wp, const u32x4 *__restrict__ Xp, float *__restrict__ part, int N,
                      int KB, int ncb, int row_lo, int row_hi, int ld_rows, int kb_per_split,
                      int32_t *__restrict__ cand_i, int topk) {
    constexpr bool SWIGLU = EPI == ROWS_EPI_SWIGLU;
    static_assert(!SWIGLU || TNB % 2 == 0, "gate and up blocks come in pairs");
    static_assert(NSETS % 2 == 0, "set s is staged in LDS buffer s & 1");
    constexpr int NT = NW * 64;
    constexpr int NL = KSTEP * TNB * 64 / NT;  // 16-byte weight loads per thread and stage
    static_assert(KSTEP * TNB * 64 % NT == 0, "a stage is a whole number of loads per thread");
    static_assert(MB % NW == 0, "whole activation blocks per wavefront");
    constexpr int WC = MB / NW;               // activation blocks per wavefront
    // Only the weight fragments go through LDS: all wavefronts use them.  A wavefront's activation
    // fragments are its own (its rows, nobody else's), so they stay in the registers they were loaded
    // into; staged like the weights they were 16 of the 24 KB written and 16 of the 80 KB read per
    // k-block of the wide tile, on the port that sets this kernel's pace.
    __shared__ u32x4 lds[2][KSTEP * TNB * 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int NBt = N >> 4;
    const int nb0 = blockIdx.x * TNB;
    const int cb0 = (row_lo >> 4) + blockIdx.z * MB;
    const int kb_begin = blockIdx.y * kb_per_split, kb_end = min(KB, kb_begin + kb_per_split);
    floatx4 acc[TNB][WC];
#pragma unroll
    for (int n = 0; n < TNB; ++n)
#pragma unroll
        for (int c = 0; c < WC; ++c) acc[n][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    if (kb_begin >= kb_end) return;
    // where this thread's weight pieces of a stage come from: piece i is fragment f of k-block `half`
    const u32x4 *src[NL];
    int half_of[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int idx = tid + i * NT, rem = idx % (TNB * 64), f = rem >> 6, l = rem & 63;
        half_of[i] = idx / (TNB * 64);
        src[i] = Wp + (size_t)min(nb0 + f, NBt - 1) * KB * 64 + l;   // rows past N: a valid block, result dropped
    }
    // and its wavefront's activation blocks (rows past the call: a valid block, result dropped)
    const u32x4 *xsrc[WC];
#pragma unroll
    for (int c = 0; c < WC; ++c) xsrc[c] = Xp + (size_t)min(cb0 + wave * WC + c, ncb - 1) * 64 + lane;
    const size_t xstride = (size_t)ncb * 64;
    struct Set {
        u32x4 w[NL];
        u32x4 x[KSTEP][WC];
    };
    auto fetch = [&](Set &r, int kb) {
#pragma unroll
        for (int i = 0; i < NL; ++i) r.w[i] = src[i][(size_t)min(kb + half_of[i], kb_end - 1) * 64];
#pragma unroll
        for (int half = 0; half < KSTEP; ++half)
#pragma unroll
            for (int c = 0; c < WC; ++c) r.x[half][c] = xsrc[c][(size_t)min(kb + half, kb_end - 1) * xstride];
    };
    auto stage = [&](const Set &r, int buf) {
#pragma unroll
        for (int i = 0; i < NL; ++i) lds[buf][tid + i * NT] = r.w[i];
    };
    // kb_limit: k-blocks from here on do not exist (what was fetched for them came from a clamped
    // address); the main loop passes a limit no step reaches, which leaves no test in its code
    auto multiply = [&](int buf, const u32x4 (&x)[KSTEP][WC], int kb, int kb_limit) {
        // The weight fragments of the step's first k-block leave LDS before its first MFMA; those of
        // every further k-block are read under the MFMAs of the one before (one read, then the MFMAs
        // of one weight block), so that only the first k-block of a step waits for LDS.
        bf16x8 afr[2][TNB];
        auto read = [&](int half) {
            const u32x4 *st = lds[buf] + half * TNB * 64;
#pragma unroll
            for (int n = 0; n < TNB; ++n) afr[half & 1][n] = __builtin_bit_cast(bf16x8, st[n * 64 + lane]);
        };
        read(0);
        __builtin_amdgcn_sched_group_barrier(0x100, TNB, 0);
#pragma unroll
        for (int half = 0; half < KSTEP; ++half) {
            if (half + 1 < KSTEP) read(half + 1);
            if (kb + half < kb_limit) {
#pragma unroll
                for (int n = 0; n < TNB; ++n)
#pragma unroll
                    for (int c = 0; c < WC; ++c)
                        acc[n][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[half & 1][n], __builtin_bit_cast(bf16x8, x[half][c]),
                                                                            acc[n][c], 0, 0, 0);
            }
            if (half + 1 < KSTEP) {
#pragma unroll
                for (int n = 0; n < TNB; ++n) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, WC, 0);
                }
            } else {
                __builtin_amdgcn_sched_group_barrier(0x008, TNB * WC, 0);
            }
        }
    };
    Set r[NSETS];
#pragma unroll
    for (int s = 0; s < NSETS; ++s) fetch(r[s], kb_begin + s * KSTEP);
    // Whole groups of NSETS steps first.  An LDS buffer is written again two steps later, behind
    // the barrier of the step in between, which every wavefront reaches only after its MFMAs on
    // that buffer.  The scheduling barriers keep each step's order: stores of its set (the only
    // wait for loads), barrier, the set's next loads, then the MFMAs that hide them.  The step's
    // activation fragments move to registers of their own before the set is requested again.
    constexpr int NEVER = 0x7fffffff;
    const int ngroups = (kb_end - kb_begin) / (NSETS * KSTEP);
    int kb = kb_begin;
    for (int g = 0; g < ngroups; ++g) {
#pragma unroll
        for (int s = 0; s < NSETS; ++s) {
            stage(r[s], s & 1);
            u32x4 x[KSTEP][WC];
#pragma unroll
            for (int half = 0; half < KSTEP; ++half)
#pragma unroll
                for (int c = 0; c < WC; ++c) x[half][c] = r[s].x[half][c];
            lds_sync();
            fetch(r[s], kb + NSETS * KSTEP);
            __builtin_amdgcn_sched_barrier(0);
            multiply(s & 1, x, 0, NEVER);
            __builtin_amdgcn_sched_barrier(0);
            kb += KSTEP;
        }
    }
    // the remaining k-blocks (less than a group) are already in the register sets
#pragma unroll
    for (int s = 0; s < NSETS; ++s) {
        if (kb < kb_end) {
            stage(r[s], s & 1);
            lds_sync();
            multiply(s & 1, r[s].x, kb, kb_end);
            kb += KSTEP;
        }
    }
    if constexpr (EPI == ROWS_EPI_TOPK) {
        constexpr int NV = TNB * 4;
        const int g4 = lane >> 4, n_tiles = gridDim.x;
        float *cand_v = part;
        auto first_of = [](float av, int ai, float bv, int bi) { return av > bv || (av == bv && ai < bi); };
#pragma unroll
        for (int c = 0; c < WC; ++c) {
            const int row = (cb0 + wave * WC + c) * 16 + (lane & 15);
            const bool store = g4 == 0 && row >= row_lo && row < row_hi;
            const size_t o = ((size_t)row * n_tiles + blockIdx.x) * topk;
            // this lane's values of the row; columns past N cannot win
            float v[NV];
#pragma unroll
            for (int e = 0; e < NV; ++e) v[e] = nb0 + e / 4 < NBt ? acc[e / 4][c][e % 4] : -INFINITY;
            const int id0 = nb0 * 16 + g4 * 4;  // id of element e: id0 + 16 * (e / 4) + e % 4
            // one round per result: the best remaining element of the lane, then of the four lanes of
            // the row (l, l + 16, l + 32, l + 48); the lane that owns the winner retires it
#pragma unroll 1
            for (int r = 0; r < topk; ++r) {
                float bv = -INFINITY;
                int bi = 0x7fffffff;
#pragma unroll
                for (int e = 0; e < NV; ++e) {
                    const int id = id0 + 16 * (e / 4) + e % 4;
                    if (v[e] != -INFINITY && first_of(v[e], id, bv, bi)) { bv = v[e]; bi = id; }
                }
#pragma unroll
                for (int off = 16; off <= 32; off <<= 1) {
                    const float ov = __shfl_xor(bv, off, 64);
                    const int oi = __shfl_xor(bi, off, 64);
                    if (first_of(ov, oi, bv, bi)) { bv = ov; bi = oi; }
                }
#pragma unroll
                for (int e = 0; e < NV; ++e)
                    if (id0 + 16 * (e / 4) + e % 4 == bi) v[e] = -INFINITY;
                if (store) {
                    cand_v[o + r] = bv;
                    cand_i[o + r] = bi == 0x7fffffff ? -1 : bi;
                }
            }
        }
    } else if constexpr (SWIGLU) {
        u32x2 *a_out = reinterpret_cast<u32x2 *>(part);  // [kb][cb][lane] fragments of 16 bytes, two halves each
        const int g4 = lane >> 4;
#pragma unroll
        for (int n = 0; n < TNB; n += 2) {
            if (nb0 + n + 1 >= NBt) break;
            const int fb = (nb0 + n) >> 1;  // 16-wide block of a: columns 16*fb + 4*g4 + j
            const int lane_out = ((((fb & 1) << 1) | (g4 >> 1)) << 4) | (lane & 15);
#pragma unroll
            for (int c = 0; c < WC; ++c) {
                const int cb = cb0 + wave * WC + c, row = cb * 16 + (lane & 15);
                if (row < row_lo || row >= row_hi) continue;
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float gt = acc[n][c][j], up = acc[n + 1][c][j];
                    o[j] = gt / (1.0f + expf(-gt)) * up;
                }
                u32x2 packed;
                packed[0] = (unsigned)__builtin_bit_cast(unsigned short, (bf16_t)o[0]) |
                            ((unsigned)__builtin_bit_cast(unsigned short, (bf16_t)o[1]) << 16);
                packed[1] = (unsigned)__builtin_bit_cast(unsigned short, (bf16_t)o[2]) |
                            ((unsigned)__builtin_bit_cast(unsigned short, (bf16_t)o[3]) << 16);
                a_out[((((size_t)(fb >> 1) * ncb + cb) * 64 + lane_out) << 1) | (g4 & 1)] = packed;
            }
        }
    } else {
        float *out = part + (size_t)blockIdx.y * ld_rows * N;
#pragma unroll
        for (int n = 0; n < TNB; ++n) {
            if (nb0 + n >= NBt) break;
#pragma unroll
            for (int c = 0; c < WC; ++c) {
                const int row = (cb0 + wave * WC + c) * 16 + (lane & 15);
                if (row >= row_lo && row < row_hi)
                    *reinterpret_cast<floatx4 *>(out + (size_t)row * N + (nb0 + n) * 16 + (lane >> 4) * 4) = acc[n][c];
            }
        }
    }
}

// float32 model: plain fused-multiply-add GEMM, one wavefront per output column, 8 rows at a time.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ W,
                                                        const float *__restrict__ X,
                                                        float *__restrict__ out, int N, int K,
                                                        int row_lo, int row_hi) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const float *wr = W + (size_t)n * K;
    for (int r0 = row_lo; r0 < row_hi; r0 += 8) {
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int k = lane; k < K; k += 64) {
            float wv = wr[k];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (r0 + i < row_hi) acc[i] = fmaf(wv, X[(size_t)(r0 + i) * K + k], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float v = acc[i];
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0 && r0 + i < row_hi) out[(size_t)(r0 + i) * N + n] = v;
        }
    }
}

template <int NB>
int launch_bf16(const vf_model *m, const void *W, const void *X, float *part, int N, int K, int ncb,
                int row_lo, int row_hi, int ld_rows, GemmPlan plan, hipStream_t st) {
    const int KB = K >> 5, NBt = N >> 4;
    const int kbps = (KB + plan.ks - 1) / plan.ks;
    const int cbs = ((row_hi + 15) >> 4) - (row_lo >> 4);
    dim3 grid((NBt + GEMM_WAVES * plan.nbw - 1) / (GEMM_WAVES * plan.nbw), plan.ks, (cbs + NB - 1) / NB);
    dim3 block(GEMM_WAVES * 64);
    auto args = [&](auto kern) {
        hipLaunchKernelGGL(kern, grid, block, 0, st, (const u32x4 *)W, (const u32x4 *)X, part, N, KB, ncb,
                           row_lo, row_hi, ld_rows, kbps);
    };
    switch (plan.nbw) {
        case 1: args(gemm_bf16_kernel<NB, 1>); break;
        case 2: args(gemm_bf16_kernel<NB, 2>); break;
        default: args(gemm_bf16_kernel<NB, 4>); break;
    }
    VF_LAUNCH_CHECK("gemm_bf16");
    return VF_OK;
}

}  // namespace

GemmPlan vf_gemm_plan(const vf_model *m, int N, int K, int rows, int force_single) {
    GemmPlan p{1, 1, 0, 0, 0, nullptr};
    if (m->cfg.dtype == VF_F32) return p;
    const int NBt = N >> 4, KB = K >> 5;
    if (rows > 64 && m->fast_path) {
        // many-row kernel: 256 rows x 8 weight blocks per workgroup for wide matrices, 128 x 4 for narrow ones
        p.tnb = NBt >= 1024 ? 8 : 4;
        const int groups = (NBt + p.tnb - 1) / p.tnb * (p.tnb == 8 ? (rows + 16 * ROWS_MB_WIDE - 1) / (16 * ROWS_MB_WIDE) : (rows + 127) / 128);
        int ks = 1;
        if (!force_single)
            while (groups * ks < 384 && KB / (ks * 2) >= 8 &&
                   (size_t)ks * 2 * m->cfg.max_rows * N <= m->part_floats) ks *= 2;
        p.ks = ks;
        return p;
    }
    const int groups1 = (NBt + GEMM_WAVES - 1) / GEMM_WAVES;
    if (groups1 >= 4096) p.nbw = 4;
    else if (groups1 >= 2048) p.nbw = 2;
    if (force_single) return p;
    const int groups = (NBt + GEMM_WAVES * p.nbw - 1) / (GEMM_WAVES * p.nbw);
    int ks = 1;
    while (groups * ks < 256 && KB / (ks * 2) >= 4) ks *= 2;
    // the partial buffer must hold ks * ld_rows * N floats
    while (ks > 1 && (size_t)ks * m->cfg.max_rows * N > m->part_floats) ks /= 2;
    p.ks = ks;
    return p;
}

int vf_launch_gemm(const vf_model *m, const void *W, const void *X, float *part, int N, int K,
                   int rows_total, int row_lo, int row_hi, int ld_rows, GemmPlan plan, hipStream_t st) {
    if (row_hi <= row_lo) return VF_OK;
    if (plan.tnb) {
        const int KB = K >> 5, NBt = N >> 4, ncb = (rows_total + 15) >> 4;
        const int kbps = (KB + plan.ks - 1) / plan.ks;
        const int cbs = ((row_hi + 15) >> 4) - (row_lo >> 4);
        const int mb = plan.tnb == 8 ? ROWS_MB_WIDE : 8;
        dim3 grid((NBt + plan.tnb - 1) / plan.tnb, plan.ks, (cbs + mb - 1) / mb);
        auto go = [&](auto kern, int nw) {
            hipLaunchKernelGGL(kern, grid, dim3(nw * 64), 0, st, (const u32x4 *)W, (const u32x4 *)X, part, N, KB, ncb,
                               row_lo, row_hi, ld_rows, kbps, plan.topk_ids, plan.topk);
        };
        if ((plan.swiglu || plan.topk) && plan.ks != 1)
            return vf_fail(VF_ERR_ARG, "the fused epilogues take no K split");
        if (plan.topk) {
            if (plan.topk > VF_TOPK_MAX || !plan.topk_ids) return vf_fail(VF_ERR_ARG, "top-k epilogue: k %d", plan.topk);
            if (plan.tnb == 8) go(gemm_rows_kernel<8, ROWS_MB_WIDE, ROWS_KSTEP_WIDE, ROWS_NW_WIDE, ROWS_SETS_WIDE, ROWS_EPI_TOPK>, ROWS_NW_WIDE);
            else go(gemm_rows_kernel<4, 8, 2, ROWS_NW_NARROW, ROWS_SETS_NARROW, ROWS_EPI_TOPK>, ROWS_NW_NARROW);
        } else if (plan.swiglu) {
            if (plan.tnb == 8) go(gemm_rows_kernel<8, ROWS_MB_WIDE, ROWS_KSTEP_WIDE, ROWS_NW_WIDE, ROWS_SETS_WIDE, ROWS_EPI_SWIGLU>, ROWS_NW_WIDE);
            else go(gemm_rows_kernel<4, 8, 2, ROWS_NW_NARROW, ROWS_SETS_NARROW, ROWS_EPI_SWIGLU>, ROWS_NW_NARROW);
        } else if (plan.tnb == 8) {
            go(gemm_rows_kernel<8, ROWS_MB_WIDE, ROWS_KSTEP_WIDE, ROWS_NW_WIDE, ROWS_SETS_WIDE, ROWS_EPI_PARTIAL>, ROWS_NW_WIDE);
        } else {
            go(gemm_rows_kernel<4, 8, 2, ROWS_NW_NARROW, ROWS_SETS_NARROW, ROWS_EPI_PARTIAL>, ROWS_NW_NARROW);
        }
        VF_LAUNCH_CHECK("gemm_rows");
        return VF_OK;
    }
    if (m->cfg.dtype == VF_F32) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 3) / 4), dim3(256), 0, st, (const float *)W,
                           (const float *)X, part, N, K, row_lo, row_hi);
        VF_LAUNCH_CHECK("gemm_f32");
        return VF_OK;
    }
    const int ncb = (rows_total + 15) >> 4;
    const int cbs = ((row_hi + 15) >> 4) - (row_lo >> 4);
    if (cbs <= 1) return launch_bf16<1>(m, W, X, part, N, K, ncb, row_lo, row_hi, ld_rows, plan, st);
    if (cbs == 2) return launch_bf16<2>(m, W, X, part, N, K, ncb, row_lo, row_hi, ld_rows, plan, st);
    if (cbs == 3) return launch_bf16<3>(m, W, X, part, N, K, ncb, row_lo, row_hi, ld_rows, plan, st);
    return launch_bf16<4>(m, W, X, part, N, K, ncb, row_lo, row_hi, ld_rows, plan, st);
}
