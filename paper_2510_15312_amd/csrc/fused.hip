// The whole verify forward pass (paper Sec. 3 / Sec. 4.3: rows [T, x_1..x_k] of every sequence of
// the batch through all decoder layers and the output head) as ONE persistent kernel.
//
// The grid is sized so that every workgroup is resident at once (one workgroup of eight
// wavefronts per CU); the phases of the pass
//   embed | per layer: QKV, attention, O, gate/up, down | output head
// are separated by grid-wide barriers instead of kernel boundaries.  What this buys over a chain
// of kernels: no launch gap and no ramp-up per phase, and the weight stream pauses only for the
// hand-over of the activations -- a workgroup issues the first loads of its next phase (weights
// do not depend on the previous phase) between arriving at a barrier and waiting on it, and
// inside a phase it refills its register ring with the next work item's fragments during the
// current item's last round.
//
// Memory protocol between workgroups (different compute dies have separate L2 caches):
//   * everything one workgroup writes and another reads later in the launch is stored through
//     to memory (agent-scope stores), and a workgroup waits until its stores have completed
//     before it signals anything (a barrier arrival, a counter) to other workgroups;
//   * bulk data is read with ordinary loads from single-assignment buffers -- one version of
//     the residual stream per half layer, one q / attention output / SwiGLU buffer and one set
//     of attention records per layer -- so no cache can hold a stale line of it: a line is never
//     read before its only write in a launch, and caches start clean at every launch;
//   * data in reused buffers (split-K partial tiles, counters) is read with agent-scope loads.
// The KV cache is written (new rows) and read (all rows) once per layer and launch, in that
// order; tiles that hold new rows are read with agent-scope loads.
//
// Results do not depend on timing: every sum has a fixed order.
#include "fast_common.h"

#include <type_traits>

namespace {

constexpr int FW = 8;            // wavefronts per workgroup
constexpr int FT = FW * 64;      // threads per workgroup
constexpr int FROWS = 48;        // most rows of a call
#ifndef BAR_COUNTERS
#define BAR_COUNTERS 64           // counters a barrier's arrivals are spread over
#endif
constexpr int ATT_COUNTERS = 4096;  // arrival counters of the attention blocks inside the barrier block (uints)
constexpr int LDS_BYTES = 152 * 1024;  // dynamic LDS of the one workgroup a CU holds (160 KB less the static part)
constexpr long long SPIN_LIMIT = 4000000;  // polls before a barrier gives up (seconds, not microseconds)

#ifndef FUSED_PREFETCH_EARLY
#define FUSED_PREFETCH_EARLY 1   // first weight loads of a phase go out before the barrier wait
#endif
#ifndef FUSED_PD_DOWN
#define FUSED_PD_DOWN 5            // ring depth of the down projection (nine fragments per wavefront at the 1.5B shape)
#endif
#ifndef FUSED_AHEAD
#define FUSED_AHEAD 3          // gate/up, down and head phases: this many steps of the item after next are held in registers too (0: off)
#endif
#ifndef FUSED_LAST_MERGES
#define FUSED_LAST_MERGES 1     // attention: the last part to arrive merges the block (0: all parts wait and merge a slice each)
#endif
#ifndef FUSED_FREE_SPLIT
#define FUSED_FREE_SPLIT 1     // a phase of at most one item per workgroup may use a K split that does not divide the grid
#endif
#ifndef FUSED_MAXP
#define FUSED_MAXP 6              // most key parts per attention block (8 parts: 1280 us per launch, 6 1261, 5 1258, 4 1254, 3 1274, 2 1318;
                                  // every setting gives the same mean logit error at the full 1.5B size, 1.3e-2, but with 4 and 5 parts one row
                                  // of 136 lands at 2.12e-2 and 2.005e-2, past the stated 2e-2: 6 is the fastest setting inside it)
#endif
// One workgroup of 8 wavefronts per CU: two wavefronts per SIMD, so each may use up to 256 vector
// registers (weight ring + staging loads in flight) without spilling.
#ifndef FUSED_G
#define FUSED_G 256
#endif

// Pointers that reach the kernel through memory lose their address space; loads through them would
// be generic (flat) loads, which the compiler orders against every other load in flight.
typedef const floatx4 __attribute__((address_space(1))) *global_f4_ptr;
__device__ inline floatx4 load_global_f4(const float *p) { return *(global_f4_ptr)(p); }
typedef const u32x4 __attribute__((address_space(1))) *global_w_ptr;

// Loads from the single-assignment buffers (one version per phase and layer, written once per launch
// before they are read): no cache can hold an older copy of such a line, so an ordinary load will do.
#ifndef FUSED_SSA_PLAIN
#define FUSED_SSA_PLAIN 1
#endif
__device__ __forceinline__ floatx4 ssa_load_f4(const float *p) {
    return FUSED_SSA_PLAIN ? *reinterpret_cast<const floatx4 *>(p) : load_coherent(p);
}
__device__ __forceinline__ u32x4 ssa_load_16(const void *p) {
    return FUSED_SSA_PLAIN ? *reinterpret_cast<const u32x4 *>(p) : load_coherent16(p);
}
__device__ __forceinline__ float ssa_load_f1(const float *p) { return FUSED_SSA_PLAIN ? *p : load_coherent1(p); }

struct FusedLayer {
    const u32x4 *wqkv, *wo, *wgu, *wd;
    const float *attn_norm, *ffn_norm, *bqkv;
};

struct FusedArgs {
    const FusedLayer *layers;
    const bf16_t *embed;
    const u32x4 *lm_head;
    const float *final_norm, *cosv, *sinv;
    const int32_t *tree_depth;      // tree-structured drafts (else NULL): depth and ancestor mask of every row
    const tree_mask_t *tree_anc;
    const int32_t *tokens;
    float *hv;        // residual stream, [2L+1][FROWS][d]
    float *ssv;       // sums of squares of its rows per 16 columns, [2L+1][d/16][64]
    bf16_t *qv, *ov, *av;  // per layer: q [FROWS][Hq*hd], attention output, SwiGLU product [FROWS][F]
    float *att_rec;   // attention records of the key parts, [L][FUSED_G][16][hd + 4]
    float *part;
    int *counters;
    unsigned *bar, *fail;
    float *logits;
    int n_layers, d, F, hq, hkv, hd, vocab, m, has_bias;
    int att_blocks, att_parts;  // (query block, kv head, sequence) blocks of the call; key parts per block
    // First attention work item of every workgroup (-1: none).  Workgroup w runs on compute die w % 8;
    // the map puts the query blocks that read the same keys (same sequence, kv head and key part) on one
    // die, so that its L2 serves all but the first of those reads.
    short att_first[FUSED_G];
    float inv_d, eps, scale_log2e;
    unsigned root0;   // value of the barrier's root counter when this launch starts
    int ks_qkv, ks_o, ks_gu, ks_down, ks_head;
    int gu_light;            // gate/up: the first gu_light workgroups (busy in the O projection) take one unit each (0: even shares)
    int wave_gu, wave_head;  // gate/up, output head: one weight block per wavefront (K unsplit and the staged rows fit)
    int lds_total;    // dynamic LDS bytes of this launch
};

// Counting barrier, split into arrive and wait.  The workgroups are spread over BAR_COUNTERS counters
// (each in a memory channel of its own, so that the increments of a barrier are not all serialised
// at one address); an arrival is one increment that returns nothing, and a barrier is complete when
// every counter has grown by the number of workgroups mapped to it.  Counters only ever grow:
// barrier number e of a launch waits for the counters' value at launch start + e * (G / BAR_COUNTERS).
// Lanes 0..BAR_COUNTERS-1 of the first wavefront poll one counter each.
struct GridBar {
    unsigned *mem, *fail;
    unsigned target, per;  // per: workgroups per counter
    bool dead;
#ifdef FUSED_ARRIVALS
    unsigned long long *stamps;  // [barrier][2][workgroup]: clock at the arrival and at the end of the wait
    int n_arr, n_wait;
#endif
    __device__ __forceinline__ void arrive() {
        stores_done();  // this wavefront's write-through stores have reached memory
        __syncthreads();
#ifdef FUSED_ARRIVALS
        if (threadIdx.x == 0) stamps[((size_t)n_arr * 2) * gridDim.x + blockIdx.x] = wall_clock64();
        ++n_arr;
#endif
        target += per;
        if (threadIdx.x == 0)
            __hip_atomic_fetch_add(mem + (blockIdx.x % BAR_COUNTERS) * 64, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __device__ __forceinline__ void wait() {
        if (threadIdx.x < 64 && !dead) {
            const int lane = threadIdx.x;
            const unsigned *mine = mem + min(lane, BAR_COUNTERS - 1) * 64;
            long long spins = 0;
            for (;;) {
                const bool done = (int)(__hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) >= 0;
                if (__all(done)) break;
                __builtin_amdgcn_s_sleep(1);
                ++spins;
                if (spins > SPIN_LIMIT ||
                    ((spins & 1023) == 0 && __hip_atomic_load(fail, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                    __hip_atomic_store(fail, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    dead = true;  // give up for good: the launch drains without waiting again
                    break;
                }
            }
        }
        lds_sync();
#ifdef FUSED_ARRIVALS
        if (threadIdx.x == 0) stamps[((size_t)n_wait * 2 + 1) * gridDim.x + blockIdx.x] = wall_clock64();
        ++n_wait;
#endif
    }
};

// Optional phase timeline of one workgroup (build with -DFUSED_TRACE=<workgroup>): thread 0 stamps the
// constant-rate clock at the marked points into the second half of the barrier block.
#ifdef FUSED_TRACE
struct Trace {
    unsigned long long *buf;
    int n;
    __device__ __forceinline__ void mark(int id) {
        if (blockIdx.x == FUSED_TRACE && threadIdx.x == 0 && n < 2040) {
            buf[2 * n] = wall_clock64();
            buf[2 * n + 1] = ((unsigned long long)clock64() << 8) | (unsigned long long)id;  // shader-clock count
            ++n;
        }
    }
};
#define TRACE(id) trace.mark(id)
#define TRACE_ARG , Trace &trace
#define TRACE_PASS , trace
#else
#define TRACE(id)
#define TRACE_ARG
#define TRACE_PASS
#endif

// Where a row of the call goes in the KV cache and which rotary angle it takes; the same in every
// layer of a launch (sequence lengths do not change while it runs), so it is worked out once.
struct RowMeta {
    bf16_t *kv;      // the sequence's KV pool
    int n_pages;     // pages in that pool
    int page, tin;   // page and row inside the page of the row's cache slot
    int pos;         // position whose rotary angle the row takes
    int live;        // 0: the slot lies outside the sequence's capacity, nothing is written
};
struct FusedShared {
    float rs_s[64];
    float rs_tmp[FW][64];
    int s_last;
    RowMeta rows[FROWS];
};

// ---- embedding: row r by workgroup r ---------------------------------------------------------------
__device__ __forceinline__ void embed_phase(const FusedArgs &a, const Batch &b) {
    const int d = a.d;
    if (blockIdx.x == gridDim.x - 1)  // arrival counters of the attention blocks start at zero in every launch
        for (int i = threadIdx.x; i < a.att_blocks; i += FT) st_u32<true>(a.bar + ATT_COUNTERS + i, 0u);
    for (int row = blockIdx.x; row < a.m; row += gridDim.x) {
        int tok = a.tokens[row];
        if (tok == VF_PENDING) tok = b.s[find_seq(b, row)].state[1];
        if (tok < 0 || tok >= a.vocab) tok = 0;
        for (int k0 = 0; k0 < d; k0 += FT) {
            const int k = k0 + threadIdx.x;
            float v = 0.f;
            if (k < d) {
                v = (float)a.embed[wfrag_index(tok, k, d)];
                st_f32<true>(a.hv + (size_t)row * d + k, v);
            }
            float sq = v * v;
            sq += __shfl_xor(sq, 8, 64);
            sq += __shfl_xor(sq, 4, 64);
            sq += __shfl_xor(sq, 2, 64);
            sq += __shfl_xor(sq, 1, 64);
            if (k < d && (threadIdx.x & 15) == 0) st_f32<true>(a.ssv + (k >> 4) * 64 + row, sq);
        }
    }
}

#ifndef FUSED_BB_AHEAD
#define FUSED_BB_AHEAD 1          // GEMM phases: activation fragments are read from LDS this many steps ahead of their MFMAs (0: right before)
#endif
#ifndef FUSED_EPI_PREFETCH
#define FUSED_EPI_PREFETCH 1      // what an epilogue reads from memory is requested before the item's MFMA loop
#endif
#ifndef FUSED_SGB
#define FUSED_SGB 1               // GEMM phases: LDS reads are scheduled this many steps ahead of their MFMAs (0: left to the compiler)
#endif
#ifndef FUSED_XP
#define FUSED_XP 16                // activation staging: loads in flight per thread (a multiple of FUSED_STAGE_GROUP)
#endif
#ifndef FUSED_SHORT_COPY
#define FUSED_SHORT_COPY 1          // plain activation staging: a copy of half the depth for calls whose pieces it covers
#endif
#ifndef FUSED_STAGE_GROUP
#define FUSED_STAGE_GROUP 4       // staging of a normalising phase: pieces whose LDS reads (1/rms, gain) are issued together
#endif

// Epilogues of the persistent kernel.  What they read from memory is requested before the item's
// MFMA loop (epi_prefetch) and only used after it, so that no round trip is left between the last
// MFMA and the stores.
//   QKV: bias, rotary embedding, q to its buffer, K and V rows into the cache (row table in LDS)
//   residual: h = h_in + y, and the tile's sums of squares for the next RMSNorm
struct EpiPre { floatx4 v, bias; };
template <int EPI>
__device__ __forceinline__ EpiPre epi_prefetch(const FastGemm &g, const FusedShared &sh, int row, int nb, int lane) {
    EpiPre p;
    p.v = floatx4{0.f, 0.f, 0.f, 0.f};
    p.bias = floatx4{0.f, 0.f, 0.f, 0.f};
    const int n0 = nb * 16 + (lane >> 4) * 4;
    if (EPI == EPI_QKV && g.bias) p.bias = load_global_f4(g.bias + n0);
    if (EPI == EPI_RESID) {
        p.v = ssa_load_f4(g.h_in + (size_t)row * g.N + n0);
    } else if (EPI == EPI_QKV) {
        const int half = g.hd >> 1, i0 = (n0 % g.hd) >> 1;
        const size_t at = (size_t)sh.rows[row].pos * half + i0;   // past the K heads: loaded, not used
        const float2 c = *reinterpret_cast<const float2 *>(g.cosv + at), sn = *reinterpret_cast<const float2 *>(g.sinv + at);
        p.v = floatx4{c.x, sn.x, c.y, sn.y};
    }
    return p;
}
__device__ __forceinline__ void epi_resid_pre(const FastGemm &g, int row, bool live, int nb, int lane, floatx4 v, const EpiPre &pre) {
    const int n0 = nb * 16 + (lane >> 4) * 4;
    floatx4 hv = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        hv = pre.v + v;
        st_f32x4<true>(g.h + (size_t)row * g.N + n0, hv);
    }
    float ssq = hv[0] * hv[0] + hv[1] * hv[1] + hv[2] * hv[2] + hv[3] * hv[3];
    ssq += __shfl_xor(ssq, 16, 64);
    ssq += __shfl_xor(ssq, 32, 64);
    if (live && (lane >> 4) == 0) st_f32<true>(g.ss_out + nb * 64 + row, ssq);
}
__device__ __forceinline__ void epi_qkv_pre(const FastGemm &g, const FusedShared &sh, int row, int nb, int lane, floatx4 v, const EpiPre &pre) {
    const int n0 = nb * 16 + (lane >> 4) * 4;
    const int hd = g.hd, half = hd >> 1;
    v += pre.bias;
    const RowMeta rm = sh.rows[row];
    if (!rm.live) return;
    const int head = n0 / hd, p0 = n0 % hd;
    if (head < g.hq + g.hkv) {
        const int i0 = p0 >> 1;  // packed columns 2i, 2i+1 are elements i and i + hd/2
        const float c0 = pre.v[0], s0 = pre.v[1], c1 = pre.v[2], s1 = pre.v[3];
        const float a0 = v[0] * c0 - v[1] * s0, b0 = v[1] * c0 + v[0] * s0;
        const float a1 = v[2] * c1 - v[3] * s1, b1 = v[3] * c1 + v[2] * s1;
        // i0 is even: elements i0, i0 + 1 are neighbours in either layout, 4-byte aligned
        bf16_t *d0, *d1;
        if (head < g.hq) {
            d0 = g.q + ((size_t)row * g.hq + head) * hd + i0;
            d1 = d0 + half;
        } else {
            d0 = rm.kv + kv_k_index(g.layer, rm.n_pages, rm.page, g.hkv, head - g.hq, rm.tin, i0, hd);
            d1 = rm.kv + kv_k_index(g.layer, rm.n_pages, rm.page, g.hkv, head - g.hq, rm.tin, i0 + half, hd);
        }
        st_u32<true>(d0, pack2_bf16(a0, a1));
        st_u32<true>(d1, pack2_bf16(b0, b1));
    } else {
        const int vh = head - g.hq - g.hkv;
        for (int i = 0; i < 4; ++i) {
            const bf16_t x = (bf16_t)v[i];
            st_u16<true>(rm.kv + kv_v_index(g.layer, rm.n_pages, rm.page, g.hkv, vh, rm.tin, p0 + i, hd),
                         __builtin_bit_cast(unsigned short, x));
        }
    }
}

// Second half of the staging of a normalising phase: x = bf16(h * rstd * gain) for the XP pieces
// (four columns of one row each) this thread loaded, written to the staged activations.  The three
// LDS arrays are distinct (restrict), which lets the reads of later pieces pass the writes of
// earlier ones.  No branch: a piece past the last row was loaded from the last row (clamped) and is
// written there again, the same value its owner writes.
template <int XP>
__device__ __forceinline__ void scale_and_stage(const floatx4 (&v)[XP], const float *__restrict__ rs, const float *__restrict__ gain,
                                                u32x2 *__restrict__ out, int row, int c, int qstep, int rstep, int chunks, int m) {
    constexpr int GRP = FUSED_STAGE_GROUP;  // pieces whose LDS reads are issued together
#pragma unroll
    for (int i0 = 0; i0 < XP; i0 += GRP) {
        float r[GRP];
        floatx4 gv[GRP];
        int at[GRP];
#pragma unroll
        for (int j = 0; j < GRP; ++j) {
            const int rr = min(row, m - 1);
            r[j] = rs[rr];
            gv[j] = *reinterpret_cast<const floatx4 *>(gain + c * 4);
            at[j] = ((c >> 3) * m + rr) * 8 + (c & 7);
            row += qstep;
            c += rstep;
            if (c >= chunks) { c -= chunks; ++row; }
        }
        asm volatile("" ::: "memory");  // the group's reads are issued before its first product
#pragma unroll
        for (int j = 0; j < GRP; ++j) {
            if (i0 + j < XP) {
                const floatx4 x = v[i0 + j < XP ? i0 + j : 0];
                out[at[j]] = pack4_bf16(x[0] * r[j] * gv[j][0], x[1] * r[j] * gv[j][1], x[2] * r[j] * gv[j][2], x[3] * r[j] * gv[j][3]);
            }
        }
    }
}

// ---- GEMM phase -------------------------------------------------------------------------------------
// Work items = (unit of UB weight blocks) x (K split); workgroup w takes items w, w + G, ...  G is
// a multiple of ks, so all items of a workgroup share one K slice and its activations are staged
// in LDS once.  The wavefronts split the slice into equal runs of `cnt` k-blocks (the last run may
// reach past the slice: those steps load a valid fragment again and multiply it by zero), and
// each streams its fragments through a ring of PD registers per weight block, refilled with the
// next item's fragments in the last round.  Trip counts are the same for every wavefront, so the
// loop has no divergent branches.  The caller has arrived at the grid barrier; this function
// waits on it after issuing the first loads.
template <int NB, int UB, int PD, int EPI>
__device__ __forceinline__ void gemm_phase(const FastGemm &g, const Batch &b, GridBar &bar, unsigned char *smem,
                                  int lds_total, FusedShared &sh TRACE_ARG) {
    constexpr bool NORMED = EPI != EPI_RESID;
    constexpr bool COH = EPI != EPI_LOGITS;  // logits are read by the next kernel only
    constexpr int RW = FW / 2;               // wavefronts whose partial sums sit in LDS at a time
    constexpr int RED_BYTES = RW * 2 * NB * 1024;
    constexpr int XP = FUSED_XP;
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));  // per-thread index math is redone per phase instead of living across all of them
    const int lane = tid & 63, wave = tid >> 6;
    const int G = gridDim.x, wg = blockIdx.x;
    const int m = g.m, KB = g.KB, NBt = g.N >> 4;
    const int n_units = (NBt + UB - 1) / UB;
    const int items = n_units * g.ks;
    const int n_my = wg < items ? (items - wg + G - 1) / G : 0;
    const int split = wg % g.ks;
    const int kb0 = split * g.kbps, kb1 = min(KB, kb0 + g.kbps), nk = kb1 - kb0;
    const int cnt = (nk + FW - 1) / FW;          // k-blocks per wavefront, the same for all
    const int rounds = (cnt + PD - 1) / PD;
    const int wk0 = kb0 + wave * cnt;            // this wavefront's run: wk0 .. wk0 + cnt - 1, valid below kb1
    u32x4 *xs = reinterpret_cast<u32x4 *>(smem);
    floatx4 *red = reinterpret_cast<floatx4 *>(smem + lds_total - RED_BYTES);
    float *gain_s = reinterpret_cast<float *>(smem + lds_total - RED_BYTES);  // staging only: red is idle then

    global_w_ptr wp[UB], wpn[UB];
    u32x4 w[PD][UB];
    // AHEAD: a second set of registers holds the first round of the item after next, so that two
    // items' worth of weights are requested before the barrier and during every item
    // slots of the second set; none with three row blocks, whose accumulators leave no room
    constexpr int A2 = (FUSED_AHEAD > 0 && UB == 2 && NB <= 2) ? (FUSED_AHEAD < PD ? FUSED_AHEAD : PD) : 0;
    constexpr bool AHEAD = A2 > 0;
    global_w_ptr wpa[UB];
    u32x4 w2[AHEAD ? A2 : 1][UB];
#pragma unroll
    for (int d = 0; d < PD; ++d)
#pragma unroll
        for (int u = 0; u < UB; ++u) w[d][u] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int d = 0; d < (AHEAD ? A2 : 1); ++d)
#pragma unroll
        for (int u = 0; u < UB; ++u) w2[d][u] = u32x4{0u, 0u, 0u, 0u};
    auto unit_ptrs = [&](int it, global_w_ptr (&dst)[UB]) {
        const int unit = (wg + it * G) / g.ks;
#pragma unroll
        for (int u = 0; u < UB; ++u) dst[u] = (global_w_ptr)g.W + (size_t)min(unit * UB + u, NBt - 1) * KB * 64 + lane;
    };
    auto frag = [&](global_w_ptr base, int kbl) {
        return __builtin_nontemporal_load(base + (size_t)min(wk0 + kbl, kb1 - 1) * 64);
    };
    // Loads are never predicated: a step past the end of the run reads the run's last fragment again
    // (a cache hit) and its product is discarded.  Straight-line loads let the compiler wait for
    // exactly the fragment it needs instead of for everything in flight.
    auto first_fragments = [&]() {
        unit_ptrs(0, wp);
#pragma unroll
        for (int d = 0; d < PD; ++d)
#pragma unroll
            for (int u = 0; u < UB; ++u) w[d][u] = frag(wp[u], min(d, cnt - 1));
        if (AHEAD && n_my > 1) {
            unit_ptrs(1, wpa);
#pragma unroll
            for (int d = 0; d < A2; ++d)
#pragma unroll
                for (int u = 0; u < UB; ++u) w2[d][u] = frag(wpa[u], min(d, cnt - 1));
        }
    };
    if (FUSED_PREFETCH_EARLY && n_my > 0) first_fragments();
    TRACE(1);
    bar.wait();
    TRACE(2);
    if (n_my == 0) return;

    // ---- stage the activations of this K slice: every global load goes out before the first use ----
    if (NORMED) {
        // x = bf16(h * rstd * gain) with rstd = 1/rms from the per-16-column sums of squares
        // (lane = row, wavefront = every FW-th block of columns); pieces of four columns
        const int chunks = nk * 8, pieces = m * chunks;
        const int qstep = FT / chunks, rstep = FT % chunks;
        // sums of squares of the column blocks wave, wave + FW, ... of row `lane`: the block index is
        // the same for the whole wavefront, so the scalar unit forms each address (uniform base +
        // per-lane offset) and the 0/1 factor of a block past the last.  Lanes past the last row
        // read the last row's sums; their 1/rms is never used.
        float t[16];
        const int wave_s = __builtin_amdgcn_readfirstlane(wave);
        const unsigned ss_lane = (unsigned)min(lane, m - 1);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int j = wave_s + i * FW;
            t[i] = ssa_load_f1(g.ss_in + min(j, g.n_ss - 1) * 64 + ss_lane) * (j < g.n_ss ? 1.f : 0.f);
        }
        floatx4 gn = load_global_f4(g.gain + (size_t)kb0 * 32 + min(tid, chunks - 1) * 4);
        const float *xh_slice = g.Xh + (size_t)kb0 * 32;
        for (int base = 0; base < pieces; base += FT * XP) {
            floatx4 v[XP];
            int row = (base + tid) / chunks, c = (base + tid) % chunks;
            const int row0 = row, c0 = c;
#pragma unroll
            for (int i = 0; i < XP; ++i) {
                v[i] = ssa_load_f4(xh_slice + (unsigned)(min(row, m - 1) * KB * 32 + c * 4));  // uniform base + 32-bit offset
                row += qstep;
                c += rstep;
                if (c >= chunks) { c -= chunks; ++row; }
            }
            if (base == 0) {
                if (!FUSED_PREFETCH_EARLY) first_fragments();
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += t[i];
                if (lane < m)
                    for (int j = wave + 16 * FW; j < g.n_ss; j += FW) sum += ssa_load_f1(g.ss_in + j * 64 + lane);
                sh.rs_tmp[wave][lane] = sum;
                for (int cc = tid; cc < chunks; cc += FT) {
                    if (cc != tid) gn = load_global_f4(g.gain + (size_t)kb0 * 32 + cc * 4);
                    *reinterpret_cast<floatx4 *>(gain_s + cc * 4) = gn;
                }
                lds_sync();
                TRACE(6);
                if (tid < 64) {
                    float part[FW], tot = 0.f;
#pragma unroll
                    for (int j = 0; j < FW; ++j) part[j] = sh.rs_tmp[j][tid];
                    asm volatile("" ::: "memory");  // the eight reads are issued together
#pragma unroll
                    for (int j = 0; j < FW; ++j) tot += part[j];
                    sh.rs_s[tid] = 1.0f / sqrtf(tot * g.inv_d + g.eps);
                }
                lds_sync();
                TRACE(7);
            }
            scale_and_stage<XP>(v, sh.rs_s, gain_s, reinterpret_cast<u32x2 *>(xs), row0, c0, qstep, rstep, chunks, m);
        }
    } else {
        const int chunks = nk * 4, pieces = m * chunks;
        const int qstep = FT / chunks, rstep = FT % chunks;
        const bf16_t *x_slice = g.X + (size_t)kb0 * 32;
        // passes of `depth` loads in flight per thread; few pieces (a K slice of a call of few rows)
        // take the short copy, which issues half as many loads that only repeat the last row
        auto stage_copy = [&](auto depth_tag) {
            constexpr int D = decltype(depth_tag)::value;
            for (int base = 0; base < pieces; base += FT * D) {
                u32x4 v[D];
                int row = (base + tid) / chunks, c = (base + tid) % chunks;
                const int row0 = row, c0 = c;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    v[i] = ssa_load_16(x_slice + (unsigned)(min(row, m - 1) * KB * 32 + c * 8));  // uniform base + 32-bit offset
                    row += qstep;
                    c += rstep;
                    if (c >= chunks) { c -= chunks; ++row; }
                }
                if (!FUSED_PREFETCH_EARLY && base == 0) first_fragments();
                row = row0;
                c = c0;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    const int rr = min(row, m - 1);  // a piece past the last row: the last row's, written again
                    xs[((c >> 2) * m + rr) * 4 + (c & 3)] = v[i];
                    row += qstep;
                    c += rstep;
                    if (c >= chunks) { c -= chunks; ++row; }
                }
            }
        };
        if (FUSED_SHORT_COPY && pieces <= FT * (XP / 2)) stage_copy(std::integral_constant<int, XP / 2>{});
        else stage_copy(std::integral_constant<int, XP>{});
    }
    lds_sync();
    TRACE(3);

    int xoff[NB];  // this lane's 16 bytes of row block c inside a k-block of the staged activations
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        const int row = min(c * 16 + (lane & 15), m - 1);
        xoff[c] = row * 4 + (lane >> 4);
    }

    for (int it = 0; it < n_my; ++it) {
        const bool has_next = it + 1 < n_my;
        const bool has_ahead = AHEAD && it + 2 < n_my;
        unit_ptrs(has_next ? it + 1 : it, wpn);
        if (AHEAD) unit_ptrs(has_ahead ? it + 2 : it, wpa);
        const int unit = (wg + it * G) / g.ks;
        const int nb0 = unit * UB;
        floatx4 acc[UB][NB];
#pragma unroll
        for (int u = 0; u < UB; ++u)
#pragma unroll
            for (int c = 0; c < NB; ++c) acc[u][c] = floatx4{0.f, 0.f, 0.f, 0.f};
        // this thread's epilogue tile (whole wavefronts: NTH is a multiple of 64) and what its epilogue reads
        constexpr int NTH_ = EPI == EPI_SWIGLU ? NB * 64 : UB * NB * 64;
        EpiPre pre;
        pre.v = floatx4{0.f, 0.f, 0.f, 0.f};
        pre.bias = floatx4{0.f, 0.f, 0.f, 0.f};
        if (FUSED_EPI_PREFETCH && (EPI == EPI_RESID || EPI == EPI_QKV) && tid < NTH_) {
            const int eu = tid / (NB * 64), ec = (tid >> 6) % NB;
            pre = epi_prefetch<EPI>(g, sh, min(ec * 16 + (lane & 15), m - 1), min(nb0 + eu, NBt - 1), lane);
        }
        // One round = PD steps of straight-line code.  REFILL: after its use every slot is loaded
        // again, with the same item's next round or, in the last round, the next item's first; the
        // final round of the final item has nothing left to load and runs without.
        auto round_body = [&](auto refill_tag, int r) {
            constexpr bool REFILL = decltype(refill_tag)::value;
            const bool last_round = r + 1 == rounds;
            global_w_ptr rp[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) rp[u] = last_round ? wpn[u] : wp[u];
            const int rbase = last_round ? 0 : (r + 1) * PD;
            // activation fragments leave LDS FUSED_BB_AHEAD steps before the MFMAs that use them, so
            // that no MFMA waits for a read issued right in front of it
            constexpr int BA = FUSED_BB_AHEAD < PD ? FUSED_BB_AHEAD : PD - 1;
            bf16x8 bb[BA + 1][NB];
            auto read_bb = [&](int d) {
                const int kx = min(wk0 + min(r * PD + d, cnt - 1), kb1 - 1) - kb0;
#pragma unroll
                for (int c = 0; c < NB; ++c) bb[d % (BA + 1)][c] = __builtin_bit_cast(bf16x8, xs[kx * m * 4 + xoff[c]]);
            };
#pragma unroll
            for (int d = 0; d < BA; ++d) read_bb(d);
#pragma unroll
            for (int d = 0; d < PD; ++d) {
                const int kbl = r * PD + d;
                const bool live = kbl < cnt && wk0 + kbl < kb1;
                bf16x8 a[UB];
#pragma unroll
                for (int u = 0; u < UB; ++u) a[u] = __builtin_bit_cast(bf16x8, live ? w[d][u] : u32x4{0u, 0u, 0u, 0u});
                if (REFILL) {
                    if (AHEAD && d < A2 && last_round) {
                        // the next item's first round is already here; its slot takes the one after
#pragma unroll
                        for (int u = 0; u < UB; ++u) w[d][u] = w2[d][u];
                        if (has_ahead) {
#pragma unroll
                            for (int u = 0; u < UB; ++u) w2[d][u] = frag(wpa[u], min(d, cnt - 1));
                        }
                    } else {
#pragma unroll
                        for (int u = 0; u < UB; ++u) w[d][u] = frag(rp[u], min(rbase + d, cnt - 1));
                    }
                }
                if (d + BA < PD) read_bb(d + BA);
#pragma unroll
                for (int c = 0; c < NB; ++c) {
                    const bf16x8 b1 = bb[d % (BA + 1)][c];
#pragma unroll
                    for (int u = 0; u < UB; ++u)
                        acc[u][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b1, acc[u][c], 0, 0, 0);
                }
            }
            // Order of the round's LDS reads and MFMAs for the instruction scheduler: the reads of
            // the first steps, then per step its MFMAs followed by the reads of a later step, so
            // that an MFMA never waits for a read issued right in front of it.
            if (FUSED_SGB > 0) {
                constexpr int SA = FUSED_SGB < PD ? FUSED_SGB : PD;
                __builtin_amdgcn_sched_group_barrier(0x100, SA * NB, 0);
#pragma unroll
                for (int d = 0; d < PD; ++d) {
                    __builtin_amdgcn_sched_group_barrier(0x008, UB * NB, 0);
                    if (d + SA < PD) __builtin_amdgcn_sched_group_barrier(0x100, NB, 0);
                }
            }
        };
#pragma unroll 1
        for (int r = 0; r + 1 < rounds; ++r) round_body(std::true_type{}, r);
        if (has_next) round_body(std::true_type{}, rounds - 1);
        else round_body(std::false_type{}, rounds - 1);
        TRACE(4);
        // ---- wavefront partial sums: upper half through LDS into the lower half, then all four ----
        // (the LDS reads of a stage are issued together, ahead of the first sum: the empty asm
        // statements keep the compiler from moving each read down to its use)
        if (wave >= RW) {
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int c = 0; c < NB; ++c) red[(((wave - RW) * UB + u) * NB + c) * 64 + lane] = acc[u][c];
        }
        lds_sync();
        if (wave < RW) {
            floatx4 other[UB][NB];
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int c = 0; c < NB; ++c) other[u][c] = red[((wave * UB + u) * NB + c) * 64 + lane];
            asm volatile("" ::: "memory");
#pragma unroll
            for (int u = 0; u < UB; ++u)
#pragma unroll
                for (int c = 0; c < NB; ++c) red[((wave * UB + u) * NB + c) * 64 + lane] = acc[u][c] + other[u][c];
        }
        lds_sync();

        constexpr int NT = UB * NB * 64;                       // tiles of 4 outputs per unit
        constexpr int NTH = EPI == EPI_SWIGLU ? NB * 64 : NT;  // tiles with an epilogue of their own
        static_assert(NTH <= FT, "one tile per thread");
        const int t = tid;
        floatx4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = {0.f, 0.f, 0.f, 0.f};
        if (t < NTH) {
            floatx4 p0[RW], p1[RW];
            if (EPI == EPI_SWIGLU) {
                const int c = t >> 6;
#pragma unroll
                for (int ww = 0; ww < RW; ++ww) {
                    p0[ww] = red[((ww * UB + 0) * NB + c) * 64 + lane];
                    p1[ww] = red[((ww * UB + (UB - 1)) * NB + c) * 64 + lane];
                }
            } else {
                const int u = t / (NB * 64), c = (t >> 6) % NB;
#pragma unroll
                for (int ww = 0; ww < RW; ++ww) {
                    p0[ww] = red[((ww * UB + u) * NB + c) * 64 + lane];
                    p1[ww] = floatx4{0.f, 0.f, 0.f, 0.f};
                }
            }
            asm volatile("" ::: "memory");
#pragma unroll
            for (int ww = 0; ww < RW; ++ww) {
                v0 += p0[ww];
                if (EPI == EPI_SWIGLU) v1 += p1[ww];
            }
        }
        bool do_epi = true;
        if (g.ks > 1) {
            float *mine = g.part + ((size_t)(unit * g.ks + split) * NT) * 4;
            if (t < NTH) {
                store_coherent(mine + (size_t)t * 4, v0);
                if (EPI == EPI_SWIGLU) store_coherent(mine + (size_t)(NTH + t) * 4, v1);
            }
            stores_done();
            __syncthreads();
            if (tid == 0) {
                const int old = __hip_atomic_fetch_add(g.counters + unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sh.s_last = old == g.ks - 1;
                if (old == g.ks - 1) __hip_atomic_store(g.counters + unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
            do_epi = sh.s_last != 0;
            if (do_epi && t < NTH) {
                v0 = floatx4{0.f, 0.f, 0.f, 0.f};
                v1 = floatx4{0.f, 0.f, 0.f, 0.f};
                for (int sp0 = 0; sp0 < g.ks; sp0 += 8) {
                    floatx4 t0[8], t1[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        t0[i] = floatx4{0.f, 0.f, 0.f, 0.f};
                        t1[i] = floatx4{0.f, 0.f, 0.f, 0.f};
                        if (sp0 + i < g.ks) {
                            const float *p = g.part + ((size_t)(unit * g.ks + sp0 + i) * NT) * 4;
                            t0[i] = load_coherent(p + (size_t)t * 4);
                            if (EPI == EPI_SWIGLU) t1[i] = load_coherent(p + (size_t)(NTH + t) * 4);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        v0 += t0[i];
                        v1 += t1[i];
                    }
                }
            }
        }
        if (do_epi && t < NTH) {  // whole wavefronts: NTH is a multiple of 64
            const int u = EPI == EPI_SWIGLU ? 0 : t / (NB * 64), c = (t >> 6) % NB;
            const int nb = nb0 + u;
            const int row = c * 16 + (lane & 15);
            const bool live = row < m && nb < NBt;
            if (EPI == EPI_RESID) {
                if (FUSED_EPI_PREFETCH) epi_resid_pre(g, row, live, nb, lane, v0, pre);
                else epi_resid<COH>(g, row, live, nb, lane, v0);
            } else if (live) {
                if (EPI == EPI_QKV && FUSED_EPI_PREFETCH) epi_qkv_pre(g, sh, row, nb, lane, v0, pre);
                else if (EPI == EPI_QKV) epi_qkv<COH>(g, b, row, nb, lane, v0);
                else if (EPI == EPI_SWIGLU) epi_swiglu<COH>(g, row, nb, lane, v0, v1);
                else __builtin_nontemporal_store(v0, reinterpret_cast<floatx4 *>(g.logits + (size_t)row * g.N + nb * 16 + (lane >> 4) * 4));
            }
        }
        TRACE(5);
        if (has_next) {
            lds_sync();  // the partial sums in LDS are consumed before the next item's arrive
#pragma unroll
            for (int u = 0; u < UB; ++u) wp[u] = wpn[u];
        }
    }
}

// ---- GEMM phase with whole weight blocks per wavefront ---------------------------------------------------
// For the matrices with many more 16-row blocks than a K split across workgroups could use (gate/up,
// output head) and a K that fits LDS whole.  A wavefront streams its share of a block's fragments
// through a ring of RING registers and keeps the accumulators to itself: no partial sums in LDS
// per work item, no workgroup barrier inside the streaming loop.  Every wavefront of the chip holds
// RING fragments in flight, issued before the barrier wait; what limits a compute unit's share of
// the stream is the bytes it has in flight, so all eight wavefronts of a workgroup carry a ring.
//   gate/up: a pass covers two units of the workgroup (unit = 16 ffn columns: a block of gate rows
//            and a block of up rows); its eight tasks (unit, gate | up, lower | upper half of K) go
//            to the eight wavefronts.  At the end of a pass the four tiles of a unit meet in LDS;
//            wavefront q of the unit adds the halves of row block q and applies SwiGLU.
//   head:    blocks w, w + W, ... (W = wavefronts of the grid) per wavefront, full K, one after
//            the other through the same ring; logits are stored from the accumulators.
#ifndef FUSED_WRING
#define FUSED_WRING 24
#endif
#ifndef FUSED_ATT_TOP
#define FUSED_ATT_TOP 1         // attention items go to the workgroups at the top of the grid
#endif
#ifndef FUSED_GU_LIGHT
#define FUSED_GU_LIGHT 1        // gate/up: workgroups busy in the O projection take one unit, the others share the rest
#endif
#ifndef FUSED_GU_REV
#define FUSED_GU_REV 1          // gate/up: the units of a partial last range go to the workgroups at the top of the grid
#endif
#ifndef FUSED_WXP
#define FUSED_WXP 8             // activation staging of these phases: loads in flight per thread (the ring is live meanwhile)
#endif
#ifndef FUSED_WAVE_PHASES
#define FUSED_WAVE_PHASES 1     // 1: gate/up and the output head run this way when K is not split across workgroups
#endif
constexpr int WAVE_TAIL_BYTES = 24 * 1024;  // LDS kept free behind the staged activations: the gain vector (up to
                                            // 6144 columns) while staging, then the tiles of a pass (FW * NB KB)
template <int NB, int EPI>
__device__ __forceinline__ void wave_phase(const FastGemm &g, int n_light, GridBar &bar, unsigned char *smem, int lds_total,
                                           FusedShared &sh TRACE_ARG) {
    static_assert(EPI == EPI_SWIGLU || EPI == EPI_LOGITS, "gate/up and output head");
    static_assert(FW * NB * 1024 <= WAVE_TAIL_BYTES && NB <= 4, "a pass's tiles fit the tail; one row block per wavefront of a unit");
    constexpr int RING = FUSED_WRING, XP = FUSED_WXP;
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = gridDim.x, wg = blockIdx.x;
    const int m = g.m, KB = g.KB, NBt = g.N >> 4;
    u32x4 *xs = reinterpret_cast<u32x4 *>(smem);
    floatx4 *exch = reinterpret_cast<floatx4 *>(smem + lds_total - WAVE_TAIL_BYTES);
    float *gain_s = reinterpret_cast<float *>(smem + lds_total - WAVE_TAIL_BYTES);  // staging only

    // this wavefront's tasks: block of task j = blk0 + j * bstride, all over the K range [kb_lo, kb_hi)
    // (gate/up: pass j, slot s covers units (2j + s) G .. + G; a range that the units fill only in part is
    //  handed out from the top workgroup downwards: the workgroups at the bottom of the grid are the ones
    //  busy in the O projection before, and the last to start here)
    // (With n_light > 0 the first n_light workgroups -- the ones that work in the O projection and so
    //  start here last, their weight ring requested behind everybody else's -- take one unit each, and
    //  the others, which have had their rings in flight since the O projection began, share the rest:
    //  unit n_light + (wg - n_light) + t H for t = 0, 1, 2, ..., H = G - n_light.)
    int blk0, bstride, n_task, kb_lo, kb_hi, passes, blk_last = -1;
    if (EPI == EPI_SWIGLU) {
        const int n_units = NBt >> 1, slot = wave >> 2, KBh = (KB + 1) >> 1;
        const int sub = (wave >> 1) & 1;
        if (n_light > 0) {
            const int H = G - n_light, T = (max(n_units - n_light, 0) + H - 1) / H;
            passes = max(1, (T + 1) / 2);
            if (wg < n_light) {
                blk0 = 2 * wg + sub;
                bstride = 0;
                n_task = (slot == 0 && wg < n_units) ? 1 : 0;
            } else {
                const int u0 = n_light + (wg - n_light) + slot * H;
                blk0 = 2 * u0 + sub;
                bstride = 4 * H;
                n_task = u0 < n_units ? (n_units - u0 + 2 * H - 1) / (2 * H) : 0;
            }
        } else {
            blk0 = 2 * (wg + slot * G) + sub;
            bstride = 4 * G;
            passes = max(1, (n_units + 2 * G - 1) / (2 * G));
            n_task = 0;
            for (int j = 0; j < passes; ++j) {
                const int start = (2 * j + slot) * G, left = n_units - start;
                if (left >= G) ++n_task;
                else if (left > 0) {
                    const int idx = FUSED_GU_REV ? G - 1 - wg : wg;
                    if (idx < left) { blk_last = 2 * (start + idx) + sub; ++n_task; }
                }
            }
        }
        kb_lo = (wave & 1) ? KBh : 0;
        kb_hi = (wave & 1) ? KB : KBh;
    } else {
        const int gw = wave * G + wg, W = FW * G;          // neighbouring blocks on different compute units
        blk0 = gw;
        bstride = W;
        n_task = gw < NBt ? (NBt - gw + W - 1) / W : 0;
        kb_lo = 0;
        kb_hi = KB;
        passes = n_task;
    }
    const int rpt = max(1, (kb_hi - kb_lo + RING - 1) / RING);  // rounds per task
    const int rounds = n_task * rpt;
    global_w_ptr wbase = (global_w_ptr)g.W + lane;
    u32x4 w[RING];
#pragma unroll
    for (int d = 0; d < RING; ++d) w[d] = u32x4{0u, 0u, 0u, 0u};
    // fragment of flat round r, slot d.  Never predicated: a step past the end of the K range (or of
    // the wavefront's tasks) reads a valid fragment again and its product is discarded.
    auto task_block = [&](int j) { return (j == n_task - 1 && blk_last >= 0) ? blk_last : blk0 + j * bstride; };
    auto frag = [&](int r, int d) {
        const int j = min(r / rpt, max(n_task - 1, 0));
        const int kb = min(kb_lo + (r % rpt) * RING + d, kb_hi - 1);
        const size_t blk = (size_t)min(task_block(j), NBt - 1);
        return __builtin_nontemporal_load(wbase + (blk * KB + kb) * 64);
    };
    if (n_task > 0) {
#pragma unroll
        for (int d = 0; d < RING; ++d) w[d] = frag(0, d);
    }
    TRACE(1);
    bar.wait();
    TRACE(2);

    // ---- stage x = bf16(h * rstd * gain) for the whole K (as in gemm_phase, one slice) ----
    {
        const int nk = KB, chunks = nk * 8, pieces = m * chunks;
        const int qstep = FT / chunks, rstep = FT % chunks;
        float t[16];
        const unsigned ss_lane = (unsigned)min(lane, m - 1);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int j = wave + i * FW;
            t[i] = ssa_load_f1(g.ss_in + min(j, g.n_ss - 1) * 64 + ss_lane) * (j < g.n_ss ? 1.f : 0.f);
        }
        floatx4 gn = load_global_f4(g.gain + min(tid, chunks - 1) * 4);
        for (int base = 0; base < pieces; base += FT * XP) {
            floatx4 v[XP];
            int row = (base + tid) / chunks, c = (base + tid) % chunks;
            const int row0 = row, c0 = c;
#pragma unroll
            for (int i = 0; i < XP; ++i) {
                v[i] = ssa_load_f4(g.Xh + (unsigned)(min(row, m - 1) * KB * 32 + c * 4));
                row += qstep;
                c += rstep;
                if (c >= chunks) { c -= chunks; ++row; }
            }
            if (base == 0) {
                float sum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += t[i];
                if (lane < m)
                    for (int j = wave + 16 * FW; j < g.n_ss; j += FW) sum += ssa_load_f1(g.ss_in + j * 64 + lane);
                sh.rs_tmp[wave][lane] = sum;
                for (int cc = tid; cc < chunks; cc += FT) {
                    if (cc != tid) gn = load_global_f4(g.gain + cc * 4);
                    *reinterpret_cast<floatx4 *>(gain_s + cc * 4) = gn;
                }
                lds_sync();
                TRACE(6);
                if (tid < 64) {
                    float part[FW], tot = 0.f;
#pragma unroll
                    for (int j = 0; j < FW; ++j) part[j] = sh.rs_tmp[j][tid];
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int j = 0; j < FW; ++j) tot += part[j];
                    sh.rs_s[tid] = 1.0f / sqrtf(tot * g.inv_d + g.eps);
                }
                lds_sync();
                TRACE(7);
            }
            scale_and_stage<XP>(v, sh.rs_s, gain_s, reinterpret_cast<u32x2 *>(xs), row0, c0, qstep, rstep, chunks, m);
        }
    }
    lds_sync();
    TRACE(3);

    int xoff[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) xoff[c] = min(c * 16 + (lane & 15), m - 1) * 4 + (lane >> 4);

    floatx4 acc[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    // one round = RING steps of straight-line code; REFILL: every slot is loaded again after its
    // use with the fragment of the next round (the same task's next K range or the next task)
    auto round_body = [&](auto refill_tag, int r) {
        constexpr bool REFILL = decltype(refill_tag)::value;
        const int kbase = kb_lo + (r % rpt) * RING;
        constexpr int BA = FUSED_BB_AHEAD < RING ? FUSED_BB_AHEAD : RING - 1;
        bf16x8 bb[BA + 1][NB];
        auto read_bb = [&](int d) {
            const int kx = min(kbase + d, kb_hi - 1);
#pragma unroll
            for (int c = 0; c < NB; ++c) bb[d % (BA + 1)][c] = __builtin_bit_cast(bf16x8, xs[kx * m * 4 + xoff[c]]);
        };
#pragma unroll
        for (int d = 0; d < BA; ++d) read_bb(d);
#pragma unroll
        for (int d = 0; d < RING; ++d) {
            const bool live = kbase + d < kb_hi;
            const bf16x8 a = __builtin_bit_cast(bf16x8, live ? w[d] : u32x4{0u, 0u, 0u, 0u});
            if (REFILL) w[d] = frag(r + 1, d);
            if (d + BA < RING) read_bb(d + BA);
#pragma unroll
            for (int c = 0; c < NB; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bb[d % (BA + 1)][c], acc[c], 0, 0, 0);
        }
        if (FUSED_SGB > 0) {
            constexpr int SA = FUSED_SGB < RING ? FUSED_SGB : RING;
            __builtin_amdgcn_sched_group_barrier(0x100, SA * NB, 0);
#pragma unroll
            for (int d = 0; d < RING; ++d) {
                __builtin_amdgcn_sched_group_barrier(0x008, NB, 0);
                if (d + SA < RING) __builtin_amdgcn_sched_group_barrier(0x100, NB, 0);
            }
        }
    };

#pragma unroll 1
    for (int j = 0; j < passes; ++j) {
        const bool mine = j < n_task;
        if (mine) {
#pragma unroll 1
            for (int rr = 0; rr < rpt; ++rr) {
                const int r = j * rpt + rr;
                if (r + 1 < rounds) round_body(std::true_type{}, r);
                else round_body(std::false_type{}, r);
            }
        }
        TRACE(4);
        const int nb = task_block(j);
        if (EPI == EPI_LOGITS) {
#pragma unroll
            for (int c = 0; c < NB; ++c) {
                const int row = c * 16 + (lane & 15);
                if (row < m)
                    __builtin_nontemporal_store(acc[c], reinterpret_cast<floatx4 *>(g.logits + (size_t)row * g.N + nb * 16 + (lane >> 4) * 4));
                acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
        } else {
            // tile (wavefront w, row block c) at exch[(w * NB + c) * 64 + lane]; wavefronts 4u .. 4u + 3 hold
            // unit u's gate lower, gate upper, up lower, up upper half
            if (j) lds_sync();   // the previous pass's tiles have been read
            if (mine) {
#pragma unroll
                for (int c = 0; c < NB; ++c) exch[(wave * NB + c) * 64 + lane] = acc[c];
            }
            lds_sync();
            const int q = wave & 3, w0 = wave & ~3;
            if (mine && q < NB) {
                floatx4 t4[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) t4[i] = exch[((w0 + i) * NB + q) * 64 + lane];
                asm volatile("" ::: "memory");
                const int row = q * 16 + (lane & 15);
                if (row < m) epi_swiglu<true>(g, row, nb & ~1, lane, t4[0] + t4[1], t4[2] + t4[3]);
            }
#pragma unroll
            for (int c = 0; c < NB; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        TRACE(5);
    }
}

// ---- attention phase -----------------------------------------------------------------------------------
// Work item = (block of 16 query items, kv head, sequence, part of the keys); a query item is a
// (row, head of the group) pair.  The eight wavefronts of a workgroup take the 32-key tiles of the
// part in turn; K and V^T fragments go from the cache straight into registers in MFMA operand
// order (no LDS staging: every fragment is used by exactly one wavefront).  Scores
// S^T[key, item] = K Q^T leave the MFMA with eight keys per lane once the K rows are fed in the
// order 8*(rho >> 2) + (rho & 3) (+ 4 for the second 16-key block): that is the B-operand layout
// of O^T[d, item] += V^T[d, key] P[key, item], and the matching V^T fragment is one 16-byte load.
// Wavefront results (running max, sum, O^T) are merged through LDS; with several parts the
// merged partials go to memory and the last workgroup to arrive merges the parts.  No second
// grid-wide phase is needed for the merge.
constexpr int FKT = ATT_TILE;  // keys per tile

// (sequence, kv head, query block, key part) of attention work item i
struct AttItem { int seq, kvh, qb, part, blk; };
__device__ __forceinline__ AttItem att_item(const FusedArgs &a, const Batch &b, int i) {
    const int group = a.hq / a.hkv;
    AttItem it;
    it.part = i / a.att_blocks;
    it.blk = i % a.att_blocks;
    int blk = it.blk, seq = 0;
    while (seq + 1 < b.n_seqs) {
        const int nb_seq = a.hkv * ((b.s[seq].nrows * group + 15) >> 4);
        if (blk < nb_seq) break;
        blk -= nb_seq;
        ++seq;
    }
    const int nqb = (b.s[seq].nrows * group + 15) >> 4;
    it.seq = seq;
    it.kvh = blk / nqb;
    it.qb = blk % nqb;
    return it;
}

// len0: length of the sequence of this workgroup's first item, read once per launch (lengths do
// not change during a launch).
template <int HD>
__device__ __forceinline__ void attn_phase(const FusedArgs &a, const Batch &b, int layer, const bf16_t *q, bf16_t *o,
                                  int len0, GridBar &bar, unsigned char *smem, FusedShared &sh TRACE_ARG) {
    constexpr int KD = HD / 32, DB = HD / 16, REC = HD + ATTF_STRIDE_PAD, MAXP = FUSED_MAXP;
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    // the wavefront's number as a scalar: which tile it takes, and whether that tile holds keys of
    // this launch, are then decided by scalar branches
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g4 = lane >> 4, l15 = lane & 15;
    const int G = gridDim.x, hq = a.hq, hkv = a.hkv, group = hq / hkv, P = a.att_parts;
    floatx4 *o_s = reinterpret_cast<floatx4 *>(smem);                      // [wave][db][lane]
    float *ml_s = reinterpret_cast<float *>(smem + FW * DB * 64 * 16);    // [wave][2][16]
    const int n_work = a.att_blocks * P;
    AttTile<HD> tile;
    auto tile_range = [&](const SeqDesc &s, const AttItem &it, int len, int &t_begin, int &t_end, int &kmax) {
        kmax = min(len + s.nrows, s.capacity);  // keys 0..kmax-1 exist
        const int blk_last = min(kmax - 1, len + min(s.nrows - 1, (it.qb * 16 + 15) / group));
        const int tiles = blk_last / FKT + 1, tpp = (tiles + P - 1) / P;
        t_begin = it.part * tpp;
        t_end = min(tiles, t_begin + tpp);
    };
    // keys below the sequence length were written by earlier calls: a first tile made of them is
    // loaded before the barrier wait
    bool preloaded = false;
    const int i_first = a.att_first[blockIdx.x];
    if (i_first >= 0) {
        const AttItem it = att_item(a, b, i_first);
        int t_begin, t_end, kmax;
        tile_range(b.s[it.seq], it, len0, t_begin, t_end, kmax);
        const int t = t_begin + wave;
        if (t < t_end && (t + 1) * FKT <= len0) {
            tile.load(b.s[it.seq], layer, hkv, it.kvh, t, false, lane);
            preloaded = true;
        }
    }
    TRACE(1);
    bar.wait();
    TRACE(2);
    // further items (more work than workgroups; then there is one part per block) follow in steps of G
    for (int i = i_first; i >= 0 && i < n_work; i += G) {
        const AttItem it = att_item(a, b, i);
        const SeqDesc &s = b.s[it.seq];
        const int kvh = it.kvh, part = it.part;
        const int n_items = s.nrows * group;
        const int len = i == i_first ? len0 : s.state[0];
        int t_begin, t_end, kmax;
        tile_range(s, it, len, t_begin, t_end, kmax);
        const int item = it.qb * 16 + l15;
        const bool valid = item < n_items;
        const int r = valid ? item / group : 0, head = kvh * group + (valid ? item % group : 0);
        const int row = s.row0 + r;
        const int last_key = valid ? len + r : -1;
        // a value every lane shares (kernel argument and the item's sequence length)
        const int own_base = a.tree_anc ? __builtin_amdgcn_readfirstlane(len) : ATT_NO_TREE;
        const tree_mask_t own_mask = a.tree_anc && valid ? a.tree_anc[row] : 0;

        bf16x8 qf[KD];
#pragma unroll
        for (int kd = 0; kd < KD; ++kd)
            qf[kd] = __builtin_bit_cast(bf16x8, ssa_load_16(q + ((size_t)row * hq + head) * HD + kd * 32 + g4 * 8));
        AttState<HD> st;
#pragma unroll
        for (int db = 0; db < DB; ++db) st.o[db] = floatx4{0.f, 0.f, 0.f, 0.f};
        st.m_run = -1e30f;
        st.l_run = 0.f;
#pragma unroll 1
        for (int t = t_begin + wave; t < t_end; t += FW) {
            const int t0 = t * FKT;
            if (!preloaded) tile.load(s, layer, hkv, kvh, t, (t + 1) * FKT > len, lane);
            preloaded = false;
            tile.mask_values(t0, kmax, lane);
            att_tile_update<HD>(st, qf, tile, t0, last_key, own_base, own_mask, a.scale_log2e, lane);
        }
        preloaded = false;
        TRACE(20);
        // ---- merge of the eight wavefronts through LDS ----
        if (i != i_first) lds_sync();  // the previous item's merge has been read
#pragma unroll
        for (int db = 0; db < DB; ++db) o_s[(wave * DB + db) * 64 + lane] = st.o[db];
        if (g4 == 0) {
            ml_s[(wave * 2 + 0) * 16 + l15] = st.m_run;
            ml_s[(wave * 2 + 1) * 16 + l15] = st.l_run;
        }
        lds_sync();
        // thread (db = wave, lane) owns O^T[d = 16*db + 4*g4 + j][item l15]; HD = 64 leaves waves 4..7 idle
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        float M = -1e30f, L = 0.f;
        if (wave < DB) {
            // all LDS reads of the merge are issued together, ahead of the arithmetic
            float mw[FW], lw[FW];
            floatx4 ow[FW];
#pragma unroll
            for (int w = 0; w < FW; ++w) {
                mw[w] = ml_s[(w * 2) * 16 + l15];
                lw[w] = ml_s[(w * 2 + 1) * 16 + l15];
                ow[w] = o_s[(w * DB + wave) * 64 + lane];
            }
            asm volatile("" ::: "memory");
#pragma unroll
            for (int w = 0; w < FW; ++w) M = fmaxf(M, mw[w]);
#pragma unroll
            for (int w = 0; w < FW; ++w) {
                const float wt = exp2f(mw[w] - M);
                L += lw[w] * wt;
                acc += ow[w] * wt;
            }
        }
        TRACE(21);
        if (P > 1) {
            // Merge across the parts of the block without a second grid-wide phase: every part
            // leaves its record in memory and counts itself in; once all P have (all of them are
            // resident and none has other work left, so the wait ends), part p merges the d-blocks
            // p, p + P, ... of all records -- wavefront w takes d-block p + w * P -- and writes
            // that slice of the output.
            float *base = a.att_rec + ((size_t)layer * FUSED_G + (size_t)it.blk * P) * 16 * REC;
            float *mine = base + (size_t)part * 16 * REC;
            if (wave < DB) {
                if (wave == 0 && g4 == 0) st_u32x2<true>(mine + l15 * REC, __builtin_bit_cast(u32x2, float2{M, L}));
                st_f32x4<true>(mine + l15 * REC + ATTF_STRIDE_PAD + wave * 16 + g4 * 4, acc);
            }
            stores_done();
            __syncthreads();
#if FUSED_LAST_MERGES
            // the part that counts itself in last merges the whole block (wavefront w takes d-block w);
            // the others are done: nobody waits, nothing is polled
            if (tid == 0) {
                unsigned *cnt = a.bar + ATT_COUNTERS + it.blk;
                const unsigned old = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sh.s_last = old + 1u == (unsigned)P * (unsigned)(layer + 1);
            }
            __syncthreads();
            TRACE(22);
            const int db = sh.s_last ? wave : DB;
#else
            if (tid == 0) {
                unsigned *cnt = a.bar + ATT_COUNTERS + it.blk;
                __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const unsigned want = (unsigned)P * (unsigned)(layer + 1);
                long long spins = 0;
                while (!bar.dead && __hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < want) {
                    __builtin_amdgcn_s_sleep(1);
                    if (++spins > SPIN_LIMIT) {
                        __hip_atomic_store(a.fail, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        bar.dead = true;
                    }
                }
            }
            lds_sync();
            TRACE(22);
            const int db = part + wave * P;
#endif
            if (db < DB) {
                // all records in flight at once (slots past P repeat the last part and weigh nothing);
                // the records of a layer have a buffer of their own, so ordinary loads see them
                float mp[MAXP], lp[MAXP];
                floatx4 op[MAXP];
#pragma unroll
                for (int pp = 0; pp < MAXP; ++pp) {
                    const float *rec = base + ((size_t)min(pp, P - 1) * 16 + l15) * REC;
                    const floatx4 hd4 = ssa_load_f4(rec);  // [max, sum, -, -]
                    mp[pp] = hd4[0];
                    lp[pp] = hd4[1];
                    op[pp] = ssa_load_f4(rec + ATTF_STRIDE_PAD + db * 16 + g4 * 4);
                }
                float Mg = -1e30f;
#pragma unroll
                for (int pp = 0; pp < MAXP; ++pp) Mg = fmaxf(Mg, mp[pp]);
                float Lg = 0.f;
                floatx4 og = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int pp = 0; pp < MAXP; ++pp) {
                    const float wt = pp < P ? exp2f(mp[pp] - Mg) : 0.f;
                    Lg += lp[pp] * wt;
                    og += op[pp] * wt;
                }
                if (valid) {
                    const float inv = 1.0f / Lg;
                    st_u32x2<true>(o + (size_t)row * hq * HD + head * HD + db * 16 + g4 * 4,
                                   pack4_bf16(og[0] * inv, og[1] * inv, og[2] * inv, og[3] * inv));
                }
            }
        } else if (wave < DB && valid) {
            const float inv = 1.0f / L;
            st_u32x2<true>(o + (size_t)row * hq * HD + head * HD + wave * 16 + g4 * 4,
                           pack4_bf16(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv));
        }
    }
}

#ifndef FUSED_MINW
#define FUSED_MINW 2
#endif
template <int NB, int HD>
__global__ __launch_bounds__(FT, FUSED_MINW) void verify_fused_kernel(FusedArgs a, Batch b) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ FusedShared sh;
#ifdef FUSED_ARRIVALS
    // debug build: stamps go behind the first 64 rows of the logits buffer (the model workspace's, when the caller passes none)
    GridBar bar{a.bar, a.fail, a.root0, gridDim.x / BAR_COUNTERS, false,
                reinterpret_cast<unsigned long long *>(a.logits + (size_t)64 * a.vocab), 0, 0};
#else
    GridBar bar{a.bar, a.fail, a.root0, gridDim.x / BAR_COUNTERS, false};
#endif
    const int d = a.d, F = a.F, hd = a.hd, nq = a.hq * hd, nkv = a.hkv * hd;
    const size_t hstride = (size_t)FROWS * d, sstride = (size_t)(d / 16) * 64;

#ifdef FUSED_TRACE
    Trace trace{reinterpret_cast<unsigned long long *>(a.bar + 8192), 0};
#endif
    // length of the sequence of this workgroup's first attention item (lengths are constant during a launch)
    int len0 = 0;
    if (a.att_first[blockIdx.x] >= 0) len0 = b.s[att_item(a, b, a.att_first[blockIdx.x]).seq].state[0];
    if ((int)threadIdx.x < FROWS) {
        const int row = min((int)threadIdx.x, a.m - 1);
        const SeqDesc &s = b.s[find_seq(b, row)];
        const int len = s.state[0], slot = len + (row - s.row0);
        RowMeta rm;
        rm.kv = reinterpret_cast<bf16_t *>(s.kv);
        rm.n_pages = s.n_pages;
        rm.live = slot >= 0 && slot < s.capacity;
        rm.page = rm.live ? kv_page(s, slot) : 0;
        rm.tin = rm.live ? slot % VF_TILE : 0;
        rm.pos = rm.live ? (a.tree_depth ? len + a.tree_depth[row] : slot) : 0;
        sh.rows[threadIdx.x] = rm;
    }
    TRACE(0);
    embed_phase(a, b);
    bar.arrive();   // (a workgroup barrier inside: the row table is visible to every wavefront from here on)

    FastGemm base;
    base.m = a.m;
    base.part = a.part;
    base.counters = a.counters;
    base.n_ss = d / 16;
    base.inv_d = a.inv_d;
    base.eps = a.eps;
    base.F = F;
    base.cosv = a.cosv;
    base.sinv = a.sinv;
    base.depth = a.tree_depth;
    base.hq = a.hq;
    base.hkv = a.hkv;
    base.hd = hd;
    base.kch = 0;
    base.X = nullptr; base.Xh = nullptr; base.gain = nullptr; base.ss_in = nullptr; base.h_in = nullptr;
    base.h = nullptr; base.ss_out = nullptr; base.a_out = nullptr; base.logits = nullptr; base.bias = nullptr;
    base.q = nullptr; base.layer = 0;

#pragma unroll 1
    for (int l = 0; l < a.n_layers; ++l) {
        const FusedLayer lp = a.layers[l];
        float *h0 = a.hv + (size_t)(2 * l) * hstride, *h1 = h0 + hstride, *h2 = h1 + hstride;
        float *ss0 = a.ssv + (size_t)(2 * l) * sstride, *ss1 = ss0 + sstride, *ss2 = ss1 + sstride;
        bf16_t *q = a.qv + (size_t)l * FROWS * nq, *o = a.ov + (size_t)l * FROWS * nq;
        bf16_t *act = a.av + (size_t)l * FROWS * F;
        {
            FastGemm g = base;
            g.W = lp.wqkv; g.N = nq + 2 * nkv; g.KB = d / 32; g.Xh = h0; g.gain = lp.attn_norm; g.ss_in = ss0;
            g.bias = a.has_bias ? lp.bqkv : nullptr; g.layer = l; g.q = q;
            g.ks = a.ks_qkv; g.kbps = (g.KB + g.ks - 1) / g.ks;
            gemm_phase<NB, 1, 6, EPI_QKV>(g, b, bar, smem, a.lds_total, sh TRACE_PASS);
        }
        bar.arrive();
        TRACE(10);
        attn_phase<HD>(a, b, l, q, o, len0, bar, smem, sh TRACE_PASS);
        bar.arrive();
        TRACE(13);
        {
            FastGemm g = base;
            g.W = lp.wo; g.N = d; g.KB = nq / 32; g.X = o; g.h_in = h0; g.h = h1; g.ss_out = ss1;
            g.ks = a.ks_o; g.kbps = (g.KB + g.ks - 1) / g.ks;
            gemm_phase<NB, 1, 6, EPI_RESID>(g, b, bar, smem, a.lds_total, sh TRACE_PASS);
        }
        bar.arrive();
        TRACE(14);
        {
            FastGemm g = base;
            g.W = lp.wgu; g.N = 2 * F; g.KB = d / 32; g.Xh = h1; g.gain = lp.ffn_norm; g.ss_in = ss1; g.a_out = act;
            g.ks = a.ks_gu; g.kbps = (g.KB + g.ks - 1) / g.ks;
            if (a.wave_gu) wave_phase<NB, EPI_SWIGLU>(g, a.gu_light, bar, smem, a.lds_total, sh TRACE_PASS);
            else gemm_phase<NB, 2, 6, EPI_SWIGLU>(g, b, bar, smem, a.lds_total, sh TRACE_PASS);
        }
        bar.arrive();
        TRACE(15);
        {
            FastGemm g = base;
            g.W = lp.wd; g.N = d; g.KB = F / 32; g.X = act; g.h_in = h1; g.h = h2; g.ss_out = ss2;
            g.ks = a.ks_down; g.kbps = (g.KB + g.ks - 1) / g.ks;
            gemm_phase<NB, 2, FUSED_PD_DOWN, EPI_RESID>(g, b, bar, smem, a.lds_total, sh TRACE_PASS);
        }
        bar.arrive();
        TRACE(16);
    }
    {
        FastGemm g = base;
        g.W = a.lm_head; g.N = a.vocab; g.KB = d / 32;
        g.Xh = a.hv + (size_t)(2 * a.n_layers) * hstride; g.gain = a.final_norm;
        g.ss_in = a.ssv + (size_t)(2 * a.n_layers) * sstride; g.logits = a.logits;
        g.ks = a.ks_head; g.kbps = (g.KB + g.ks - 1) / g.ks;
        if (a.wave_head) wave_phase<NB, EPI_LOGITS>(g, 0, bar, smem, a.lds_total, sh TRACE_PASS);
        else gemm_phase<NB, 2, 6, EPI_LOGITS>(g, b, bar, smem, a.lds_total, sh TRACE_PASS);
    }
    TRACE(99);
#ifdef FUSED_ARRIVALS
    if (threadIdx.x == 0) bar.stamps[((size_t)bar.n_arr * 2) * gridDim.x + blockIdx.x] = wall_clock64();  // end of the head phase
#endif
}

// ---- host side -------------------------------------------------------------------------------------

// Largest K slice (in 32-wide blocks) whose activations fit LDS next to the partial sums.
int slice_limit(int lds_total, int rows, int nb) {
    const int x_bytes = lds_total - (FW / 2) * 2 * nb * 1024;
    return x_bytes / (rows * 64);
}

// K split for a phase: a divisor of G, at least what LDS demands; with allow_fill as many more
// splits as keep the item count within one item per workgroup.  0: nothing fits.
int pick_split(int G, int lds_total, int units, int KB, int rows, int nb, bool allow_fill) {
    const int lim = slice_limit(lds_total, rows, nb);
    int best = 0;
    for (int ks = 1; ks <= G && ks <= KB; ++ks) {
        // workgroup w takes items w, w + G, ...: they share a K slice if ks divides G, or if there is
        // at most one item per workgroup
        if (G % ks && !(FUSED_FREE_SPLIT && allow_fill && units * ks <= G)) continue;
        const int kbps = (KB + ks - 1) / ks;
        if ((KB + kbps - 1) / kbps != ks) continue;  // every split must own k-blocks
        if (kbps > lim) continue;
        if (!best) best = ks;
        if (!allow_fill) break;
        if (units * ks <= G && kbps >= FW) best = ks;
    }
    return best;
}

template <int NB, int HD>
int launch_fused(vf_model *m, FusedArgs &a, const Batch &b, int G, hipStream_t st) {
    auto kern = verify_fused_kernel<NB, HD>;
    static int max_wgs = -1;  // workgroups that can be resident at once
    if (max_wgs < 0) {
        VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   LDS_BYTES));
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        VF_HIP(hipGetDevice(&dev));
        VF_HIP(hipGetDeviceProperties(&prop, dev));
        VF_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kern), FT, LDS_BYTES));
        max_wgs = per_cu * prop.multiProcessorCount;
    }
    if (G > max_wgs)
        return vf_fail(VF_ERR_UNSUPPORTED, "persistent kernel: %d workgroups wanted, %d can be resident", G, max_wgs);
    hipLaunchKernelGGL(kern, dim3(G), dim3(FT), a.lds_total, st, a, b);
    VF_LAUNCH_CHECK("verify_fused");
    return VF_OK;
}

}  // namespace

size_t vf_fused_workspace_bytes(const vf_config &c) {
    if (c.dtype != VF_BF16) return 0;
    const size_t L = c.n_layers, d = c.d_model, nq = (size_t)c.n_q_heads * c.head_dim, F = c.d_ffn;
    size_t n = 0;
    auto add = [&](size_t bytes) { n += (bytes + 255) & ~(size_t)255; };
    add((2 * L + 1) * FROWS * d * 4);
    add((2 * L + 1) * (d / 16) * 64 * 4);
    add(L * FROWS * nq * 2);
    add(L * FROWS * nq * 2);
    add(L * FROWS * F * 2);
    add(L * FUSED_G * 16 * ((size_t)c.head_dim + ATTF_STRIDE_PAD) * 4);
    add(65536);
    add(L * sizeof(FusedLayer));
    return n;
}

int vf_fused_init(vf_model *m, char *ws, hipStream_t st) {
    const vf_config &c = m->cfg;
    const size_t L = c.n_layers, d = c.d_model, nq = (size_t)c.n_q_heads * c.head_dim, F = c.d_ffn;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = ws + off; off += (bytes + 255) & ~(size_t)255; return p; };
    m->fz_h = (float *)take((2 * L + 1) * FROWS * d * 4);
    m->fz_ss = (float *)take((2 * L + 1) * (d / 16) * 64 * 4);
    m->fz_q = take(L * FROWS * nq * 2);
    m->fz_o = take(L * FROWS * nq * 2);
    m->fz_a = take(L * FROWS * F * 2);
    m->fz_att = (float *)take(L * FUSED_G * 16 * ((size_t)c.head_dim + ATTF_STRIDE_PAD) * 4);
    m->fz_bar = (unsigned *)take(65536);
    m->fz_layers = take(L * sizeof(FusedLayer));
    std::vector<FusedLayer> host(L);
    for (size_t l = 0; l < L; ++l) {
        const LayerPacked &lp = m->layers[l];
        host[l] = FusedLayer{(const u32x4 *)lp.wqkv, (const u32x4 *)lp.wo, (const u32x4 *)lp.wgu, (const u32x4 *)lp.wd,
                             lp.attn_norm, lp.ffn_norm, lp.bqkv};
    }
    VF_HIP(hipMemcpyAsync(m->fz_layers, host.data(), L * sizeof(FusedLayer), hipMemcpyHostToDevice, st));
    VF_HIP(hipStreamSynchronize(st));  // the host array goes away
    m->fz_epoch = 0;
    return VF_OK;
}

// Whether the persistent kernel can run this call; fills the grid size, LDS size and K splits.
// K splits of the six GEMM phases for a call of `rows` rows (nb blocks of 16), and the floats of
// partial-sum workspace they need.  false: some phase does not fit.
struct Splits { int qkv, o, gu, down, head; };
static bool plan_splits(const vf_config &c, int rows, int nb, Splits *sp, size_t *part_floats) {
    const int d = c.d_model, F = c.d_ffn, hd = c.head_dim, nq = c.n_q_heads * hd, nkv = c.n_kv_heads * hd;
    if (c.dtype != VF_BF16 || rows > FROWS || d % 64) return false;
    if (std::max(std::max((nq + 2 * nkv) / 16, F / 16), (c.vocab / 16 + 1) / 2) > VF_N_COUNTERS) return false;
    const int G = FUSED_G, lds = LDS_BYTES;
    if (G % BAR_COUNTERS) return false;
    sp->qkv = pick_split(G, lds, (nq + 2 * nkv) / 16, d / 32, rows, nb, false);
    sp->o = pick_split(G, lds, d / 16, nq / 32, rows, nb, false);
    sp->gu = pick_split(G, lds, F / 16, d / 32, rows, nb, false);
    sp->down = pick_split(G, lds, (d / 16 + 1) / 2, F / 32, rows, nb, true);
    sp->head = pick_split(G, lds, (c.vocab / 16 + 1) / 2, d / 32, rows, nb, false);
    if (!sp->qkv || !sp->o || !sp->gu || !sp->down || !sp->head) return false;
    // the gain slice of a normalising phase is staged where the partial sums go later
    const int red_bytes = (FW / 2) * 2 * nb * 1024;
    auto slice_bytes = [&](int ks) { return (d / 32 + ks - 1) / ks * 128; };
    if (slice_bytes(sp->gu) > red_bytes || slice_bytes(sp->qkv) > red_bytes || slice_bytes(sp->head) > red_bytes)
        return false;
    // partial tiles of the split phases: units * ks tiles of UB * NB * 256 floats
    size_t tiles = std::max(std::max((nq + 2 * nkv) / 16 * sp->qkv, d / 16 * sp->o),
                            std::max(F / 16 * sp->gu, (d / 16 + 1) / 2 * sp->down));
    if (sp->head > 1) tiles = std::max(tiles, (size_t)((c.vocab / 16 + 1) / 2) * sp->head);
    *part_floats = tiles * 2 * nb * 256;
    return true;
}

// Partial-sum workspace (floats) the persistent kernel may ask for with this model, over all row counts.
size_t vf_fused_part_floats(const vf_config &c) {
    size_t need = 0;
    for (int nb = 1; nb * 16 <= FROWS; ++nb) {
        if (c.max_rows < (nb - 1) * 16 + 1) break;
        // the most rows a call of nb blocks can have: the smallest K slices, the most splits
        Splits sp;
        size_t pf = 0;
        if (plan_splits(c, std::min(nb * 16, (int)c.max_rows), nb, &sp, &pf)) need = std::max(need, pf);
    }
    return need;
}

static bool plan_fused(const vf_model *m, const Batch &b, FusedArgs &a, int *G_out) {
    if (!m->fz_h) return false;
    const int rows = b.total_rows, nb = (rows + 15) / 16;
    Splits sp;
    size_t pf = 0;
    if (!plan_splits(m->cfg, rows, nb, &sp, &pf) || pf > m->part_floats) return false;
    a.ks_qkv = sp.qkv;
    a.ks_o = sp.o;
    a.ks_gu = sp.gu;
    a.ks_down = sp.down;
    a.ks_head = sp.head;
    a.lds_total = LDS_BYTES;
    *G_out = FUSED_G;
    return true;
}

bool vf_fused_ok(const vf_model *m, const Batch &b) {
    FusedArgs a;
    int G;
    return plan_fused(m, b, a, &G);
}

int vf_run_fused(vf_model *m, const Batch &b, const int32_t *tokens, float *logits_out, bool tree, hipStream_t st) {
    const vf_config &c = m->cfg;
    FusedArgs a;
    memset(&a, 0, sizeof a);
    int G = 0;
    if (!plan_fused(m, b, a, &G)) return vf_fail(VF_ERR_UNSUPPORTED, "persistent kernel does not apply to this call");
    int max_keys = 0;
    for (int i = 0; i < b.n_seqs; ++i) max_keys = std::max(max_keys, b.s[i].len_ub + b.s[i].nrows);
    // attention: blocks of 16 query items per (sequence, kv head); as many key parts per block as
    // fill the grid, but no more than give every wavefront of a part a tile of its own
    const int group = c.n_q_heads / c.n_kv_heads;
    int blocks = 0;
    for (int i = 0; i < b.n_seqs; ++i) blocks += c.n_kv_heads * ((b.s[i].nrows * group + 15) / 16);
    int parts = std::max(1, std::min(G / std::max(1, blocks), ((max_keys + FKT - 1) / FKT + FW - 1) / FW));
    parts = std::min(parts, FUSED_MAXP);
    if (blocks > VF_N_COUNTERS) return vf_fail(VF_ERR_UNSUPPORTED, "%d attention blocks", blocks);
    if (blocks * parts > FUSED_G) parts = 1;  // records have room for one per workgroup
    a.layers = (const FusedLayer *)m->fz_layers;
    a.embed = (const bf16_t *)m->embed;
    a.lm_head = (const u32x4 *)m->lm_head;
    a.final_norm = m->final_norm;
    a.cosv = m->rope_cos;
    a.sinv = m->rope_sin;
    a.tree_depth = tree ? m->tree_depth : nullptr;
    a.tree_anc = tree ? m->tree_anc : nullptr;
    a.tokens = tokens;
    a.hv = m->fz_h;
    a.ssv = m->fz_ss;
    a.qv = (bf16_t *)m->fz_q;
    a.ov = (bf16_t *)m->fz_o;
    a.av = (bf16_t *)m->fz_a;
    a.att_rec = m->fz_att;
    a.part = m->part;
    a.counters = m->counters;
    a.bar = m->fz_bar;
    a.fail = m->fz_bar + 8000;
    a.logits = logits_out;
    a.n_layers = c.n_layers;
    a.d = c.d_model;
    a.F = c.d_ffn;
    a.hq = c.n_q_heads;
    a.hkv = c.n_kv_heads;
    a.hd = c.head_dim;
    a.vocab = c.vocab;
    a.m = b.total_rows;
    a.att_blocks = blocks;
    a.att_parts = parts;
    {
        // item = part * blocks + block, block = (sequence, kv head, query block) in that order
        const int n_work = blocks * parts;
        for (int w = 0; w < FUSED_G; ++w) a.att_first[w] = (short)(w < n_work && n_work > G ? w : -1);
        if (n_work <= G) {
            // from the top of the grid downwards: the QKV phase before it keeps the lowest workgroups busy
            // (one item each), and a workgroup that is idle there has worked out its attention item and
            // requested its first key tile by the time the others arrive
            int next[8], die = 0;
            for (int x = 0; x < 8; ++x) next[x] = FUSED_ATT_TOP ? G - 8 + x : x;
            int blk0 = 0;
            for (int sq = 0; sq < b.n_seqs; ++sq) {
                const int nqb = (b.s[sq].nrows * group + 15) / 16;
                for (int kvh = 0; kvh < c.n_kv_heads; ++kvh)
                    for (int p = 0; p < parts; ++p) {
                        for (int qb = 0; qb < nqb; ++qb) {
                            int x = die;
                            for (int tries = 0; tries < 8 && (next[x] >= G || next[x] < 0); ++tries) x = (x + 1) % 8;  // that die is full
                            a.att_first[next[x]] = (short)(p * blocks + blk0 + kvh * nqb + qb);
                            next[x] += FUSED_ATT_TOP ? -8 : 8;
                        }
                        die = (die + 1) % 8;
                    }
                blk0 += c.n_kv_heads * nqb;
            }
        }
    }
    a.has_bias = c.qkv_bias;
    a.inv_d = 1.0f / (float)c.d_model;
    a.eps = c.rms_eps;
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)c.head_dim);
    a.root0 = m->fz_epoch;
    m->fz_epoch += (1u + 5u * (unsigned)c.n_layers) * (unsigned)(G / BAR_COUNTERS);  // barriers per launch x arrivals per counter
    const int rows = b.total_rows;
    {
        const bool fits = FUSED_WAVE_PHASES && (size_t)(c.d_model / 32) * rows * 64 + WAVE_TAIL_BYTES <= (size_t)LDS_BYTES &&
                          (size_t)c.d_model * 4 <= (size_t)WAVE_TAIL_BYTES;
        a.wave_gu = fits && a.ks_gu == 1;
        {
            // one unit for each workgroup of the O projection, if the others can take the rest in at most
            // three units each (two passes)
            const int n_o = (c.d_model / 16) * a.ks_o, units = c.d_ffn / 16, H = G - n_o;
            a.gu_light = (FUSED_GU_LIGHT && n_o > 0 && H > 0 && n_o < units && units - n_o <= 3 * H && units - n_o > H) ? n_o : 0;
        }
        a.wave_head = fits && a.ks_head == 1;
    }
    ProfScope ps(m, VF_SITE_STEP, st);
    if (c.head_dim == 128) {
        if (rows <= 16) return launch_fused<1, 128>(m, a, b, G, st);
        if (rows <= 32) return launch_fused<2, 128>(m, a, b, G, st);
        return launch_fused<3, 128>(m, a, b, G, st);
    }
    if (rows <= 16) return launch_fused<1, 64>(m, a, b, G, st);
    if (rows <= 32) return launch_fused<2, 64>(m, a, b, G, st);
    return launch_fused<3, 64>(m, a, b, G, st);
}

// Whether any barrier of an earlier launch gave up (the stream must be idle).
int vf_fused_check(vf_model *m) {
    if (!m->fz_bar) return VF_OK;
    unsigned flag = 0;
    VF_HIP(hipMemcpy(&flag, m->fz_bar + 8000, 4, hipMemcpyDeviceToHost));
    if (flag) {
        // counters are out of step now: start over from zero
        VF_HIP(hipMemset(m->fz_bar, 0, 65536));
        VF_HIP(hipMemset(m->counters, 0, VF_N_COUNTERS * 4));
        m->fz_epoch = 0;
        return vf_fail(VF_ERR_HIP, "persistent verify kernel: a grid barrier timed out; results of that call are invalid");
    }
    return VF_OK;
}

#ifdef FUSED_ARRIVALS
// Copies the arrival / release stamps of the last launch (logits left in the model workspace): [barrier][2][workgroup].
extern "C" int vf_debug_arrivals(vf_model *m, unsigned long long *out_host, int n_barriers) {
    VF_HIP(hipDeviceSynchronize());
    VF_HIP(hipMemcpy(out_host, m->logits + (size_t)64 * m->cfg.vocab, (size_t)n_barriers * 2 * FUSED_G * 8, hipMemcpyDeviceToHost));
    return VF_OK;
}
#endif

#ifdef FUSED_TRACE
// Copies the phase timeline of the traced workgroup's last launch: pairs (clock, mark id).
extern "C" int vf_debug_trace(vf_model *m, unsigned long long *out_host, int n_pairs) {
    VF_HIP(hipDeviceSynchronize());
    VF_HIP(hipMemcpy(out_host, m->fz_bar + 8192, (size_t)n_pairs * 16, hipMemcpyDeviceToHost));
    return VF_OK;
}
#endif
