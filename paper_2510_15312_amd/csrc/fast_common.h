// Device code shared by the few-row verify kernels (one kernel per GEMM) and the persistent
// whole-step kernel: GEMM descriptors and epilogues, and the MFMA attention building blocks
// (paper Sec. 3 / Sec. 4.3: the k+1 rows [T, x_1..x_k] of one verify step).
#pragma once

#include "vf_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct FastGemm {
    const u32x4 *W;   // packed fragments
    int N, KB;        // output features, K / 32
    const bf16_t *X;  // [m, K] row-major bfloat16 operand (EPI_RESID)
    const float *Xh;  // [m, K] float32 residual stream, normalised while staging (other epilogues)
    const float *gain;  // RMSNorm gain applied with Xh
    int m;
    int ks, kbps;     // K split across workgroups, k-blocks per split
    int kch;          // k-blocks staged in LDS at a time
    float *part;      // ks > 1: partial tiles
    int *counters;    // ks > 1: arrivals per unit
    const float *ss_in;  // per-16-column sums of squares of the rows of h, [n_ss][64]
    int n_ss;
    float inv_d, eps;
    // EPI_RESID: h_out = h_in + y (the two may be the same buffer)
    const float *h_in;
    float *h;
    float *ss_out;
    // EPI_SWIGLU
    bf16_t *a_out;
    int F;
    // EPI_LOGITS
    float *logits;
    // EPI_QKV
    const float *bias, *cosv, *sinv;
    bf16_t *q;
    int layer, hq, hkv, hd;
    const int32_t *depth;  // tree-structured drafts: depth of every row (NULL: row r of a sequence has depth r)
};

__device__ inline u32x4 load_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// Stores that other workgroups read later in the same launch go through to memory (agent scope);
// COH = false is an ordinary store for data only a later kernel reads.
template <bool COH> __device__ inline void st_u16(void *p, unsigned short v) {
    if (COH) __hip_atomic_store(reinterpret_cast<unsigned short *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *reinterpret_cast<unsigned short *>(p) = v;
}
template <bool COH> __device__ inline void st_u32(void *p, unsigned v) {
    if (COH) __hip_atomic_store(reinterpret_cast<unsigned *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *reinterpret_cast<unsigned *>(p) = v;
}
template <bool COH> __device__ inline void st_f32(float *p, float v) {
    if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
template <bool COH> __device__ inline void st_u32x2(void *p, u32x2 v) {
    if (COH)
        __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *reinterpret_cast<u32x2 *>(p) = v;
}
#ifndef VF_STORE16_WT
#define VF_STORE16_WT 1   // 16-byte write-through stores as one instruction (0: two 8-byte atomic stores)
#endif
template <bool COH> __device__ inline void st_f32x4(float *p, floatx4 v) {
    if (COH) {
#if VF_STORE16_WT
        // one 16-byte store with the agent-scope (write-through) cache policy: what the 8-byte atomic
        // stores compile to, at twice the width.  Readers never depend on the 16 bytes arriving together.
        // A store of more than 8 bytes reads its data registers for some cycles after it has issued, and
        // the compiler, which keeps the next instruction from overwriting them after its own stores, does
        // not look inside this statement: the two idle cycles the hardware asks for are part of it.
        typedef float __attribute__((address_space(1))) *global_f32_ptr;
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"((global_f32_ptr)p), "v"(v) : "memory");
#else
        const u32x4 r = __builtin_bit_cast(u32x4, v);
        st_u32x2<true>(p, u32x2{r[0], r[1]});
        st_u32x2<true>(p + 2, u32x2{r[2], r[3]});
#endif
    } else {
        *reinterpret_cast<floatx4 *>(p) = v;
    }
}
__device__ inline void store_coherent(float *p, floatx4 v) { st_f32x4<true>(p, v); }
// Waits until every store this wavefront has issued has completed at its scope.  A workgroup-scope
// release fence does not: within a workgroup the memory pipeline keeps stores in order, so the
// compiler emits no wait for it, and a signal to ANOTHER workgroup (a counter increment) could
// then overtake the write-through stores it is meant to publish.
__device__ inline void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
#ifndef VF_COH_LOAD_SCOPE
#define VF_COH_LOAD_SCOPE __HIP_MEMORY_SCOPE_AGENT
#endif
__device__ inline floatx4 load_coherent(const float *p) {
    const unsigned long long *q = reinterpret_cast<const unsigned long long *>(p);
    const unsigned long long a = __hip_atomic_load(q, __ATOMIC_RELAXED, VF_COH_LOAD_SCOPE);
    const unsigned long long b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, VF_COH_LOAD_SCOPE);
    const u32x2 lo = __builtin_bit_cast(u32x2, a), hi = __builtin_bit_cast(u32x2, b);
    return __builtin_bit_cast(floatx4, u32x4{lo[0], lo[1], hi[0], hi[1]});
}
__device__ inline u32x4 load_coherent16(const void *p) {
    return __builtin_bit_cast(u32x4, load_coherent(reinterpret_cast<const float *>(p)));
}
__device__ inline float load_coherent1(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, VF_COH_LOAD_SCOPE);
}

__device__ inline u32x2 pack4_bf16(float a, float b, float c, float d) {
    bf16x4 v = {(bf16_t)a, (bf16_t)b, (bf16_t)c, (bf16_t)d};
    return __builtin_bit_cast(u32x2, v);
}
__device__ inline unsigned pack2_bf16(float a, float b) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = {(bf16_t)a, (bf16_t)b};
    return __builtin_bit_cast(unsigned, v);
}

// ---- epilogues: thread holds Y[row][n0 .. n0+3] ------------------------------------------------

template <bool COH>
__device__ inline void epi_resid(const FastGemm &g, int row, bool live, int nb, int lane, floatx4 v) {
    const int n0 = nb * 16 + (lane >> 4) * 4;
    floatx4 hv = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        const float *hp = g.h_in + (size_t)row * g.N + n0;
        hv = *reinterpret_cast<const floatx4 *>(hp) + v;  // a buffer other workgroups wrote in an earlier phase, never rewritten
        st_f32x4<COH>(g.h + (size_t)row * g.N + n0, hv);
    }
    float ssq = hv[0] * hv[0] + hv[1] * hv[1] + hv[2] * hv[2] + hv[3] * hv[3];
    ssq += __shfl_xor(ssq, 16, 64);
    ssq += __shfl_xor(ssq, 32, 64);
    if (live && (lane >> 4) == 0) st_f32<COH>(g.ss_out + nb * 64 + row, ssq);
}

template <bool COH>
__device__ inline void epi_qkv(const FastGemm &g, const Batch &b, int row, int nb, int lane, floatx4 v) {
    const int n0 = nb * 16 + (lane >> 4) * 4;
    const int hd = g.hd, half = hd >> 1;
    if (g.bias)
        for (int i = 0; i < 4; ++i) v[i] += g.bias[n0 + i];
    const SeqDesc &s = b.s[find_seq(b, row)];
    // slot: the cache row the call's row is written to; pos: the position whose rotary angle it
    // takes (its depth below the pending token when the drafts form a tree)
    const int slot = s.state[0] + (row - s.row0);
    const int pos = g.depth ? s.state[0] + g.depth[row] : slot;
    if (slot < 0 || slot >= s.capacity) return;
    const int head = n0 / hd, p0 = n0 % hd;
    bf16_t *kv = reinterpret_cast<bf16_t *>(s.kv);
    if (head < g.hq + g.hkv) {
        const int i0 = p0 >> 1;  // packed columns 2i, 2i+1 are elements i and i + hd/2
        const float c0 = g.cosv[(size_t)pos * half + i0], s0 = g.sinv[(size_t)pos * half + i0];
        const float c1 = g.cosv[(size_t)pos * half + i0 + 1], s1 = g.sinv[(size_t)pos * half + i0 + 1];
        const float a0 = v[0] * c0 - v[1] * s0, b0 = v[1] * c0 + v[0] * s0;
        const float a1 = v[2] * c1 - v[3] * s1, b1 = v[3] * c1 + v[2] * s1;
        // i0 is even: elements i0, i0 + 1 are neighbours in either layout, 4-byte aligned
        bf16_t *d0, *d1;
        if (head < g.hq) {
            d0 = g.q + ((size_t)row * g.hq + head) * hd + i0;
            d1 = d0 + half;
        } else {
            const int page = kv_page(s, slot), tin = slot % VF_TILE;
            d0 = kv + kv_k_index(g.layer, s.n_pages, page, g.hkv, head - g.hq, tin, i0, hd);
            d1 = kv + kv_k_index(g.layer, s.n_pages, page, g.hkv, head - g.hq, tin, i0 + half, hd);
        }
        st_u32<COH>(d0, pack2_bf16(a0, a1));
        st_u32<COH>(d1, pack2_bf16(b0, b1));
    } else {
        const int vh = head - g.hq - g.hkv;
        const int page = kv_page(s, slot), tin = slot % VF_TILE;
        for (int i = 0; i < 4; ++i) {
            const bf16_t x = (bf16_t)v[i];
            st_u16<COH>(kv + kv_v_index(g.layer, s.n_pages, page, g.hkv, vh, tin, p0 + i, hd),
                        __builtin_bit_cast(unsigned short, x));
        }
    }
}

template <bool COH>
__device__ inline void epi_swiglu(const FastGemm &g, int row, int nb_gate, int lane, floatx4 vg, floatx4 vu) {
    const int f0 = (nb_gate >> 1) * 16 + (lane >> 4) * 4;
    float o[4];
    for (int i = 0; i < 4; ++i) {
        const float gt = vg[i], up = vu[i];
        o[i] = gt / (1.0f + expf(-gt)) * up;
    }
    st_u32x2<COH>(g.a_out + (size_t)row * g.F + f0, pack4_bf16(o[0], o[1], o[2], o[3]));
}

// ---- attention ----------------------------------------------------------------------------------
constexpr int ATTF_STRIDE_PAD = 4;  // partial record: [max, sum, -, -, O[hd]]

// One key slice of ATT_KEYS keys of one kv head is first copied into LDS (every load in flight at
// once: one memory round trip).  Query items (row, head in group) are tiled 16 per MFMA column
// block.  Scores S^T[key, item] = K * Q^T leave the MFMA with four consecutive keys per lane and
// one item per lane column, which is already the B-operand layout of
// O^T[d, item] += V^T[d, key] * P[key, item] when the V^T fragment is read with the same key
// order; the softmax statistics of an item live in the four lanes l, l+16, l+32, l+48 and are
// merged with two shuffles.
constexpr int ATT_KEYS = 128;

template <int HD> struct AttLds {
    static constexpr int KROW = HD + 8, VROW = ATT_KEYS + 8;  // padded rows: conflict-free fragment reads
    bf16_t Ks[ATT_KEYS * KROW];
    bf16_t Vs[HD * VROW];
};

// Copy of keys [k_begin, k_begin + 128) of one kv head into LDS: K as [key][d], V^T as [d][key];
// keys at or past kmax read as zero.  THREADS threads take part; load() issues every global load,
// store() writes them to LDS, so other work can sit between the two.
template <int HD, int THREADS> struct AttStage {
    static constexpr int KROW = AttLds<HD>::KROW, VROW = AttLds<HD>::VROW;
    static constexpr int KP = HD / 8;                   // 16-byte pieces per key row
    static constexpr int NK = ATT_KEYS * KP / THREADS;  // pieces per thread
    u32x4 kreg[NK], vreg[NK];

    __device__ inline void load(const SeqDesc &s, int layer, int hkv, int kvh, int k_begin, int kmax, int tid) {
        const bf16_t *kv = reinterpret_cast<const bf16_t *>(s.kv);
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            const int pidx = i * THREADS + tid, key = pidx / KP, piece = pidx % KP, t = k_begin + key;
            kreg[i] = zero4;
            if (t < kmax)
                kreg[i] = *reinterpret_cast<const u32x4 *>(
                    kv + kv_k_index(layer, s.n_pages, kv_page(s, t), hkv, kvh, t % VF_TILE, piece * 8, HD));
        }
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            // V^T tiles: per 64-key page [d][64]; piece = 8 consecutive keys of one d
            const int pidx = i * THREADS + tid, d = pidx / (ATT_KEYS / 8), piece = pidx % (ATT_KEYS / 8);
            const int t = k_begin + piece * 8;
            vreg[i] = zero4;
            if (t < kmax)
                vreg[i] = *reinterpret_cast<const u32x4 *>(
                    kv + kv_v_index(layer, s.n_pages, kv_page(s, t), hkv, kvh, t % VF_TILE, d, HD));
        }
    }
    __device__ inline void store(AttLds<HD> &L, int k_begin, int kmax, int tid) const {
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            const int pidx = i * THREADS + tid, key = pidx / KP, piece = pidx % KP;
            *reinterpret_cast<u32x4 *>(L.Ks + key * KROW + piece * 8) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            const int pidx = i * THREADS + tid, d = pidx / (ATT_KEYS / 8), piece = pidx % (ATT_KEYS / 8);
            const int t = k_begin + piece * 8;
            bf16x8 v = __builtin_bit_cast(bf16x8, vreg[i]);
            if (t + 8 > kmax) {  // cache rows past the last key may hold anything: zero them
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (t + j >= kmax) v[j] = (bf16_t)0.f;
            }
            *reinterpret_cast<bf16x8 *>(L.Vs + d * VROW + piece * 8) = v;
        }
    }
};

// Copies keys [k_begin, k_begin + 128) of one kv head into LDS: K as [key][d], V^T as [d][key];
// keys at or past kmax read as zero.  256 threads; every load is issued before the first store.
template <int HD>
__device__ inline void att_stage(const SeqDesc &s, int layer, int hkv, int kvh, int k_begin, int kmax,
                                 AttLds<HD> &L, int tid) {
    constexpr int KROW = AttLds<HD>::KROW, VROW = AttLds<HD>::VROW;
    constexpr int KP = HD / 8;               // 16-byte pieces per key row
    constexpr int NK = ATT_KEYS * KP / 256;  // pieces per thread
    const bf16_t *kv = reinterpret_cast<const bf16_t *>(s.kv);
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    u32x4 kreg[NK], vreg[NK];
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        const int pidx = i * 256 + tid, key = pidx / KP, piece = pidx % KP, t = k_begin + key;
        kreg[i] = zero4;
        if (t < kmax)
            kreg[i] = *reinterpret_cast<const u32x4 *>(
                kv + kv_k_index(layer, s.n_pages, kv_page(s, t), hkv, kvh, t % VF_TILE, piece * 8, HD));
    }
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        // V^T tiles: per 64-key page [d][64]; piece = 8 consecutive keys of one d
        const int pidx = i * 256 + tid, d = pidx / (ATT_KEYS / 8), piece = pidx % (ATT_KEYS / 8);
        const int t = k_begin + piece * 8;
        vreg[i] = zero4;
        if (t < kmax)
            vreg[i] = *reinterpret_cast<const u32x4 *>(
                kv + kv_v_index(layer, s.n_pages, kv_page(s, t), hkv, kvh, t % VF_TILE, d, HD));
    }
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        const int pidx = i * 256 + tid, key = pidx / KP, piece = pidx % KP;
        *reinterpret_cast<u32x4 *>(L.Ks + key * KROW + piece * 8) = kreg[i];
    }
#pragma unroll
    for (int i = 0; i < NK; ++i) {
        const int pidx = i * 256 + tid, d = pidx / (ATT_KEYS / 8), piece = pidx % (ATT_KEYS / 8);
        const int t = k_begin + piece * 8;
        bf16x8 v = __builtin_bit_cast(bf16x8, vreg[i]);
        if (t + 8 > kmax) {  // cache rows past the last key may hold anything: zero them
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (t + j >= kmax) v[j] = (bf16_t)0.f;
        }
        *reinterpret_cast<bf16x8 *>(L.Vs + d * VROW + piece * 8) = v;
    }
}

// Online-softmax state of one block of 16 query items in one wavefront.
template <int HD> struct AttState {
    floatx4 o[HD / 16];
    float m_run, l_run;
};

// One staged slice for one block of 16 items: S^T = K Q^T, masked online softmax, O^T += V^T P.
// last_key: last visible key of this lane's item; blk_last: of any item in the block.
template <int HD>
__device__ inline void att_slice(AttState<HD> &st, const bf16x8 (&qf)[HD / 32], const AttLds<HD> &L, int k_begin,
                                 int last_key, int blk_last, float scale_log2e, int lane) {
    constexpr int KD = HD / 32, DB = HD / 16, KROW = AttLds<HD>::KROW, VROW = AttLds<HD>::VROW;
    const int g4 = lane >> 4, l15 = lane & 15;
#pragma unroll 1
    for (int tl = 0; tl < ATT_KEYS; tl += 32) {
        const int t0 = k_begin + tl;
        if (t0 > blk_last) break;
        floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kd = 0; kd < KD; ++kd) {
            const bf16x8 k0 = *reinterpret_cast<const bf16x8 *>(L.Ks + (tl + l15) * KROW + kd * 32 + g4 * 8);
            const bf16x8 k1 = *reinterpret_cast<const bf16x8 *>(L.Ks + (tl + 16 + l15) * KROW + kd * 32 + g4 * 8);
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[kd], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[kd], s1, 0, 0, 0);
        }
        // lane holds keys t0 + 4*g4 + j (s0) and t0 + 16 + 4*g4 + j (s1) of item l15
        float tmax = -1e30f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s0[j] = (t0 + g4 * 4 + j <= last_key) ? s0[j] * scale_log2e : -1e30f;
            s1[j] = (t0 + 16 + g4 * 4 + j <= last_key) ? s1[j] * scale_log2e : -1e30f;
            tmax = fmaxf(tmax, fmaxf(s0[j], s1[j]));
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
        const float m_new = fmaxf(st.m_run, tmax);
        const float corr = exp2f(st.m_run - m_new);
        float p[8], psum = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            p[j] = (t0 + g4 * 4 + j <= last_key) ? exp2f(s0[j] - m_new) : 0.f;
            p[4 + j] = (t0 + 16 + g4 * 4 + j <= last_key) ? exp2f(s1[j] - m_new) : 0.f;
            psum += p[j] + p[4 + j];
        }
        psum += __shfl_xor(psum, 16, 64);
        psum += __shfl_xor(psum, 32, 64);
        st.l_run = st.l_run * corr + psum;
        st.m_run = m_new;
        // probabilities as a sum of two bfloat16 values (16 significant bits): the P * V product
        // then carries no more rounding than its bfloat16 V operand
        bf16x8 pf, pl;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            pf[j] = (bf16_t)p[j];
            pl[j] = (bf16_t)(p[j] - (float)pf[j]);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const bf16_t *vr = L.Vs + (db * 16 + l15) * VROW + tl + g4 * 4;
            const u32x2 lo = *reinterpret_cast<const u32x2 *>(vr);
            const u32x2 hi = *reinterpret_cast<const u32x2 *>(vr + 16);
            const u32x4 raw = {lo[0], lo[1], hi[0], hi[1]};
            const bf16x8 vf = __builtin_bit_cast(bf16x8, raw);
            st.o[db] = st.o[db] * corr;
            st.o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf, st.o[db], 0, 0, 0);
            st.o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pl, st.o[db], 0, 0, 0);
        }
    }
}


// ---- register-fed attention tiles -----------------------------------------------------------------
// A tile is 32 keys of one kv head.  K rows are fed to the first MFMA in the order
// 8*(rho >> 2) + (rho & 3) (+ 4 for the second 16-key block), which makes the score tile
// S^T[key, item] = K Q^T come out with eight consecutive keys per lane: the B-operand layout of
// O^T[d, item] += V^T[d, key] P[key, item]; the matching V^T fragment is one 16-byte load.
constexpr int ATT_TILE = 32;

template <int HD> struct AttTile {
    bf16x8 kf[2][HD / 32], vf[HD / 16];
    // coh: the tile holds keys written during this launch by other workgroups
    __device__ __forceinline__ void load(const SeqDesc &s, int layer, int hkv, int kvh, int t, bool coh, int lane) {
        // one branch, two straight-line copies: every load of a copy is issued before any is waited for
        if (coh) load_as<true>(s, layer, hkv, kvh, t, lane);
        else load_as<false>(s, layer, hkv, kvh, t, lane);
    }
    template <bool coh>
    __device__ __forceinline__ void load_as(const SeqDesc &s, int layer, int hkv, int kvh, int t, int lane) {
        load_page<coh>(s, layer, hkv, kvh, t, kv_page(s, t * ATT_TILE), lane);
    }
    // page: the cache page of tile t, for a caller that has looked it up already
    template <bool coh>
    __device__ __forceinline__ void load_page(const SeqDesc &s, int layer, int hkv, int kvh, int t, int page, int lane) {
        // the cache keeps a tile's fragments in operand order: fragment f of the tile is the kilobyte at
        // 512 * f elements, a lane's share the 16 bytes at 8 * lane
        const bf16_t *kv = reinterpret_cast<const bf16_t *>(s.kv);
        const int t0 = t * ATT_TILE, tin = t0 % VF_TILE;
        const bf16_t *kb = kv + kv_k_index(layer, s.n_pages, page, hkv, kvh, tin, 0, HD) + lane * 8;
        const bf16_t *vb = kv + kv_v_index(layer, s.n_pages, page, hkv, kvh, tin, 0, HD) + lane * 8;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int kd = 0; kd < HD / 32; ++kd) {
                const bf16_t *kp = kb + (h * (HD / 32) + kd) * 512;
                kf[h][kd] = coh ? __builtin_bit_cast(bf16x8, load_coherent16(kp)) : *reinterpret_cast<const bf16x8 *>(kp);
            }
#pragma unroll
        for (int db = 0; db < HD / 16; ++db) {
            const bf16_t *vp = vb + db * 512;
            vf[db] = coh ? __builtin_bit_cast(bf16x8, load_coherent16(vp)) : *reinterpret_cast<const bf16x8 *>(vp);
        }
    }
    // rows of the cache at or past kmax may hold anything: keep them out of the P V product
    __device__ __forceinline__ void mask_values(int t0, int kmax, int lane) {
        if (t0 + ATT_TILE > kmax) {
            const int g4 = lane >> 4;
#pragma unroll
            for (int db = 0; db < HD / 16; ++db)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (t0 + g4 * 8 + j >= kmax) vf[db][j] = (bf16_t)0.f;
        }
    }
};

// One tile for one block of 16 query items: masked online softmax update of st.
// last_key: last visible key of this lane's item (-1: none).  Tree-structured drafts: of the keys
// from own_base on (the rows of the same call) only those whose bit is set in own_mask are
// visible; a plain causal call passes ATT_NO_TREE as own_base.
constexpr int ATT_NO_TREE = 0x7fffffff;
template <int HD>
__device__ __forceinline__ void att_tile_update(AttState<HD> &st, const bf16x8 (&qf)[HD / 32], const AttTile<HD> &T, int t0,
                                                int last_key, int own_base, tree_mask_t own_mask,
                                                float scale_log2e, int lane) {
    constexpr int KD = HD / 32, DB = HD / 16;
    const int g4 = lane >> 4;
    floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kd = 0; kd < KD; ++kd) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(T.kf[0][kd], qf[kd], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(T.kf[1][kd], qf[kd], s1, 0, 0, 0);
    }
    // lane holds keys t0 + 8*g4 + j (s0) and t0 + 8*g4 + 4 + j (s1) of item (lane & 15)
    float p[8], tmax = -1e30f;
    bool vis[8];
    if (own_base == ATT_NO_TREE) {  // the same for every lane: a scalar branch, the causal test alone
#pragma unroll
        for (int j = 0; j < 8; ++j) vis[j] = t0 + g4 * 8 + j <= last_key;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int key = t0 + g4 * 8 + j;
            vis[j] = key <= last_key && (key < own_base || ((own_mask >> ((unsigned)(key - own_base) & 63u)) & 1));
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        p[j] = vis[j] ? s0[j] * scale_log2e : -1e30f;
        p[4 + j] = vis[4 + j] ? s1[j] * scale_log2e : -1e30f;
        tmax = fmaxf(tmax, fmaxf(p[j], p[4 + j]));
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(st.m_run, tmax);
    const float corr = exp2f(st.m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        p[j] = vis[j] ? exp2f(p[j] - m_new) : 0.f;
        psum += p[j];
    }
    psum += __shfl_xor(psum, 16, 64);
    psum += __shfl_xor(psum, 32, 64);
    st.l_run = st.l_run * corr + psum;
    st.m_run = m_new;
    // probabilities as a sum of two bfloat16 values (16 significant bits): the P * V product
    // then carries no more rounding than its bfloat16 V operand
    bf16x8 pf, pl;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        pf[j] = (bf16_t)p[j];
        pl[j] = (bf16_t)(p[j] - (float)pf[j]);
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        st.o[db] = st.o[db] * corr;
        st.o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(T.vf[db], pf, st.o[db], 0, 0, 0);
        st.o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(T.vf[db], pl, st.o[db], 0, 0, 0);
    }
}

}  // namespace
