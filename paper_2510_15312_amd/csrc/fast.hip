// The verify hot path for few rows (pending token + drafts, paper Sec. 3 / Sec. 4.3), bfloat16.
//
// Per decoder layer four fused GEMM kernels, attention and its merge:
//   QKV     : x * Wqkv^T          -> row scale, bias, rotary embedding, q and KV-cache append
//   attn    : split-KV causal attention of all rows over the cache (MFMA), then the merge
//   O       : o * Wo^T            -> residual add, next norm's input and sums of squares
//   gate/up : x * [Wg|Wu]^T       -> row scale, SwiGLU
//   down    : a * Wd^T            -> residual add, next norm's input and sums of squares
// and the output head  x * E^T -> row scale -> float32 logits.
//
// RMSNorm is fused into the GEMM that consumes it: the producer of the residual stream h also
// writes per-16-column sums of h^2; the consumer turns them into rstd = rsqrt(mean(h^2) + eps)
// per row and builds its bfloat16 operand x = bf16(h * rstd * gain) while staging h in LDS.
//
// GEMM kernel: one workgroup per unit of UB weight blocks (16 rows each); its wavefronts split
// the K range, stream their weight fragments from HBM straight into registers (1 KiB per
// wavefront load, read once, non-temporal) and take the activations from LDS.  Wavefront
// partial sums are added in LDS in a fixed order.  With a K split across workgroups (ks > 1)
// each workgroup leaves its partial tile in memory and the last one to arrive adds them in split
// order, so results do not depend on timing.
#include "fast_common.h"

namespace {

// NB: 16-row activation blocks (rows <= 16*NB); UB: weight blocks per unit; PD: fragments in flight
// per weight stream and wavefront; NW: wavefronts per workgroup.
template <int NB, int UB, int PD, int EPI, int NW>
__global__ __launch_bounds__(NW * 64) VF_MFMA_KERNEL void gemm_fast_kernel(FastGemm g, Batch b) {
    constexpr int FAST_THREADS = NW * 64, FAST_WAVES = NW;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    u32x4 *xs = reinterpret_cast<u32x4 *>(smem_raw);
    floatx4 *red = reinterpret_cast<floatx4 *>(smem_raw);
    __shared__ float rs_s[64];
    __shared__ float rs_tmp[FAST_WAVES][64];
    __shared__ int s_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = g.m, KB = g.KB, NBt = g.N >> 4;
    const int unit = blockIdx.x, split = blockIdx.y;
    const int nb0 = unit * UB;
    const int kb0 = split * g.kbps, kb1 = min(KB, kb0 + g.kbps);

    floatx4 acc[UB][NB];
#pragma unroll
    for (int u = 0; u < UB; ++u)
#pragma unroll
        for (int c = 0; c < NB; ++c) acc[u][c] = floatx4{0.f, 0.f, 0.f, 0.f};
    const u32x4 *wp[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) wp[u] = g.W + (size_t)min(nb0 + u, NBt - 1) * KB * 64 + lane;
    int rowc[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) rowc[c] = min(c * 16 + (lane & 15), m - 1);

    // Loads go out in the order: row statistics (needed first), weights, activations.
    constexpr bool NORMED = EPI != EPI_RESID;
    float rs_t[16];
    if (NORMED) {
        // lane = row, wavefront = every NW-th block of 16 columns (first 16 * NW blocks)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int j = wave + i * FAST_WAVES;
            rs_t[i] = (lane < m && j < g.n_ss) ? g.ss_in[j * 64 + lane] : 0.f;
        }
    }

    for (int kc0 = kb0; kc0 < kb1; kc0 += g.kch) {
        const int kc1 = min(kb1, kc0 + g.kch), nk = kc1 - kc0;
        const int wk0 = kc0 + nk * wave / FAST_WAVES, wk1 = kc0 + nk * (wave + 1) / FAST_WAVES, nw = wk1 - wk0;
        u32x4 w[PD][UB];
#pragma unroll
        for (int d = 0; d < PD; ++d)
            if (d < nw)
#pragma unroll
                for (int u = 0; u < UB; ++u) w[d][u] = load_stream(wp[u] + (size_t)(wk0 + d) * 64);
        if (NORMED && kc0 == kb0) {
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += rs_t[i];
            if (lane < m)
                for (int j = wave + 16 * FAST_WAVES; j < g.n_ss; j += FAST_WAVES) sum += g.ss_in[j * 64 + lane];
            rs_tmp[wave][lane] = sum;
            __syncthreads();
            if (tid < 64) {
                float tot = 0.f;
                for (int j = 0; j < FAST_WAVES; ++j) tot += rs_tmp[j][tid];
                rs_s[tid] = 1.0f / sqrtf(tot * g.inv_d + g.eps);
            }
        }
        __syncthreads();  // previous chunk consumed; row scales visible
        if (NORMED) {
            // x = bf16(h * rstd * gain): pieces of four columns
            const int chunks = nk * 8, pieces = m * chunks;
            for (int base = tid; base < pieces; base += FAST_THREADS * 4) {
                floatx4 v[4], gn[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = base + i * FAST_THREADS;
                    if (idx < pieces) {
                        const int row = idx / chunks, c = idx % chunks;
                        v[i] = *reinterpret_cast<const floatx4 *>(g.Xh + (size_t)row * KB * 32 + (size_t)kc0 * 32 + c * 4);
                        gn[i] = *reinterpret_cast<const floatx4 *>(g.gain + (size_t)kc0 * 32 + c * 4);
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = base + i * FAST_THREADS;
                    if (idx < pieces) {
                        const int row = idx / chunks, c = idx % chunks;
                        const float r = rs_s[row];
                        u32x2 *dst = reinterpret_cast<u32x2 *>(xs) + (((c >> 3) * m + row) * 8 + (c & 7));
                        *dst = pack4_bf16(v[i][0] * r * gn[i][0], v[i][1] * r * gn[i][1], v[i][2] * r * gn[i][2],
                                          v[i][3] * r * gn[i][3]);
                    }
                }
            }
        } else {
            const int chunks = nk * 4, pieces = m * chunks;
            for (int base = tid; base < pieces; base += FAST_THREADS * 4) {
                u32x4 v[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = base + i * FAST_THREADS;
                    if (idx < pieces) {
                        const int row = idx / chunks, c = idx % chunks;
                        v[i] = *reinterpret_cast<const u32x4 *>(g.X + (size_t)row * KB * 32 + (size_t)kc0 * 32 + c * 8);
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = base + i * FAST_THREADS;
                    if (idx < pieces) {
                        const int row = idx / chunks, c = idx % chunks;
                        xs[((c >> 2) * m + row) * 4 + (c & 3)] = v[i];
                    }
                }
            }
        }
        __syncthreads();
#pragma unroll 1
        for (int k0 = 0; k0 < nw; k0 += PD) {
#pragma unroll
            for (int d = 0; d < PD; ++d) {
                const int kbl = k0 + d;
                if (kbl < nw) {
                    bf16x8 a[UB];
#pragma unroll
                    for (int u = 0; u < UB; ++u) a[u] = __builtin_bit_cast(bf16x8, w[d][u]);
                    if (kbl + PD < nw)
#pragma unroll
                        for (int u = 0; u < UB; ++u) w[d][u] = load_stream(wp[u] + (size_t)(wk0 + kbl + PD) * 64);
                    const int kx = wk0 + kbl - kc0;
#pragma unroll
                    for (int c = 0; c < NB; ++c) {
                        const bf16x8 bb = __builtin_bit_cast(bf16x8, xs[(kx * m + rowc[c]) * 4 + (lane >> 4)]);
#pragma unroll
                        for (int u = 0; u < UB; ++u)
                            acc[u][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], bb, acc[u][c], 0, 0, 0);
                    }
                }
            }
        }
    }
    __syncthreads();  // activations no longer needed: the same LDS now takes the wavefront partials
#pragma unroll
    for (int u = 0; u < UB; ++u)
#pragma unroll
        for (int c = 0; c < NB; ++c) red[((wave * UB + u) * NB + c) * 64 + lane] = acc[u][c];
    __syncthreads();

    constexpr int NT = UB * NB * 64;                           // tiles of 4 outputs per unit
    constexpr int NTH = EPI == EPI_SWIGLU ? NB * 64 : NT;      // tiles with an epilogue of their own
    constexpr int TPT = (NTH + FAST_THREADS - 1) / FAST_THREADS;  // tiles per thread
    floatx4 v0[TPT], v1[TPT];
#pragma unroll
    for (int it = 0; it < TPT; ++it) {
        const int t = tid + it * FAST_THREADS;
        v0[it] = floatx4{0.f, 0.f, 0.f, 0.f};
        v1[it] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (t < NTH) {
            if (EPI == EPI_SWIGLU) {
                const int c = t >> 6;
                for (int w = 0; w < FAST_WAVES; ++w) {
                    v0[it] += red[((w * UB + 0) * NB + c) * 64 + lane];
                    v1[it] += red[((w * UB + 1) * NB + c) * 64 + lane];
                }
            } else {
                const int u = t / (NB * 64), c = (t >> 6) % NB;
                for (int w = 0; w < FAST_WAVES; ++w) v0[it] += red[((w * UB + u) * NB + c) * 64 + lane];
            }
        }
    }
    if (g.ks > 1) {
        float *mine = g.part + ((size_t)(unit * g.ks + split) * NT) * 4;
#pragma unroll
        for (int it = 0; it < TPT; ++it) {
            const int t = tid + it * FAST_THREADS;
            if (t < NTH) {
                store_coherent(mine + (size_t)t * 4, v0[it]);
                if (EPI == EPI_SWIGLU) store_coherent(mine + (size_t)(NTH + t) * 4, v1[it]);
            }
        }
        stores_done();
        __syncthreads();
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(g.counters + unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == g.ks - 1;
            if (s_last) __hip_atomic_store(g.counters + unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!s_last) return;
#pragma unroll
        for (int it = 0; it < TPT; ++it) {
            const int t = tid + it * FAST_THREADS;
            v0[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            v1[it] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (t < NTH) {
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
                        v0[it] += t0[i];
                        v1[it] += t1[i];
                    }
                }
            }
        }
    }
#pragma unroll
    for (int it = 0; it < TPT; ++it) {
        const int t = tid + it * FAST_THREADS;
        if (t >= NTH) break;  // whole wavefronts leave together: NTH is a multiple of 64
        const int u = EPI == EPI_SWIGLU ? 0 : t / (NB * 64), c = (t >> 6) % NB;
        const int nb = nb0 + u;
        const int row = c * 16 + (lane & 15);
        const bool live = row < m && nb < NBt;
        if (EPI == EPI_RESID) {
            epi_resid<false>(g, row, live, nb, lane, v0[it]);
        } else if (live) {
            if (EPI == EPI_QKV) epi_qkv<false>(g, b, row, nb, lane, v0[it]);
            else if (EPI == EPI_SWIGLU) epi_swiglu<false>(g, row, nb, lane, v0[it], v1[it]);
            else *reinterpret_cast<floatx4 *>(g.logits + (size_t)row * g.N + nb * 16 + (lane >> 4) * 4) = v0[it];
        }
    }
}

// ---- embedding ----------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void embed_fast_kernel(const bf16_t *__restrict__ E, const int32_t *__restrict__ tokens,
                                                         Batch b, float *__restrict__ h, float *__restrict__ ss,
                                                         int d, int vocab) {
    const int row = blockIdx.x;
    int tok = tokens[row];
    if (tok == VF_PENDING) tok = b.s[find_seq(b, row)].state[1];
    if (tok < 0 || tok >= vocab) tok = 0;
    for (int k0 = 0; k0 < d; k0 += 256) {
        const int k = k0 + threadIdx.x;
        float v = 0.f;
        if (k < d) {
            v = (float)E[wfrag_index(tok, k, d)];
            h[(size_t)row * d + k] = v;
        }
        float sq = v * v;
        sq += __shfl_xor(sq, 8, 64);
        sq += __shfl_xor(sq, 4, 64);
        sq += __shfl_xor(sq, 2, 64);
        sq += __shfl_xor(sq, 1, 64);
        if (k < d && (threadIdx.x & 15) == 0) ss[(k >> 4) * 64 + row] = sq;
    }
}

// ---- attention ----------------------------------------------------------------------------------
// Few rows: one workgroup per (key slice, kv head, sequence); partial results per slice.
template <int HD>
__global__ __launch_bounds__(256) VF_MFMA_KERNEL void attn_fast_kernel(Batch b, int layer, const bf16_t *__restrict__ q,
                                                        float *__restrict__ part, int hq, int hkv, int n_splits,
                                                        float scale_log2e) {
    constexpr int KD = HD / 32, DB = HD / 16, REC = HD + ATTF_STRIDE_PAD;
    __shared__ __align__(16) AttLds<HD> L;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g4 = lane >> 4, l15 = lane & 15;
    const int split = blockIdx.x, kvh = blockIdx.y;
    const SeqDesc &s = b.s[blockIdx.z];
    const int group = hq / hkv, n_items = s.nrows * group;
    const int len = s.state[0];
    const int kmax = min(len + s.nrows, s.capacity);  // keys 0..kmax-1 exist
    const int k_begin = split * ATT_KEYS;
    if (k_begin >= kmax) return;
    att_stage<HD>(s, layer, hkv, kvh, k_begin, kmax, L, tid);
    __syncthreads();
    const int nqb = (n_items + 15) >> 4;
    for (int qb = wave; qb < nqb; qb += 4) {
        const int item = qb * 16 + l15;
        const bool valid = item < n_items;
        const int r = valid ? item / group : 0, head = kvh * group + (valid ? item % group : 0);
        const int row = s.row0 + r;
        const int last_key = valid ? len + r : -1;
        const int blk_last = len + min(s.nrows - 1, (qb * 16 + 15) / group);
        bf16x8 qf[KD];
#pragma unroll
        for (int kd = 0; kd < KD; ++kd)
            qf[kd] = *reinterpret_cast<const bf16x8 *>(q + ((size_t)row * hq + head) * HD + kd * 32 + g4 * 8);
        AttState<HD> st;
#pragma unroll
        for (int db = 0; db < DB; ++db) st.o[db] = floatx4{0.f, 0.f, 0.f, 0.f};
        st.m_run = -1e30f;
        st.l_run = 0.f;
        att_slice<HD>(st, qf, L, k_begin, last_key, blk_last, scale_log2e, lane);
        if (valid) {
            float *out = part + (((size_t)row * hq + head) * n_splits + split) * REC;
            if (g4 == 0) { out[0] = st.m_run; out[1] = st.l_run; }
#pragma unroll
            for (int db = 0; db < DB; ++db)
                *reinterpret_cast<floatx4 *>(out + ATTF_STRIDE_PAD + db * 16 + g4 * 4) = st.o[db];
        }
    }
}

// Many rows (a prefill chunk, or a large batch): one workgroup of eight wavefronts per (ROWS_QB blocks
// of 16 query items, kv head, sequence, part of the keys).  The wavefronts take the 32-key tiles its
// items can see in turn (tile t goes to wavefront t mod 8); a tile's K and V^T fragments go from the
// cache straight into registers (the cache keeps them in operand order: every load a contiguous
// kilobyte), once, and serve every item block.  Each wavefront keeps an online softmax state per item
// block; the eight states are merged through LDS at the end.  Output in the bf16 activation (MFMA
// B-operand) layout the general GEMM reads; with more than one key part, a record per (row, head) for
// the merge kernel.  Measured and not taken: the tiles of a workgroup of 128 items handed through LDS
// to eight wavefronts that own 16 items each, with the parts merged by the last one to arrive (no
// faster: the merging workgroup pulls every part's state through one compute unit); the next tile
// requested ahead of the current one's arithmetic, and twice the wavefronts per SIMD (both slower).
#ifndef ROWS_QB_N
#define ROWS_QB_N 1
#endif
#ifndef ROWS_PART_TILES
#define ROWS_PART_TILES 64   // key tiles (of 32 keys) per workgroup of the many-row attention before the keys are split
#endif
constexpr int ROWS_QB = ROWS_QB_N, ROWS_WAVES = 8;

template <int HD>
__global__ __launch_bounds__(ROWS_WAVES * 64) void attn_rows_kernel(Batch b, int layer, const bf16_t *__restrict__ q,
                                                                   bf16_t *__restrict__ o, int hq, int hkv, int ncb,
                                                                   float scale_log2e, int n_parts,
                                                                   float *__restrict__ part) {
    constexpr int KD = HD / 32, DB = HD / 16;
    extern __shared__ __align__(16) unsigned char rows_smem[];
    floatx4 *o_s = reinterpret_cast<floatx4 *>(rows_smem);                            // [wave][db][lane]
    float *ml_s = reinterpret_cast<float *>(rows_smem + ROWS_WAVES * DB * 64 * 16);  // [wave][2][16]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g4 = lane >> 4, l15 = lane & 15;
    // n_parts > 1: the keys of a block are shared out over n_parts workgroups (blockIdx.z = sequence *
    // n_parts + part), each leaving an unnormalised record [max, sum, -, -, O[hd]] per (row, head) for
    // the merge kernel; long contexts then fill the GPU with more than one workgroup per block
    const int kvh = blockIdx.y, kpart = blockIdx.z % n_parts;
    const SeqDesc &s = b.s[blockIdx.z / n_parts];
    const int group = hq / hkv, n_items = s.nrows * group;
    const int item0 = blockIdx.x * (16 * ROWS_QB);
    if (item0 >= n_items) return;
    const int len = s.state[0];
    const int kmax = min(len + s.nrows, s.capacity);
    bf16x8 qf[ROWS_QB][KD];
    AttState<HD> st[ROWS_QB];
    int last_key[ROWS_QB], blk_last[ROWS_QB], row[ROWS_QB], head[ROWS_QB];
    bool valid[ROWS_QB];
#pragma unroll
    for (int c = 0; c < ROWS_QB; ++c) {
        const int item = item0 + c * 16 + l15;
        valid[c] = item < n_items;
        const int r = valid[c] ? item / group : 0;
        head[c] = kvh * group + (valid[c] ? item % group : 0);
        row[c] = s.row0 + r;
        last_key[c] = valid[c] ? len + r : -1;
        blk_last[c] = min(kmax - 1, len + min(s.nrows - 1, (item0 + c * 16 + 15) / group));
#pragma unroll
        for (int kd = 0; kd < KD; ++kd)
            qf[c][kd] = *reinterpret_cast<const bf16x8 *>(q + ((size_t)row[c] * hq + head[c]) * HD + kd * 32 + g4 * 8);
#pragma unroll
        for (int db = 0; db < DB; ++db) st[c].o[db] = floatx4{0.f, 0.f, 0.f, 0.f};
        st[c].m_run = -1e30f;
        st[c].l_run = 0.f;
    }
    const int tiles = blk_last[ROWS_QB - 1] / ATT_TILE + 1;  // the last block sees the most keys
    const int tpp = (tiles + n_parts - 1) / n_parts;
    const int t_begin = kpart * tpp, t_end = min(tiles, t_begin + tpp);
    // The pages of this part's tiles, one per lane, read once: a look-up in the block table per tile
    // would be a second memory round trip in front of every tile's loads.
    const int page0 = t_begin * ATT_TILE / VF_TILE;
    int page_v = 0;
    if (s.block_table) page_v = s.block_table[min(page0 + lane, (tiles * ATT_TILE - 1) / VF_TILE)];
    auto request = [&](AttTile<HD> &tile, int t) {
        const int t0 = min(t, t_end - 1) * ATT_TILE;  // past the end: the part's last tile again, not used
        const int pi = t0 / VF_TILE - page0;          // the same for the whole wavefront
        const int page = !s.block_table ? t0 / VF_TILE
                         : pi < 64      ? __builtin_amdgcn_readlane(page_v, pi)
                                        : __builtin_amdgcn_readfirstlane(kv_page(s, t0));
        tile.template load_page<false>(s, layer, hkv, kvh, t0 / ATT_TILE, page, lane);
    };
    auto work = [&](AttTile<HD> &tile, int t) {
        const int t0 = t * ATT_TILE;
        tile.mask_values(t0, kmax, lane);
#pragma unroll
        for (int c = 0; c < ROWS_QB; ++c)
            if (t0 <= blk_last[c]) att_tile_update<HD>(st[c], qf[c], tile, t0, last_key[c], ATT_NO_TREE, 0, scale_log2e, lane);
    };
    AttTile<HD> tile;
#pragma unroll 1
    for (int t = t_begin + wave; t < t_end; t += ROWS_WAVES) {
        request(tile, t);
        work(tile, t);
    }
    // merge of the eight wavefronts, one item block at a time: thread (db = wave, lane) owns
    // O^T[d = 16*db + 4*g4 + j][item l15]; HD = 64 leaves wavefronts 4..7 idle here
#pragma unroll
    for (int c = 0; c < ROWS_QB; ++c) {
        if (c) lds_sync();
#pragma unroll
        for (int db = 0; db < DB; ++db) o_s[(wave * DB + db) * 64 + lane] = st[c].o[db];
        if (g4 == 0) {
            ml_s[(wave * 2 + 0) * 16 + l15] = st[c].m_run;
            ml_s[(wave * 2 + 1) * 16 + l15] = st[c].l_run;
        }
        lds_sync();
        if (wave < DB) {
            float M = -1e30f, L = 0.f;
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < ROWS_WAVES; ++w) M = fmaxf(M, ml_s[(w * 2) * 16 + l15]);
#pragma unroll
            for (int w = 0; w < ROWS_WAVES; ++w) {
                const float wt = exp2f(ml_s[(w * 2) * 16 + l15] - M);
                L += ml_s[(w * 2 + 1) * 16 + l15] * wt;
                acc += o_s[(w * DB + wave) * 64 + lane] * wt;
            }
            if (valid[c] && n_parts > 1) {
                float *rec = part + (((size_t)row[c] * hq + head[c]) * n_parts + kpart) * (HD + ATTF_STRIDE_PAD);
                if (wave == 0 && g4 == 0) *reinterpret_cast<float2 *>(rec) = float2{M, L};
                *reinterpret_cast<floatx4 *>(rec + ATTF_STRIDE_PAD + wave * 16 + g4 * 4) = acc;
            } else if (valid[c]) {
                const float inv = 1.0f / L;
                const int k = head[c] * HD + wave * 16 + g4 * 4;
                *reinterpret_cast<u32x2 *>(o + xfrag_index(row[c], k, ncb)) =
                    pack4_bf16(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
            }
        }
    }
}

// Merge of the key slices by log-sum-exp; one workgroup per (row, head), one thread per d.
template <int HD>
__global__ __launch_bounds__(HD) void attn_fast_combine_kernel(Batch b, const float *__restrict__ part,
                                                               bf16_t *__restrict__ o, int hq, int n_splits) {
    constexpr int REC = HD + ATTF_STRIDE_PAD;
    __shared__ float ws[VF_ATTN_SPLIT_MAX], ls[VF_ATTN_SPLIT_MAX];
    const int row = blockIdx.x / hq, head = blockIdx.x % hq, d = threadIdx.x;
    const SeqDesc &s = b.s[find_seq(b, row)];
    const int kmax = min(s.state[0] + s.nrows, s.capacity);
    const int used = min(n_splits, (kmax + ATT_KEYS - 1) / ATT_KEYS);  // slices that had keys
    const float *p = part + ((size_t)row * hq + head) * n_splits * REC;
    for (int i = d; i < used; i += HD) {
        ws[i] = p[i * REC];
        ls[i] = p[i * REC + 1];
    }
    __syncthreads();
    float M = -1e30f;
    for (int i = 0; i < used; ++i) M = fmaxf(M, ws[i]);
    __syncthreads();
    for (int i = d; i < used; i += HD) ws[i] = exp2f(ws[i] - M);
    __syncthreads();
    float L = 0.f, acc = 0.f;
    for (int i = 0; i < used; ++i) L += ls[i] * ws[i];
    int i = 0;
    for (; i + 8 <= used; i += 8) {
        float t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = p[(i + j) * REC + ATTF_STRIDE_PAD + d];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += t[j] * ws[i + j];
    }
    for (; i < used; ++i) acc += p[i * REC + ATTF_STRIDE_PAD + d] * ws[i];
    o[(size_t)row * hq * HD + head * HD + d] = (bf16_t)(acc / L);
}

// The same merge for the many-row kernel's key parts; the output goes to the activation layout.
template <int HD>
__global__ __launch_bounds__(HD) void attn_rows_combine_kernel(const float *__restrict__ part, bf16_t *__restrict__ o,
                                                               int hq, int n_parts, int ncb) {
    constexpr int REC = HD + ATTF_STRIDE_PAD;
    const int row = blockIdx.x / hq, head = blockIdx.x % hq, d = threadIdx.x;
    const float *p = part + ((size_t)row * hq + head) * n_parts * REC;
    float M = -1e30f;
    for (int i = 0; i < n_parts; ++i) M = fmaxf(M, p[i * REC]);
    float L = 0.f, acc = 0.f;
    for (int i = 0; i < n_parts; ++i) {
        const float w = exp2f(p[i * REC] - M);
        L += p[i * REC + 1] * w;
        acc += p[i * REC + ATTF_STRIDE_PAD + d] * w;
    }
    o[xfrag_index(row, head * HD + d, ncb)] = (bf16_t)(acc / L);
}

// ---- host side -------------------------------------------------------------------------------------

constexpr size_t LDS_X_BUDGET = 53 * 1024;
// launch shapes: wavefronts per workgroup and the workgroup count to reach by splitting K
#ifndef QKV_NW
#define QKV_NW 16
#define QKV_WGS 0
#define O_NW 16
#define O_WGS 0
#define GU_NW 4
#define GU_WGS 0
#define DOWN_NW 4
#define DOWN_WGS 768
#define HEAD_NW 4
#endif

// want_wgs: workgroups to aim for by splitting K across workgroups (0: never split).
template <int NB, int UB, int PD, int EPI, int NW>
int launch_gemm(FastGemm g, const Batch &b, int units, int want_wgs, hipStream_t st) {
    const int m = g.m;
    int ks = 1;
    while (units * ks < want_wgs && g.KB / (ks * 2) >= NW) ks *= 2;
    int kbps = (g.KB + ks - 1) / ks;
    ks = (g.KB + kbps - 1) / kbps;
    int kch = kbps;
    while ((size_t)kch * m * 64 > LDS_X_BUDGET) kch = (kch + 1) / 2;
    g.ks = ks;
    g.kbps = kbps;
    g.kch = kch;
    size_t lds = (size_t)kch * m * 64;
    const size_t red = (size_t)NW * UB * NB * 1024;
    if (red > lds) lds = red;
    auto kern = gemm_fast_kernel<NB, UB, PD, EPI, NW>;
    static bool attr_done = false;
    if (!attr_done) {
        VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)(LDS_X_BUDGET > red ? LDS_X_BUDGET : red)));
        attr_done = true;
    }
    hipLaunchKernelGGL(kern, dim3(units, ks), dim3(NW * 64), lds, st, g, b);
    VF_LAUNCH_CHECK("gemm_fast");
    return VF_OK;
}

template <int NB>
int run_fast(vf_model *m, const Batch &b, const int32_t *tokens, float *logits_out, hipStream_t st) {
    const vf_config &c = m->cfg;
    const int rows = b.total_rows;
    const int d = c.d_model, F = c.d_ffn, hd = c.head_dim, nq = c.n_q_heads * hd, nkv = c.n_kv_heads * hd;
    bf16_t *o = (bf16_t *)m->o, *a = (bf16_t *)m->a, *q = (bf16_t *)m->q;
    int rc;
    hipLaunchKernelGGL(embed_fast_kernel, dim3(rows), dim3(256), 0, st, (const bf16_t *)m->embed, tokens, b, m->h,
                       m->ss, d, c.vocab);
    VF_LAUNCH_CHECK("embed_fast");

    FastGemm base;
    memset(&base, 0, sizeof base);
    base.m = rows;
    base.part = m->part;
    base.counters = m->counters;
    base.ss_in = m->ss;
    base.n_ss = d / 16;
    base.inv_d = 1.0f / (float)d;
    base.eps = c.rms_eps;
    base.h_in = m->h;
    base.h = m->h;
    base.ss_out = m->ss;
    base.a_out = a;
    base.F = F;
    base.cosv = m->rope_cos;
    base.sinv = m->rope_sin;
    base.q = q;
    base.hq = c.n_q_heads;
    base.hkv = c.n_kv_heads;
    base.hd = hd;

    // attention split
    int max_keys = 0;
    for (int i = 0; i < b.n_seqs; ++i) max_keys = max(max_keys, b.s[i].len_ub + b.s[i].nrows);
    const int n_splits = (max_keys + ATT_KEYS - 1) / ATT_KEYS;
    if (n_splits > VF_ATTN_SPLIT_MAX) return vf_fail(VF_ERR_UNSUPPORTED, "context of %d keys", max_keys);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)hd);

    for (int l = 0; l < c.n_layers; ++l) {
        const LayerPacked &lp = m->layers[l];
        {
            ProfScope ps(m, VF_SITE_QKV, st);
            FastGemm g = base;
            g.W = (const u32x4 *)lp.wqkv; g.N = nq + 2 * nkv; g.KB = d / 32; g.Xh = m->h; g.gain = lp.attn_norm;
            g.bias = c.qkv_bias ? lp.bqkv : nullptr; g.layer = l;
            if ((rc = launch_gemm<NB, 1, 8, EPI_QKV, QKV_NW>(g, b, g.N / 16, QKV_WGS, st))) return rc;
        }
        {
            ProfScope ps(m, VF_SITE_ATTN, st);
            if (hd == 128) {
                hipLaunchKernelGGL(attn_fast_kernel<128>, dim3(n_splits, c.n_kv_heads, b.n_seqs), dim3(256), 0, st, b, l,
                                   q, m->attn_part, c.n_q_heads, c.n_kv_heads, n_splits, scale_log2e);
                hipLaunchKernelGGL(attn_fast_combine_kernel<128>, dim3(rows * c.n_q_heads), dim3(128), 0, st, b,
                                   m->attn_part, o, c.n_q_heads, n_splits);
            } else {
                hipLaunchKernelGGL(attn_fast_kernel<64>, dim3(n_splits, c.n_kv_heads, b.n_seqs), dim3(256), 0, st, b, l,
                                   q, m->attn_part, c.n_q_heads, c.n_kv_heads, n_splits, scale_log2e);
                hipLaunchKernelGGL(attn_fast_combine_kernel<64>, dim3(rows * c.n_q_heads), dim3(64), 0, st, b,
                                   m->attn_part, o, c.n_q_heads, n_splits);
            }
            VF_LAUNCH_CHECK("attn_fast");
        }
        {
            ProfScope ps(m, VF_SITE_O, st);
            FastGemm g = base;
            g.W = (const u32x4 *)lp.wo; g.N = d; g.KB = nq / 32; g.X = o;
            if ((rc = launch_gemm<NB, 1, 8, EPI_RESID, O_NW>(g, b, d / 16, O_WGS, st))) return rc;
        }
        {
            ProfScope ps(m, VF_SITE_GATEUP, st);
            FastGemm g = base;
            g.W = (const u32x4 *)lp.wgu; g.N = 2 * F; g.KB = d / 32; g.Xh = m->h; g.gain = lp.ffn_norm;
            if ((rc = launch_gemm<NB, 2, 6, EPI_SWIGLU, GU_NW>(g, b, F / 16, GU_WGS, st))) return rc;
        }
        {
            ProfScope ps(m, VF_SITE_DOWN, st);
            FastGemm g = base;
            g.W = (const u32x4 *)lp.wd; g.N = d; g.KB = F / 32; g.X = a;
            if ((rc = launch_gemm<NB, 1, 8, EPI_RESID, DOWN_NW>(g, b, d / 16, DOWN_WGS, st))) return rc;
        }
    }
    {
        ProfScope ps(m, VF_SITE_HEAD, st);
        FastGemm g = base;
        g.W = (const u32x4 *)m->lm_head; g.N = c.vocab; g.KB = d / 32; g.Xh = m->h; g.gain = m->final_norm; g.logits = logits_out;
        const int units = (c.vocab / 16 + 1) / 2;
        if ((rc = launch_gemm<NB, 2, 6, EPI_LOGITS, HEAD_NW>(g, b, units, 0, st))) return rc;
    }
    return VF_OK;
}

}  // namespace

int vf_launch_attention_rows(const vf_model *m, const Batch &b, int layer, hipStream_t st) {
    const vf_config &c = m->cfg;
    const int group = c.n_q_heads / c.n_kv_heads;
    int max_items = 0, max_keys = 0;
    for (int i = 0; i < b.n_seqs; ++i) {
        max_items = max(max_items, b.s[i].nrows * group);
        max_keys = max(max_keys, b.s[i].len_ub + b.s[i].nrows);
    }
    // about ROWS_PART_TILES key tiles per workgroup; the record buffer has room for 16 parts per (row, head)
    const int max_tiles = (max_keys + ATT_TILE - 1) / ATT_TILE;
    int n_parts = min(16, max(1, (max_tiles + ROWS_PART_TILES - 1) / ROWS_PART_TILES));
    const size_t rec_floats = (size_t)b.total_rows * c.n_q_heads * (c.head_dim + ATTF_STRIDE_PAD);
    while (n_parts > 1 && rec_floats * n_parts > m->attn_part_floats) --n_parts;
    const dim3 grid((max_items + 16 * ROWS_QB - 1) / (16 * ROWS_QB), c.n_kv_heads, b.n_seqs * n_parts);
    const int ncb = (b.total_rows + 15) >> 4;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)c.head_dim);
    const int lds = ROWS_WAVES * (c.head_dim / 16) * 64 * 16 + ROWS_WAVES * 2 * 16 * 4;
    static bool attr_done = false;
    if (!attr_done) {
        VF_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(attn_rows_kernel<128>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, ROWS_WAVES * 8 * 64 * 16 + 1024));
        attr_done = true;
    }
    if (c.head_dim == 128)
        hipLaunchKernelGGL(attn_rows_kernel<128>, grid, dim3(ROWS_WAVES * 64), lds, st, b, layer, (const bf16_t *)m->q,
                           (bf16_t *)m->o, c.n_q_heads, c.n_kv_heads, ncb, scale_log2e, n_parts, m->attn_part);
    else
        hipLaunchKernelGGL(attn_rows_kernel<64>, grid, dim3(ROWS_WAVES * 64), lds, st, b, layer, (const bf16_t *)m->q,
                           (bf16_t *)m->o, c.n_q_heads, c.n_kv_heads, ncb, scale_log2e, n_parts, m->attn_part);
    VF_LAUNCH_CHECK("attn_rows");
    if (n_parts > 1) {
        if (c.head_dim == 128)
            hipLaunchKernelGGL(attn_rows_combine_kernel<128>, dim3(b.total_rows * c.n_q_heads), dim3(128), 0, st,
                               m->attn_part, (bf16_t *)m->o, c.n_q_heads, n_parts, ncb);
        else
            hipLaunchKernelGGL(attn_rows_combine_kernel<64>, dim3(b.total_rows * c.n_q_heads), dim3(64), 0, st,
                               m->attn_part, (bf16_t *)m->o, c.n_q_heads, n_parts, ncb);
        VF_LAUNCH_CHECK("attn_rows_combine");
    }
    return VF_OK;
}

bool vf_fast_path_ok(const vf_model *m, int total_rows) {
    return m->cfg.dtype == VF_BF16 && total_rows <= 48 && m->cfg.d_model % 64 == 0;
}

int vf_run_fast(vf_model *m, const Batch &b, const int32_t *tokens, float *logits_out, hipStream_t st) {
    const int rows = b.total_rows;
    if (rows <= 16) return run_fast<1>(m, b, tokens, logits_out, st);
    if (rows <= 32) return run_fast<2>(m, b, tokens, logits_out, st);
    return run_fast<3>(m, b, tokens, logits_out, st);
}
