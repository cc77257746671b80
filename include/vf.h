/*
 * vf.h -- C ABI of the draft-verify library for AMD MI355X (gfx950).
 *
 * What it computes.  A small decoder-only language model (RMSNorm, rotary
 * embedding, grouped-query attention, SwiGLU, tied output head) is run over a
 * KV cache in the two regimes the paper's speculative decoding uses:
 *
 *   - chunked prefill: the prompt is fed in fixed-size chunks, each appended to
 *     the KV cache (paper Sec. 2 "on-device inference", Sec. 4.1);
 *   - verify: the pending token T and k draft tokens x_1..x_k are scored in ONE
 *     forward pass, giving predictions y_1..y_{k+1} (paper Sec. 3
 *     "draft-then-verify", Sec. 4.3 "x = [T, x_1..x_n], y = [y_1..y_{n+1}]");
 *   - accept: the longest draft prefix that matches the predictions is kept,
 *     everything from the first mismatch on is dropped, and one corrected (or
 *     bonus) token is emitted (paper Sec. 3, draft-then-verify; Sec. 4.3:
 *     accepted prefix x_1..x_{e-1}, y_e).  Greedy (strict) acceptance and the
 *     distribution-preserving stochastic rule (speculative sampling, from the
 *     work the paper cites in Sec. 3 for its lossless property) are both
 *     provided.
 *
 * Conventions.
 *   - Every function returns int: VF_OK or a negative VF_ERR_* code.  Nothing
 *     throws or aborts.  vf_last_error() gives a thread-local message for the
 *     last failing call on this thread.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *     host memory.  The library never allocates device memory: every device
 *     buffer (raw weights, packed model, KV pool, sequence state, inputs,
 *     outputs) is owned by the caller and must outlive its use.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     work is enqueued asynchronously on it; no call synchronises except where
 *     stated.  Calls that touch the same model or sequence must be issued on
 *     one stream (or be ordered by the caller).
 *   - Errors detected on the host (bad arguments, capacity) are reported
 *     before anything is enqueued and leave all state unchanged.
 */
#ifndef VF_H
#define VF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VF_OK               0
#define VF_ERR_ARG         (-1)  /* NULL / out-of-range / inconsistent argument            */
#define VF_ERR_CAP         (-2)  /* KV capacity or workspace rows exceeded; state unchanged */
#define VF_ERR_HIP         (-3)  /* a HIP runtime call failed                               */
#define VF_ERR_UNSUPPORTED (-4)  /* shape or dtype the kernels are not built for            */

#define VF_F32   0   /* weights, activations and KV cache in float32                        */
#define VF_BF16  1   /* bfloat16 weights / activations / KV cache, float32 accumulation     */

#define VF_GREEDY      0
#define VF_STOCHASTIC  1

#define VF_PENDING   (-1)   /* token id meaning "the sequence's pending token on the device" */
#define VF_MAX_BATCH   32   /* sequences per vf_verify / vf_accept call                      */
#define VF_TOPK_MAX      8   /* largest k of vf_prefill_chunk_topk                            */
#define VF_MAX_DRAFTS  32   /* draft tokens per sequence per verify (paper Sec. 5.1: cap 32) */

typedef struct vf_model vf_model;   /* opaque; host struct describing a packed model */
typedef struct vf_seq   vf_seq;     /* opaque; host struct describing one sequence   */

/* Model shape.  head_dim must be a multiple of 32, at most 128 and even; d_model, d_ffn and
 * n_q_heads*head_dim multiples of 32; vocab a multiple of 16; n_q_heads a multiple of
 * n_kv_heads.  max_rows = largest number of token rows one call may process (a prefill
 * chunk, or the sum over the batch of k_b+1 for a verify).  max_positions = largest position
 * + 1 any sequence may reach (rotary table size). */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;                 /* VF_F32 | VF_BF16 */
    float   rope_theta, rms_eps;
    int32_t tie_embeddings;        /* 1: output head = embedding matrix (lm_head ignored) */
    int32_t qkv_bias;              /* 1: bq/bk/bv are added before the rotary embedding   */
    int32_t max_rows;
    int32_t max_positions;
} vf_config;

/* Raw weights, DEVICE pointers, caller-owned, read only during vf_model_create.
 * Matrices are row-major [out_features, in_features] in the model dtype (bfloat16 bits or
 * float32).  Vectors (norm gains, biases) are always float32. */
typedef struct {
    const void *attn_norm;                 /* f32 [d_model]                              */
    const void *wq, *wk, *wv;              /* [Hq*hd, d], [Hkv*hd, d], [Hkv*hd, d]       */
    const void *bq, *bk, *bv;              /* f32, NULL unless qkv_bias                  */
    const void *wo;                        /* [d, Hq*hd]                                 */
    const void *ffn_norm;                  /* f32 [d_model]                              */
    const void *w_gate, *w_up, *w_down;    /* [F, d], [F, d], [d, F]                     */
} vf_layer_w;

typedef struct {
    const void *embed;                     /* [vocab, d]                                 */
    const void *lm_head;                   /* [vocab, d]; ignored when tie_embeddings    */
    const void *final_norm;                /* f32 [d]                                    */
    const vf_layer_w *layers;              /* HOST array of n_layers entries             */
} vf_weights;

const char *vf_last_error(void);

/* ---- model --------------------------------------------------------------------------------- */

/* Bytes of device memory vf_model_create needs for the re-packed weights, the rotary tables
 * and the activation workspace.  0 on invalid config (see vf_last_error). */
size_t vf_model_packed_bytes(const vf_config *cfg);

/* Re-packs the weights into `packed_dev` (packed_bytes >= vf_model_packed_bytes, 256-byte
 * aligned) on `stream`; the raw weights may be released once the stream has drained.  On
 * success *out owns only host memory. */
int vf_model_create(const vf_config *cfg, const vf_weights *w, void *packed_dev,
                    size_t packed_bytes, void *stream, vf_model **out);
int vf_model_destroy(vf_model *m);

/* ---- sequences and the KV cache ------------------------------------------------------------ */

/* Bytes of one sequence's device state (current length, pending token). */
size_t vf_seq_state_bytes(const vf_model *m);

/* Bytes of a KV pool.  page_tokens == 0: a private contiguous cache for `n` tokens (n is
 * rounded up to a multiple of 64 internally).  page_tokens == 64: a pool of `n` pages shared
 * by many sequences through their block tables.  Layout inside the pool is private to the
 * library (K row-major, V transposed in 64-token tiles); use vf_kv_read to inspect it. */
size_t vf_kv_bytes(const vf_model *m, int page_tokens, int n);

/* Binds a sequence to its KV memory.
 *   contiguous: page_tokens = 0, block_table_dev = NULL, kv_dev = private buffer of
 *               vf_kv_bytes(m, 0, capacity_tokens) bytes;
 *   paged:      page_tokens = 64, kv_dev = the shared pool of pool_pages pages,
 *               block_table_dev = int32[ceil(capacity_tokens/64)] page ids (device), which
 *               must stay valid and unchanged while the sequence is in use.
 * state_dev: vf_seq_state_bytes bytes; initialised (length 0, no pending token) on `stream`. */
int vf_seq_create(vf_model *m, void *kv_dev, size_t kv_bytes, int page_tokens, int pool_pages,
                  int capacity_tokens, const int32_t *block_table_dev, void *state_dev,
                  void *stream, vf_seq **out);
int vf_seq_destroy(vf_seq *s);

/* Sets the sequence length (positions >= len are dead and will be overwritten): roll-back,
 * teacher forcing.  Also resets the host-side upper bound of the length. */
int vf_seq_set_len(vf_seq *s, int len, void *stream);
/* Sets the pending token T (the last emitted token, not yet in the KV cache). */
int vf_seq_set_pending(vf_seq *s, int32_t token, void *stream);
/* Reads length and pending token back (synchronises the stream) and tightens the host-side
 * upper bound of the length to the true value.  Either output pointer may be NULL. */
int vf_seq_get_state(vf_seq *s, int32_t *len_host, int32_t *pending_host, void *stream);
/* The host-side bound of the length.  The true length lives on the device; the host keeps an
 * upper bound of it, which is what capacity checks (VF_ERR_CAP) and launch sizes use:
 * vf_prefill_chunk adds n_tokens to it, vf_accept adds the whole m_b = k_b + 1 (the device
 * commits only 1 + a_b of them), vf_seq_set_len and vf_seq_get_state set it to the true value.
 * A caller that learns the true length without vf_seq_get_state (it copied n_accept to the host
 * anyway) tightens the bound with this call: host only, no device work, no synchronisation.
 * `len` must not be below the true length after all work enqueued so far (a bound that is too
 * low lets later calls overrun the cache's capacity check); VF_ERR_ARG outside 0..capacity. */
int vf_seq_note_len(vf_seq *s, int len);

/* Debug / test accessor: copies K and V of `layer` for positions [t0, t0+n) into row-major
 * float32 arrays k_out_dev, v_out_dev of shape [n, n_kv_heads, head_dim]. */
int vf_kv_read(vf_model *m, vf_seq *s, int layer, int t0, int n, float *k_out_dev,
               float *v_out_dev, void *stream);

/* The inverse: overwrites K and V of `layer` for positions [t0, t0+n) with the given float32
 * arrays of shape [n, n_kv_heads, head_dim] (rounded to the model dtype; K is taken as is, i.e.
 * with the rotary embedding already applied).  Imports a cache computed elsewhere; the length
 * is not changed (use vf_seq_set_len). */
int vf_kv_write(vf_model *m, vf_seq *s, int layer, int t0, int n, const float *k_in_dev,
                const float *v_in_dev, void *stream);

/* ---- the three operations ------------------------------------------------------------------ */

/* Chunked prefill (paper Sec. 2, Sec. 4.1): runs n_tokens ids (tokens_dev, int32) at
 * positions len..len+n_tokens-1, appends their K/V, and advances the length.
 *   logits_mode 0: no logits returned; 1: float32 logits of the last row to
 *   logits_out_dev[vocab]; 2: of all rows to logits_out_dev[n_tokens, vocab] (the all-position
 *   logits the paper's calibration step consumes, Sec. 4.2).
 *   sample_first != 0: the last row also produces the pending token T: arg-max when
 *   temperature == 0, else an inverse-CDF sample of softmax(z/temperature) with the uniform
 *   u_dev[0] (float32 in [0,1), device).
 * n_tokens <= cfg.max_rows; VF_ERR_CAP if the host-side bound of the length (see vf_seq_note_len)
 * plus n_tokens exceeds the capacity. */
int vf_prefill_chunk(vf_model *m, vf_seq *s, const int32_t *tokens_dev, int n_tokens,
                     int logits_mode, float *logits_out_dev, int sample_first,
                     const float *u_dev, float temperature, void *stream);

/* Verify forward (paper Sec. 3, Sec. 4.3) for a ragged batch.  row_off_host[0..n_seqs] are
 * prefix sums of the per-sequence row counts m_b = k_b + 1 (1 <= m_b <= VF_MAX_DRAFTS+1).
 * tokens_dev[row_off[b]] is sequence b's pending token (or VF_PENDING to take it from the
 * device state), followed by its k_b drafts.  Rows sit at positions len_b .. len_b + k_b.
 * Writes K/V for all rows (the length is NOT advanced: vf_accept commits it) and leaves the
 * float32 logits of all rows for vf_accept: in logits_out_dev[total_rows, vocab] if that is
 * not NULL, else in the model workspace.
 * VF_ERR_CAP if the host-side bound of a sequence's length (see vf_seq_note_len) plus m_b exceeds
 * its capacity, or total rows exceed cfg.max_rows. */
int vf_verify(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
              const int32_t *row_off_host, float *logits_out_dev, void *stream);

typedef struct {
    int32_t mode;            /* VF_GREEDY | VF_STOCHASTIC                                    */
    float   temperature;     /* stochastic: target logits are divided by it (> 0)             */
    const float *q_dev;      /* stochastic: draft distributions [k_b, vocab] (rows sum to 1), */
                             /* or NULL for a deterministic drafter (one-hot at each draft)   */
    const float *u_dev;      /* stochastic: 2*(k_b+1) uniforms in [0,1): u[i] decides draft   */
                             /* i+1, u[k_b+1+i] drives the replacement/bonus draw at row i    */
} vf_accept_params;

/* Acceptance (paper Sec. 3, Sec. 4.3) on logits_dev[total_rows, vocab], or, if that is NULL,
 * on the logits the preceding vf_verify on this model left, for the same seqs / tokens_dev /
 * row_off_host.  Per sequence b, with a_b = number of accepted drafts:
 *   n_accept_dev[b]                         = a_b
 *   out_tokens_dev[row_off[b] .. +a_b]      = x_1..x_{a_b} then the corrected/bonus token
 *                                             (remaining entries of the slice are set to -1)
 *   y_dev[row_off[b] + i]                   = arg-max of row i's logits, for ALL rows (what
 *                                             the draft-reuse rule of Sec. 4.3 compares with)
 * and on the device: len_b += 1 + a_b, pending_b = the emitted token.  Arg-max ties go to
 * the lowest id.  Stochastic decisions use float64 probabilities from the float32 logits. */
int vf_accept(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
              const int32_t *row_off_host, const vf_accept_params *params_host,
              const float *logits_dev, int32_t *n_accept_dev, int32_t *out_tokens_dev,
              int32_t *y_dev, void *stream);

/* vf_accept for callers that must not allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results,
 * same state commit as vf_accept; the only difference is where the kernels keep their
 * intermediate results (per-chunk row statistics, draw descriptors, per-chunk draw sums): in
 * about 0.53 MB of device memory that is part of the loaded library itself (one copy per GPU,
 * held until the process ends) instead of the model workspace.  The call allocates nothing and
 * frees nothing, on the device or through any library.
 *   - total rows (row_off[n_seqs]) must not exceed VF_ACCEPT_STATIC_MAX_ROWS: VF_ERR_CAP.
 *   - every call on one GPU uses the same scratch, whichever model or stream it is given:
 *     calls that overlap in time on one GPU race; issue them on one stream or order them.
 *   - nothing in the scratch needs to start at zero; a call overwrites what it reads. */
#define VF_ACCEPT_STATIC_MAX_ROWS 512
int vf_accept_static(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                     const int32_t *row_off_host, const vf_accept_params *params_host,
                     const float *logits_dev, int32_t *n_accept_dev, int32_t *out_tokens_dev,
                     int32_t *y_dev, void *stream);

/* ---- top successors of every prefill position (next to the three operations) ---------------- */

/* vf_prefill_chunk that also returns, for EVERY row of the chunk, the top_k largest next-token
 * logits and their ids (paper Sec. 4.2, workflow step "Sample": the top-probability successors
 * of each context token, from which the calibrated token tree is built), without handing the
 * [n_tokens, vocab] logits to the caller:
 *   topk_logit_dev[n_tokens, top_k] float32, topk_id_dev[n_tokens, top_k] int32,
 * in falling order of the logit, equal logits by rising id (entry 0 is the arg-max of the row).
 * 1 <= top_k <= VF_TOPK_MAX.  sample_first / u_dev / temperature as in vf_prefill_chunk.  On a
 * bfloat16 model with more than 64 rows the candidates come out of the output-head GEMM's
 * epilogue and the logits are never written; otherwise they are computed into the model
 * workspace first.  Both give the top_k of the same float32 logits vf_prefill_chunk with
 * logits_mode 2 would return. */
int vf_prefill_chunk_topk(vf_model *m, vf_seq *s, const int32_t *tokens_dev, int n_tokens, int top_k,
                          float *topk_logit_dev, int32_t *topk_id_dev, int sample_first,
                          const float *u_dev, float temperature, void *stream);

/* ---- tree-structured drafts (next to the three operations) ---------------------------------- */

/* Verify forward for drafts that form a token tree per sequence (paper Sec. 4, workflow: the
 * drafts of a step are built and verified as a tree).  Arguments as vf_verify,
 * plus parent_host[total_rows] (HOST, int32): -1 for a sequence's first row (the pending token,
 * root of its tree), otherwise the row, counted within the sequence, of the node's parent, which
 * must be smaller than the node's own row.  Row r stands at position len + depth(r) (rotary
 * angle), sees the whole cache and, of the call's rows, only its ancestors and itself, and
 * predicts the token after its root path.  Its K/V go to cache row len + r; vf_accept_tree
 * moves the accepted path into place.  A chain (parent r-1 for every r) is exactly vf_verify.
 * VF_ERR_ARG for a malformed parent table; otherwise errors as vf_verify. */
int vf_verify_tree(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                   const int32_t *row_off_host, const int32_t *parent_host, float *logits_out_dev,
                   void *stream);

/* Acceptance over the tree, for the same seqs / tokens_dev / row_off_host / parent_host.  From the
 * root, the walk moves to a child while one is accepted and emits one more token at the node
 * where it stops:
 *   VF_GREEDY      the child whose token equals the arg-max at the current node (the lowest row
 *                  among children with equal tokens); the emitted token is that arg-max;
 *   VF_STOCHASTIC  deterministic drafter only (q_dev must be NULL, else VF_ERR_UNSUPPORTED): the
 *                  children are tried in row order against the residual r of the node's target
 *                  distribution (r = p at first): child c with token x is kept when
 *                  u[c-1] * sum(r) < r(x); a refused child's token is struck from r; the emitted
 *                  token is drawn from r by inverse CDF with u[m_b + node].  For a chain this is
 *                  vf_accept with a deterministic drafter.
 * Outputs as vf_accept (n_accept_dev[b] = a_b accepted drafts, out_tokens_dev = their tokens then
 * the emitted one, y_dev = arg-max of every row), plus
 *   path_dev[row_off[b] + j] = row of the j-th node of the accepted path, j = 0..a_b (path[0] = 0),
 *                              -1 beyond.
 * On the device: the K/V rows of the path move to cache rows len_b + 1 .. len_b + a_b,
 * len_b += 1 + a_b, pending_b = the emitted token. */
int vf_accept_tree(vf_model *m, vf_seq *const *seqs, int n_seqs, const int32_t *tokens_dev,
                   const int32_t *row_off_host, const int32_t *parent_host,
                   const vf_accept_params *params_host, const float *logits_dev, int32_t *n_accept_dev,
                   int32_t *out_tokens_dev, int32_t *y_dev, int32_t *path_dev, void *stream);

/* ---- reuse of rejected draft tokens (next to the three operations) --------------------------- */

/* The segment of a rejected draft worth keeping (paper Sec. 4.3, "Reuse strategy", Eq. (reuse)):
 * per sequence b with drafts x_1..x_k = tokens_dev[row_off[b]+1 ..], predictions
 * y_i = y_dev[row_off[b] + i - 1] (what vf_accept wrote) and a_b = n_accept_dev[b] accepted
 * drafts, i.e. a rejection at e = a_b + 1, finds the longest run of positions i in (e, k] with
 * x_i == y_i, the earliest among runs of equal length, and writes
 *   seg_dev[2b] = its first position (1-based draft index), seg_dev[2b+1] = its length;
 * both 0 when a_b == k or no position agrees.  All pointers but row_off_host are device
 * memory (int32); nothing else is read or written; asynchronous on `stream`. */
int vf_reuse_select(int n_seqs, const int32_t *tokens_dev, const int32_t *row_off_host,
                    const int32_t *y_dev, const int32_t *n_accept_dev, int32_t *seg_dev, void *stream);

/* The segment held between steps (paper Sec. 4.3: kept for at least one step, dropped once its
 * lifetime or the total draft length passes a limit; the limit on the length is 32, Sec. 5.1).
 * Plain host memory owned by the caller; the functions touch no device.  One segment is held:
 * a newly found one replaces it only if it is longer, and then starts a new lifetime. */
typedef struct {
    int32_t tokens[VF_MAX_DRAFTS];
    int32_t len;        /* tokens held (0 = none)                          */
    int32_t age;        /* verify steps since the held segment was found   */
    int32_t max_age;    /* the segment is dropped when age exceeds this    */
    int32_t cap;        /* largest total number of drafts of a step        */
} vf_reuse_pool;

/* 0 <= max_age, 1 <= cap <= VF_MAX_DRAFTS. */
int vf_reuse_pool_init(vf_reuse_pool *p, int max_age, int cap);
/* After a verify step whose drafts were drafts_host[0..n_drafts) and whose segment
 * (seg_start, seg_len) came from vf_reuse_select: ages the held segment by one step, drops it
 * past max_age, then takes the new one if it is longer. */
int vf_reuse_pool_update(vf_reuse_pool *p, const int32_t *drafts_host, int n_drafts, int seg_start,
                         int seg_len);
/* Appends the held segment to the n_fresh drafts in drafts_host (room for cap entries) if the
 * total stays within cap; a segment that does not fit is dropped, not cut.  Returns the new
 * number of drafts (>= n_fresh), or a negative VF_ERR_* code. */
int vf_reuse_pool_extend(vf_reuse_pool *p, int32_t *drafts_host, int n_fresh);

/* A retrieval drafter over the token history (paper Sec. 3: the context is the draft source;
 * Sec. 5.1: suffix-automaton retrieval).  Host memory only, no device work.  Finds the longest
 * suffix of history_host[0..n) of length min_suffix..max_suffix that also occurs earlier (ending
 * before the last token), takes its most recent such occurrence and copies up to k tokens that
 * followed it (the copy stops at the end of the history) to drafts_host.  Returns the number of
 * drafts written (0 if no suffix matches), or a negative VF_ERR_* code.  k <= VF_MAX_DRAFTS. */
int vf_draft_suffix_match(const int32_t *history_host, int n, int max_suffix, int min_suffix, int k,
                          int32_t *drafts_host);

/* ---- options ---------------------------------------------------------------------------------- */

/* VF_OPT_FAST_PATH (default 1): vf_verify on a bfloat16 model with at most 48 rows in total runs
 * the fused few-row kernels; 0 forces the general kernels (any row count), which compute the
 * same function. */
#define VF_OPT_FAST_PATH 1
/* VF_OPT_PERSISTENT (default 1): when the few-row kernels apply and the activations of the call fit
 * on-chip memory, vf_verify runs the whole forward pass as one persistent kernel whose phases are
 * separated by grid-wide barriers; 0 keeps one kernel per GEMM.  Same function, same rounding
 * points; sums are taken in a different (fixed) order.  The persistent kernel occupies the whole
 * GPU: two vf_verify calls on the same model must not overlap (they share its workspace anyway),
 * and a barrier that cannot complete within seconds (the GPU shared with another process that
 * keeps workgroups from becoming resident) gives up; vf_seq_get_state and vf_profile_read then
 * report VF_ERR_HIP. */
#define VF_OPT_PERSISTENT 2
int vf_set_option(vf_model *m, int option, int value);

/* ---- measurement hook (not part of the method) ---------------------------------------------- */

/* Kernel sites timed by vf_profile: the five GEMMs of the forward pass, attention (both
 * kernels), the small norm / epilogue kernels together, acceptance, and the persistent whole-pass kernel
 * (which replaces the first six when it runs). */
#define VF_SITE_QKV     0
#define VF_SITE_O       1
#define VF_SITE_GATEUP  2
#define VF_SITE_DOWN    3
#define VF_SITE_HEAD    4
#define VF_SITE_ATTN    5
#define VF_SITE_SMALL   6
#define VF_SITE_ACCEPT  7
#define VF_SITE_STEP    8
#define VF_N_SITES      9

/* enable != 0: from now on every launch group of the sites above is bracketed by a pair of
 * HIP events on the call's stream (costs about a microsecond per event; leave it off when
 * timing whole steps).  enable == 0: stop recording. */
int vf_profile(vf_model *m, int enable);
/* Synchronises with the recorded events, adds up elapsed milliseconds and launch counts per
 * site into ms_host[VF_N_SITES] / count_host[VF_N_SITES], and clears the record. */
int vf_profile_read(vf_model *m, float *ms_host, int32_t *count_host);

/* Yardstick for the roofline: one kernel that reads every packed weight of the model (what a verify
 * step must stream at least) and does nothing else.  Returns the number of bytes it reads in
 * *bytes_host; the caller times it with events on `stream`.  Writes 4 bytes of workspace. */
int vf_stream_read(vf_model *m, size_t *bytes_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VF_H */
