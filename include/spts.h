/*
 * spts.h -- C ABI of the SPTS token-skipped decoder-layer prefill for AMD MI355X (gfx950).
 *
 * SPTS ("Probe and Skip: Self-Predictive Token Skipping") runs each decoder layer of a
 * prefill on a subset of the candidate tokens:
 *   PAP  (Sec. 3.2, Eq. (mha_importance), Alg. 1 "Partial Attention Probing" block): keys of all
 *        candidates + queries of the trailing probe window give a score S^MHA per candidate; the
 *        top M_a candidates take Q/V projection, causal attention and the output projection, the
 *        others keep their residual (Eq. (skip));
 *   LTP  (Sec. 3.3, Eq. (proxy_ffn), (ffn_transformation), (ffn_importance), (ffn_selection)): a
 *        rank-r proxy of the SwiGLU FFN predicts each token's update norm C^FFN; the top M_f
 *        candidates by C^FFN * S^MHA take the full FFN (Eq. (ffn_function));
 *   MSDP (Sec. 3.4, Eq. (stage_prune)): at a stage end the candidate set itself is cut down to the
 *        top N_{s+1} candidates by the last S^MHA and the hidden states are compacted.
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned, valid until the
 *    stream work queued by the call has finished.  The library keeps no caller pointer after a call
 *    returns except the workspace and stream given to spts_create.
 *  - All calls are asynchronous on the context's HIP stream and never synchronise with the host.
 *    All counts (N, budgets) are host integers.
 *  - Element type of hidden states, weights, K/V: spts_model_desc.dtype (fp32, or bf16 with fp32
 *    accumulation).  Scores are fp32, indices and positions int32.
 *  - Matrices are row-major.  Every weight/factor matrix is stored [d_out, d_in] so that a
 *    projection is y = x * W^T (the layout checkpoints use for linear layers).  In the paper's
 *    notation (y = x W): Wq = W_Q^T [H*d, D], Wk = W_K^T [Hkv*d, D], Wv = W_V^T [Hkv*d, D],
 *    Wo = W_O^T [D, H*d], Wgate = W_gate^T [Dff, D], Wup = W_up^T [Dff, D], Wdown = W_down [D, Dff]
 *    (the paper applies W_down transposed), Ug = U_gate^T [r, D], Vg = V_gate^T [Dlow, r],
 *    Uu = U_up^T [r, D], Vu = V_up^T [Dlow, r], Ud = U_down [D, r], Vd = V_down [r, Dlow].
 *  - Candidates are rows 0..N-1 of x with strictly ascending absolute positions pos[]; rotary
 *    embedding (pairing (j, j+d/2), theta_j = rope_base^(-2j/d)) and the causal mask use pos[].
 *    RMSNorm precedes attention and FFN (pre-norm block).
 *  - Selected index lists are ascending; TopK is the k largest under (score descending, index
 *    ascending), -0.0 == +0.0; NaN scores are a caller error.  With protect_last != 0 and k >= 1 the
 *    last candidate is always selected.
 *  - Return value: SPTS_OK or a negative spts_status.  Arguments are validated before any launch;
 *    after an error the outputs are unspecified.  Nothing throws across this boundary.
 */
#ifndef SPTS_H
#define SPTS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SPTS_OK = 0,
    SPTS_EINVAL = -1,     /* null pointer, negative size, k > N, probe_len > N or < 1 ...          */
    SPTS_ESHAPE = -2,     /* unsupported dimensions (H % Hkv, odd d, d > 256, sizes beyond create) */
    SPTS_EALIGN = -3,     /* a data pointer is not 16-byte aligned                                 */
    SPTS_EWORKSPACE = -4, /* workspace given to spts_create is too small for this call            */
    SPTS_EDTYPE = -5,     /* dtype is neither SPTS_F32 nor SPTS_BF16                               */
    SPTS_EHIP = -6        /* a HIP call failed; see spts_last_hip_error                            */
} spts_status;

typedef enum { SPTS_F32 = 0, SPTS_BF16 = 1 } spts_dtype;

/* Layer dimensions in the paper's notation: D hidden, H query heads, Hkv key/value heads,
 * d head dimension, Dff FFN inner dimension (Sec. 3.2, 3.3). */
typedef struct {
    int32_t D, H, Hkv, d, Dff;
    float rms_eps;
    float rope_base;
    int32_t dtype; /* spts_dtype */
} spts_model_desc;

/* Device pointers to one layer's parameters, layouts as listed above.  gamma1/gamma2 are the
 * RMSNorm gains [D] in the model dtype.  The proxy factors may be NULL for a layer that is only
 * ever run with skip = 0. */
typedef struct {
    const void *Wq, *Wk, *Wv, *Wo, *gamma1;
    const void *Wgate, *Wup, *Wdown, *gamma2;
    const void *Ug, *Vg, *Uu, *Vu, *Ud, *Vd;
    int32_t r;    /* proxy rank                         */
    int32_t Dlow; /* proxy inner dimension (<= Dff)     */
    /* Optional slab-major copies of the projection / FFN matrices and of five proxy factors made by spts_pack_slab32 (NULL = none; bf16 only).
     * The prefill calls read a matrix through its copy where their matrix-core GEMM takes it (same arithmetic, same
     * results; the copy only changes which bytes a load instruction fetches together); the decode calls and the fp32
     * path always read the row-major originals, which must be given in any case.  Wgate_s and Wup_s go together, and
     * so do Vg_s and Vu_s, and Ug_s and Uu_s.
     * Contract: X_s must be spts_pack_slab32(X) of the matrix X given in the same struct, made after the last write
     * to X.  The library cannot tell a stale copy from a fresh one: prefill would then compute with the copy and
     * decode with the original, silently.  Re-pack whenever X changes. */
    const void *Wq_s, *Wk_s, *Wv_s, *Wo_s, *Wgate_s, *Wup_s, *Wdown_s;
    const void *Vg_s, *Vu_s, *Vd_s, *Ug_s, *Uu_s;
    /* Non-zero: the caller states that the columns of Ud are orthonormal, as a truncated SVD of W_down with the singular
     * values folded into Vd leaves them (all-zero columns of a zero-padded rank are fine when the matching rows of Vd
     * are zero too).  The norm of the proxy's output, C^FFN = || z Ud^T ||_2 (Eq. (ffn_transformation)), then equals
     * || z ||_2 and the library takes it from z without evaluating the output projection.  In exact arithmetic the two
     * are the same number; with factors rounded to bf16 they differ by the orthogonality defect of the rounded Ud
     * (below 1e-3 relative at D = 4096, r = 256).  The library does not check the statement: with a Ud that is not
     * orthonormal the scores are those of a different proxy.  0 = evaluate || z Ud^T ||_2 as written. */
    int32_t Ud_orthonormal;
} spts_layer_weights;

/* Per-layer control (Alg. 1: skip flag, budgets M_fixed; Sec. 3.4). */
typedef struct {
    int32_t skip;         /* 0: dense layer (the else-branches of Alg. 1); 1: PAP + LTP          */
    int32_t probe_len;    /* P >= 1 trailing candidates used as probe queries (P = 1 in Sec. 3.2)  */
    int64_t m_attn;       /* M_fixed for attention; the library applies min(N, m)                  */
    int64_t m_ffn;        /* M_fixed for the FFN; >= N: every candidate is active, the proxy is
                           * not evaluated (TopK of all N is the whole set)                      */
    int32_t protect_last; /* != 0: the last candidate is always active                             */
    int32_t kv_mode;      /* 0: keys/values of the active set only (Alg. 1); 1: of all candidates  */
} spts_layer_cfg;

/* KV cache of one layer (Sec. 3.2 last paragraph: only active pairs are cached).
 * k, v: [capacity, Hkv, d] model dtype, post-rotary keys; pos: [capacity] int32; caller-owned
 * device memory.  count lives on the host: spts_layer_prefill sets it to the number of rows it
 * filled, spts_decode_layer appends one row at index count and increments it. */
typedef struct {
    void *k, *v;
    int32_t *pos;
    int64_t capacity;
    int64_t count;
} spts_kv_out;

typedef struct spts_ctx spts_ctx;

/* Slab-major copy of a row-major matrix W [rows, K] of 2-byte elements (bf16): out[(s * rows + r) * 32 + j] =
 * W[r * K + 32 * s + j], i.e. the 32 columns of K slab s of consecutive rows lie next to each other (64 bytes per row).
 * A GEMM load instruction then moves 16 rows of a slab as 1 KB of whole cache lines instead of 64-byte halves of 16
 * lines (a layout choice of this library, not part of the method; Sec. 3.2 / 3.3 define the products it serves).
 * W and out are device pointers, 16-byte aligned, rows * K elements each, not overlapping; K % 32 == 0.
 * SPTS_EINVAL / SPTS_EALIGN / SPTS_ESHAPE on bad arguments; the copy is enqueued on the context's stream. */
int spts_pack_slab32(spts_ctx *ctx, const void *W, int64_t rows, int64_t K, void *out);

/* Bytes of device workspace a context needs to serve calls with N <= max_tokens,
 * probe_len <= max_probe, r <= max_r, Dlow <= max_dlow.  0 on invalid arguments. */
size_t spts_workspace_bytes(const spts_model_desc *model, int64_t max_tokens, int32_t max_probe,
                            int32_t max_r, int32_t max_dlow);

/* Creates a context bound to a HIP stream (hipStream_t passed as void*; NULL = default stream)
 * and to a caller-owned device workspace of at least spts_workspace_bytes(...) bytes, which must
 * stay allocated until spts_destroy.  The limits must be the ones the workspace was sized for.
 * Calls on one context must not overlap. */
int spts_create(spts_ctx **ctx, const spts_model_desc *model, void *hip_stream, void *workspace,
                size_t workspace_bytes, int64_t max_tokens, int32_t max_probe, int32_t max_r,
                int32_t max_dlow);
void spts_destroy(spts_ctx *ctx);
const char *spts_strerror(int status);
/* Last hipError_t seen by this context (0 if none), as an int. */
int spts_last_hip_error(const spts_ctx *ctx);
/* 1 if the matrix-core (MFMA bf16) kernels serve this context's shapes, 0 if the generic kernels do. */
int spts_uses_mfma(const spts_ctx *ctx);

/* PAP probe (Sec. 3.2, Eq. (mha_importance); Alg. 1 PAP block, first two lines).
 * x [N, D]: hidden states before the layer.  Computes the post-rotary keys of all candidates
 * k_out [N, Hkv, d] and s_mha[n] = mean over the P*H probe rows of softmax(q k^T / sqrt(d))[n],
 * where probe row p is candidate N-P+p and sees candidates 0..N-P+p.  Needs 1 <= probe_len <= N. */
int spts_probe_attn(spts_ctx *ctx, const void *x, const int32_t *pos, int64_t N,
                    const spts_layer_weights *w, int32_t probe_len, void *k_out, float *s_mha);

/* LTP probe (Sec. 3.3, Eq. (proxy_ffn), (ffn_transformation), (ffn_importance)).
 * x [N, D]: residual stream after the attention update.  c_ffn[n] = || f(rmsnorm(x_n)) ||_2,
 * s_ffn[n] = c_ffn[n] * s_mha[n].  s_mha may be NULL (then s_ffn = c_ffn); c_ffn may be NULL. */
int spts_probe_ffn(spts_ctx *ctx, const void *x, int64_t N, const spts_layer_weights *w,
                   const float *s_mha, float *c_ffn, float *s_ffn);

/* TopK (Sec. 3.2; Eq. (ffn_selection)).  idx_out [k] ascending.  0 <= k <= N; k == 0 writes nothing. */
int spts_select_topk(spts_ctx *ctx, const float *scores, int64_t N, int64_t k, int32_t protect_last,
                     int32_t *idx_out);

/* spts_select_topk for callers that cannot allocate device memory and so cannot give a context its workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no context, no workspace.
 * Same selection and same output as spts_select_topk (bit-identical), always through the chip-wide radix select,
 * whose histogram tables (about 257 KB) live in a file-scope device array of the library: every GPU the library
 * runs on holds one copy until the process ends.  The call allocates nothing, frees nothing and calls no
 * allocating routine; its first use on a device looks the array's address up (hipGetSymbolAddress, no allocation).
 * hip_stream: hipStream_t as void* (NULL = default stream) on the current device; scores [N] and idx_out [k] are
 * device pointers, 16-byte aligned.  0 <= k <= N <= SPTS_TOPK_STATIC_MAX_N: a longer row is rejected with
 * SPTS_ESHAPE before anything is launched (SPTS_EINVAL / SPTS_EALIGN / SPTS_EHIP as for the other calls).
 * All calls on one GPU share that GPU's array: two calls must not overlap in time (issue them on one stream, or
 * order the streams), otherwise they race on the tables.  Nothing in the array has to be cleared between calls. */
#define SPTS_TOPK_STATIC_MAX_N 1048576
int spts_select_topk_static(void *hip_stream, const float *scores, int64_t N, int64_t k, int32_t protect_last,
                            int32_t *idx_out);

/* TopK over `batch` independent score rows (Sec. 3.2 TopK applied per sequence of a batch):
 * scores [batch, N] row-major, idx_out [batch, k], every row selected and ordered as by
 * spts_select_topk.  0 <= batch <= 65535, N <= the context's max_tokens (as for the single-row
 * call), 0 <= k <= N.  Device pointers, 16-byte aligned; the call uses no workspace. */
int spts_select_topk_batched(spts_ctx *ctx, const float *scores, int64_t N, int64_t k,
                             int32_t protect_last, int32_t batch, int32_t *idx_out);

/* TopK per sequence of a variable-length batch (Sec. 3.2 TopK on each sequence's scores): sequence b
 * owns scores[seg_offsets[b] .. seg_offsets[b+1]), keeps min(seg_k[b], its length) candidates and
 * writes their indices (local to the sequence, ascending) at idx_out + out_offsets[b].  The three
 * descriptor arrays are device int64 arrays ([batch+1], [batch], [batch]); max_len >= the longest
 * sequence (it selects the kernel variant; longer sequences than max_len are a caller error) and
 * max_len <= the context's max_tokens.  A sequence with budget <= 0 writes nothing. */
int spts_select_topk_segmented(spts_ctx *ctx, const float *scores, const int64_t *seg_offsets,
                               const int64_t *seg_k, const int64_t *out_offsets, int32_t batch,
                               int64_t max_len, int32_t protect_last, int32_t *idx_out);

/* One decoder layer of Alg. 1 in place on x [N, D] (PAP block then LTP block, or the dense
 * branches when cfg->skip == 0).  Optional outputs (NULL = not wanted): kv, s_mha [N],
 * idx_attn [min(N, m_attn)], idx_ffn [min(N, m_ffn)].  With skip == 0 the optional score/index
 * outputs are not written and kv receives all N rows. */
int spts_layer_prefill(spts_ctx *ctx, void *x, const int32_t *pos, int64_t N,
                       const spts_layer_weights *w, const spts_layer_cfg *cfg, spts_kv_out *kv,
                       float *s_mha, int32_t *idx_attn, int32_t *idx_ffn);

/* The same layer over a batch of sequences of different lengths (kv_mode 0: active-pair caches): x
 * [Ntot, D] and pos [Ntot] hold the sequences back to back, sequence b in rows
 * [seq_offsets[b], seq_offsets[b+1]).  seq_offsets [batch+1], m_attn [batch] and m_ffn [batch] are HOST
 * arrays (seq_offsets[0] = 0; budgets as in spts_layer_cfg, min(length, m) applies per sequence).  Every
 * sequence is probed with its own last probe_len rows, selects within itself (Eq. (mha_importance),
 * Eq. (ffn_importance) and TopK per sequence) and attends to itself only; the projections and the FFN
 * run over the rows of all sequences at once.  Every sequence needs at least probe_len rows
 * (SPTS_EINVAL otherwise); batch <= SPTS_MAX_BATCH.  skip == 0 runs the dense branches: no probe, no
 * selection, every row active (probe_len and the budgets are ignored, the score / index outputs are
 * not written, the caches receive every row).  Optional outputs: kv [batch] (one cache per
 * sequence, filled with its active pairs), s_mha [Ntot], idx_attn / idx_ffn: the active sets of the
 * sequences back to back, as ascending row numbers of the batch (sequence b's share starts at
 * sum over b' < b of min(len_b', m_b')).
 * Like every call, this one only enqueues work and returns: the host arrays are read before it returns (their
 * values reach the device as kernel arguments, not through a copy of host memory), so they may be freed at once,
 * and the call may be recorded under stream capture. */
#define SPTS_MAX_BATCH 1024
int spts_layer_prefill_batched(spts_ctx *ctx, void *x, const int32_t *pos, const int64_t *seq_offsets,
                               int32_t batch, const spts_layer_weights *w, int32_t skip,
                               int32_t probe_len, const int64_t *m_attn, const int64_t *m_ffn,
                               int32_t protect_last,
                               spts_kv_out *kv, float *s_mha, int32_t *idx_attn, int32_t *idx_ffn);

/* Decode phase of Alg. 1 for one new token (Is_prefill_phase() is false, so skip is false: standard
 * MHA with residual and cache update, standard FFN).  x [D] in/out: the token's hidden state.
 * The token's rotary key and its value are written to row cache->count of the cache (Sec. 3.2 last
 * paragraph and the appendix on KV-cache flexibility: the cache holds the prefill's active pairs plus
 * the decoded tokens), attention runs over rows [0, count], then cache->count is incremented on the
 * host.  `pos` is the token's absolute position (prefill length + decode step).  Needs
 * count < capacity, H / Hkv <= 8, d in {16, 32, 64, 128}, D, H*d, Hkv*d and Dff multiples of 4
 * (SPTS_ESHAPE otherwise).  Uses the context's workspace; device pointers, 16-byte aligned. */
int spts_decode_layer(spts_ctx *ctx, void *x, int32_t pos, const spts_layer_weights *w,
                      spts_kv_out *cache);

/* The decode step for a batch of sequences, one new token each (batch <= SPTS_MAX_DECODE_BATCH): x
 * [batch, D] in/out, pos [batch] HOST array of the tokens' absolute positions, caches [batch]: one
 * cache per sequence (distinct buffers), each appended to and attended over as in spts_decode_layer.
 * The projections and the FFN read the layer's weights once for the whole batch. */
#define SPTS_MAX_DECODE_BATCH 16
int spts_decode_layer_batched(spts_ctx *ctx, void *x, const int32_t *pos, int32_t batch,
                              const spts_layer_weights *w, spts_kv_out *caches);

/* Greedy next token after the last layer: RMSNorm with gamma_f [D], logits = table [V, D] applied
 * to the normed state (fp32), token = argmax with ties to the lowest id.  The vocabulary table is a
 * harness input (the method does not define one); it also serves as the embedding: x_next [D]
 * receives table[token, :] when not NULL.  token_out: device int32.  logits_out [V] fp32 may be
 * NULL (then the workspace must hold V floats: SPTS_EWORKSPACE otherwise).  V % 4 == 0. */
int spts_greedy_token(spts_ctx *ctx, const void *x, const void *gamma_f, const void *table,
                      int32_t V, int32_t *token_out, float *logits_out, void *x_next);

/* spts_greedy_token for a batch of states x [batch, D] (batch <= SPTS_MAX_DECODE_BATCH): the
 * vocabulary table is read once.  token_out [batch]; logits_out [batch, V] or NULL (the workspace must
 * then hold batch * V floats); x_next [batch, D] or NULL. */
int spts_greedy_token_batched(spts_ctx *ctx, const void *x, const void *gamma_f, const void *table,
                              int32_t V, int32_t batch, int32_t *token_out, float *logits_out,
                              void *x_next);

/* Offline proxy construction, channel scores (Sec. 3.3: activation saliency and
 * Eq. (channel_importance)).  x_cal [T, D]: calibration tokens as the FFN sees them (states after
 * the pre-FFN RMSNorm).  importance_out [Dff] fp32: for every FFN channel the mean of the k
 * largest |silu(x Wgate) * (x Wup)| over the T tokens (k = rho * T in the paper).  The Dlow
 * channels to keep are spts_select_topk(importance_out, Dff, Dlow, 0).  1 <= k <= T <= max_tokens;
 * uses w->Wgate, w->Wup only; device pointers, 16-byte aligned. */
int spts_channel_importance(spts_ctx *ctx, const void *x_cal, int64_t T, const spts_layer_weights *w,
                            int64_t k, float *importance_out);

/* Stage-end pruning (Sec. 3.4, Eq. (stage_prune); Alg. 1 last block): keeps the
 * N' = min(N, N_next) candidates with the largest s_mha.  Out of place: x_out [N', D],
 * pos_out [N'], map_new2old [N'] (ascending), map_old2new [N] (-1 for dropped rows; may be NULL).
 * x_out must not overlap x_in. */
int spts_msdp_compact(spts_ctx *ctx, const void *x_in, const int32_t *pos_in, const float *s_mha,
                      int64_t N, int64_t N_next, int32_t protect_last, void *x_out, int32_t *pos_out,
                      int32_t *map_new2old, int32_t *map_old2new);

/* Stage-end pruning of a batch of sequences laid back to back (layout as in
 * spts_layer_prefill_batched; seq_offsets [batch+1] and n_next [batch] are HOST arrays): every sequence
 * keeps its own min(length, n_next[b]) candidates with the largest s_mha.  The kept rows of the
 * sequences follow each other in x_out / pos_out; the new offsets are the prefix sums of the kept
 * counts (the caller computes them on the host).  map_new2old [sum kept] and map_old2new [Ntot]
 * (-1 for dropped rows; may be NULL) are rows of the batch.  x_out must not overlap x_in. */
int spts_msdp_compact_batched(spts_ctx *ctx, const void *x_in, const int32_t *pos_in, const float *s_mha,
                              const int64_t *seq_offsets, int32_t batch, const int64_t *n_next,
                              int32_t protect_last, void *x_out, int32_t *pos_out,
                              int32_t *map_new2old, int32_t *map_old2new);

/* Per-phase timing for benchmarks.  Between spts_profile_begin and spts_profile_end every phase of
 * every call on this context (k_proj, probe_attn, topk, attention, ffn_gate_up, ...) is bracketed
 * by two HIP events on the context's stream.  spts_profile_end synchronises the stream (the only
 * call of this library that does) and accumulates the elapsed milliseconds and the number of
 * bracketed launches per phase; spts_profile_get reads phase i in [0, spts_profile_count). */
int spts_profile_begin(spts_ctx *ctx);
int spts_profile_end(spts_ctx *ctx);
int spts_profile_count(const spts_ctx *ctx);
int spts_profile_get(const spts_ctx *ctx, int i, const char **name, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* SPTS_H */
