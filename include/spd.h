/*
 * libspd -- Superposed Decoding (arXiv 2405.18400) hot path for AMD MI355X (gfx950).
 *
 * One SPD timestep (Section 3; Algorithm 1, else-branch), entirely on the GPU:
 *   superposition weights (Section 3.1, Eq. 2) -> superposed input embedding (Eq. 1) ->
 *   batch-1 decoder forward over one shared key/value cache (Section 3, "Next Timesteps")
 *   -> full-vocabulary log-softmax with temperature and KeepTopK (Algorithm 1) ->
 *   k x k draft options -> n-gram mixture (Section 3.2, Eq. 3) -> interpolation (Eq. 4)
 *   or the no-overlap penalty form (Eq. 5) -> keep the k most probable options and update
 *   their probabilities (Section 3, Eq. for D and P).
 * Around it: the pass over the prefix (Section 3, "First Timestep"; spd_prefill), one pass of
 * nucleus sampling on the same forward (the comparison decoder of Section 4.3;
 * spd_nucleus_step), and committing one draft to restart from it (resets, Section 5.3; a
 * nucleus-sampled opening in front of Superposed Decoding, Section 4.5; spd_commit).
 *
 * Conventions
 *   - Every function returns SPD_OK (0) or a negative spd_status.  No exceptions, no global
 *     state.  spd_last_error() gives a human-readable reason for the last failure on a ctx.
 *   - "device" pointers are HIP device memory owned by the CALLER (the library never
 *     allocates or frees device memory); "host" pointers are ordinary host memory.
 *   - All GPU work is enqueued on the hipStream_t given to spd_create (passed as void*;
 *     NULL = the default stream).  A call that fills host outputs synchronises that stream
 *     before returning; a call with no host outputs does not synchronise.
 *   - Scores cross this boundary as natural-log probabilities.
 *   - Matrices are row-major [out_features, in_features], contiguous, 16-byte aligned,
 *     stored in cfg.dtype (fp32, or bf16 bit patterns).  Norm gains use the same dtype.
 *   - One ctx serves one generation at a time; calls on one ctx must not overlap.
 */
#ifndef SPD_H
#define SPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPD_K_MAX 16      /* compile-time ceiling on the number of drafts k            */
#define SPD_MIN_ORDER 2   /* n-gram orders n = 2..6 (Section 3.2)                      */
#define SPD_MAX_ORDER 6
#define SPD_N_ORDERS 5
#define SPD_TAIL 5        /* tokens of history an order-6 context needs                */

typedef enum {
    SPD_OK = 0,
    SPD_EINVAL = -1,        /* bad argument (null pointer, shape, alignment, range)      */
    SPD_ESTATE = -2,        /* call out of order (e.g. step before prefill)              */
    SPD_ECTX_OVERFLOW = -3, /* the key/value cache would exceed cfg.max_ctx              */
    SPD_EWORKSPACE = -4,    /* workspace / table buffer too small or misaligned          */
    SPD_ETABLE = -5,        /* n-gram table rejected (duplicate key, id >= vocab, ...)   */
    SPD_EHIP = -6           /* a HIP runtime call failed                                 */
} spd_status;

typedef enum { SPD_DTYPE_FP32 = 0, SPD_DTYPE_BF16 = 1, SPD_DTYPE_FP16 = 2 /* key/value cache only */ } spd_dtype;

/* Decoder-only transformer f_theta: RMSNorm, rotary on adjacent pairs (x_2i, x_2i+1) with
 * angle pos * rope_theta^(-2i/d_head), causal attention scaled by 1/sqrt(d_head), SwiGLU
 * feed-forward, untied embedding / LM head, no biases.  d_head = d_model / n_heads. */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab;
    int32_t max_ctx;   /* key/value cache capacity in positions (prefix + generated)        */
    int32_t k_max;     /* largest k any spd_step will use, 1..SPD_K_MAX                     */
    int32_t dtype;     /* spd_dtype of the weights: SPD_DTYPE_FP32 or SPD_DTYPE_BF16        */
    float rms_eps, rope_theta;
    int32_t kv_dtype;  /* element type of the key/value cache: SPD_DTYPE_FP32 (0, the default: every
                        * cached key and value keeps the fp32 result of its projection) or, with
                        * bf16 weights only, SPD_DTYPE_FP16 (rounded to nearest even on the way in:
                        * half the cache bytes per step and per position; adds about 3e-3 of the
                        * logit scale over 32 layers, within the 2e-2 of a bf16 model's rounding) */
} spd_model_cfg;

typedef struct {
    const void *attn_norm; /* [d_model]                                                    */
    const void *wqkv;      /* [(n_heads + 2 n_kv_heads) d_head, d_model]: q rows, k, v      */
    const void *wo;        /* [d_model, n_heads d_head]                                     */
    const void *ffn_norm;  /* [d_model]                                                    */
    const void *w_gate;    /* [d_ffn, d_model]                                              */
    const void *w_up;      /* [d_ffn, d_model]                                              */
    const void *w_down;    /* [d_model, d_ffn]                                              */
} spd_layer_weights;

/* Borrowed device pointers; they must stay valid until spd_destroy. `layers` is a HOST
 * array of n_layers structs (copied by spd_create). */
typedef struct {
    const void *embed;      /* [vocab, d_model] token embeddings z (Section 3.1)            */
    const spd_layer_weights *layers;
    const void *final_norm; /* [d_model]                                                   */
    const void *lm_head;    /* [vocab, d_model]                                             */
} spd_weight_ptrs;

/* N-gram frequency tables (Section 4: every unique n-gram with its count), HOST memory.
 * Order n uses index n-2.  keys[n-2] is int32 [n_entries[n-2], n] row-major (oldest token
 * first, predicted token last); counts[n-2] is uint32 [n_entries[n-2]].  An order may be
 * empty (n_entries 0, pointers may be NULL).  lambda[n-2] is that order's mixture weight
 * (Eq. 3); the paper's values are 0.01, 0.04, 0.15, 0.18, 0.12 (Appendix B). */
typedef struct {
    const int32_t *keys[SPD_N_ORDERS];
    const uint32_t *counts[SPD_N_ORDERS];
    int64_t n_entries[SPD_N_ORDERS];
    float lambda[SPD_N_ORDERS];
} spd_ngram_host_tables;

/* Per-call decoding parameters (Appendix B): number of drafts k, interpolation weight
 * alpha in [0,1] (0 = n-gram smoothing disabled), temperature tau > 0 applied to the logits
 * of the full-vocabulary softmax, no-overlap penalty delta > 0 (Eq. 5). */
typedef struct {
    int32_t k;
    float alpha, tau, delta;
} spd_decode_cfg;

typedef struct spd_ctx spd_ctx;

/* Bytes of device workspace spd_create needs for this shape (KV cache, activations,
 * attention partials, draft state, token history). Host-only; touches no GPU. */
int spd_workspace_bytes(const spd_model_cfg *cfg, size_t *out_bytes);

/* Create a decoding context.  `workspace` is caller-owned DEVICE memory of at least
 * spd_workspace_bytes() bytes, 256-byte aligned, untouched by the caller until
 * spd_destroy.  `hip_stream` is a hipStream_t (or NULL).  Validates shapes and alignment
 * before any GPU work.  *out is set only on success and is freed by spd_destroy. */
int spd_create(const spd_model_cfg *cfg, const spd_weight_ptrs *weights, void *workspace,
               size_t workspace_bytes, void *hip_stream, spd_ctx **out);
void spd_destroy(spd_ctx *ctx);

/* Bytes of DEVICE memory spd_load_ngrams needs for these tables (exact-key hash table of
 * all n-grams plus one context-total entry per distinct context).  Host-only. */
int spd_ngram_table_bytes(const spd_ngram_host_tables *tables, size_t *out_bytes);

/* Build the device-resident n-gram store (Section 3.2; the paper keeps these in host
 * dictionaries, Section 4.3) in `dev_buf` (caller-owned DEVICE memory, 256-byte aligned,
 * kept alive while in use) and attach it to ctx.  Rejects (SPD_ETABLE) a duplicate key, a
 * token id outside [0, vocab) or a zero count.  May be called again at any time outside a
 * step to swap tables.  Synchronises the stream.  Without tables only alpha = 0 is legal. */
int spd_load_ngrams(spd_ctx *ctx, const spd_ngram_host_tables *tables, void *dev_buf,
                    size_t dev_bytes);

/* First-timestep forward (Section 3, "First Timestep"): reset the generation, run the
 * model over prefix[0..m-1] (HOST int32 ids in [0, vocab), 1 <= m < max_ctx), fill cache
 * positions 0..m-1 and keep the last position's logits.  Does not synchronise. */
int spd_prefill(spd_ctx *ctx, const int32_t *prefix, int32_t m);

/* Advance every draft by one token.  The first call after spd_prefill gives draft i the
 * i-th most probable token of p_theta(. | M) with that token's log-probability as its
 * score (no n-gram term); later calls run one full SPD timestep.  dc->k must stay the same
 * between a prefill and the end of its generation.  Outputs are HOST arrays of k entries,
 * best draft first, each may be NULL: the newest token of each surviving draft, the index
 * (0..k-1, in the previous step's order; -1 at the first step) of the draft it extends,
 * and its log-score.  If all three are NULL the call does not synchronise. */
int spd_step(spd_ctx *ctx, const spd_decode_cfg *dc, int32_t *out_last_tokens,
             int32_t *out_parents, float *out_logscores);

/* Algorithm 1 end to end: spd_prefill + n_tokens spd_steps, then rebuild the drafts from
 * the per-step parent indices.  out_drafts is HOST int32 [k, n_tokens] row-major, best
 * draft first; out_logscores HOST float [k].  Synchronises. */
int spd_generate(spd_ctx *ctx, const int32_t *prefix, int32_t m, const spd_decode_cfg *dc,
                 int32_t n_tokens, int32_t *out_drafts, float *out_logscores);

/* ---- state access: resets (Section 5.3) and step-by-step comparison with a reference ---- */

/* Read the k drafts' bookkeeping (HOST outputs, any may be NULL): tails int32 [k, SPD_TAIL]
 * = the last 5 tokens of (prefix, draft), oldest first, -1 where the history is shorter;
 * logscores float [k]; gamma float [k] = the superposition weights (Eq. 2) of the current
 * scores.  Synchronises. */
int spd_get_state(spd_ctx *ctx, int32_t *out_k, int32_t *out_tails, float *out_logscores,
                  float *out_gamma);
/* Overwrite the drafts' bookkeeping (HOST inputs) between steps; the KV cache is untouched.
 * Legal once the first step after a prefill has run.  Synchronises. */
int spd_set_state(spd_ctx *ctx, int32_t k, const int32_t *tails, const float *logscores);
/* Copy the logits [vocab] of the most recent forward pass to HOST memory.  Synchronises. */
int spd_read_logits(spd_ctx *ctx, float *out_logits);

/* What the most recent step decided (HOST outputs, any may be NULL): the kept token ids
 * int32 [k] and their log p_theta float [k] (Algorithm 1, KeepTopK); for each option
 * (i, j) = draft i + kept token j, row-major [k, k]: its score log p_i + log p_f (float),
 * whether it was an option at all (int32 0/1; options outside the overlap set are not,
 * Section 3.2) and the n-gram mixture value p_ngram (float, Eq. 3).  Synchronises. */
int spd_get_step_info(spd_ctx *ctx, int32_t *out_top_ids, float *out_top_logp,
                      float *out_cand_scores, int32_t *out_cand_valid, float *out_cand_pngram);

/* Run only the post-forward part of a timestep (KeepTopK, expansion, n-gram probes,
 * interpolation, prune, state update) on caller-supplied DEVICE logits float [vocab], as
 * if the forward pass had produced them.  `first` != 0 performs the first-timestep
 * initialisation instead.  Requires a prior spd_prefill (it provides the history).  Does
 * not touch the KV cache or the position.  Does not synchronise. */
int spd_expand_prune(spd_ctx *ctx, const spd_decode_cfg *dc, const float *dev_logits, int32_t first);

/* Commit one draft and restart (Section 5.3, "Superposed Decoding Resets": every s timesteps
 * one of the k drafts is sampled and draft generation restarts; Section 4.5: a nucleus-sampled
 * generation of any length serves as the prefix of a Superposed Decoding run).
 * Draft i is sampled with its superposition weight gamma_i (Eq. 2) by inverse CDF over the
 * drafts in rank order with the caller's draw u in [0, 1); its tokens since the last
 * spd_prefill / spd_commit are appended to the text, the cache positions they occupy are
 * recomputed from the tokens themselves (with one draft, k = 1, only the newest token's), and
 * the context is left as after spd_prefill of the extended text: the next spd_step (any k) or
 * spd_nucleus_step starts a generation from it.  Outputs are HOST, each may be NULL: the
 * sampled draft's index, its tokens (cap entries available) and their number.  Synchronises. */
int spd_commit(spd_ctx *ctx, float u, int32_t *out_chosen, int32_t *out_tokens, int32_t cap, int32_t *out_n);

/* ---- the comparison decoder: one pass of nucleus (top-p) sampling ----
 * Section 4.3 times Superposed Decoding against k independent passes of nucleus sampling;
 * Section 2 describes the sampler: the next-token distribution is cut to the smallest set of
 * most probable tokens whose cumulative probability reaches top_p and renormalised.  Here:
 * probabilities are the full-vocabulary softmax of logits / tau; tokens are ordered by
 * probability, the lower id first among equals; the nucleus is the shortest prefix of that
 * order whose mass reaches top_p; the draw u in [0, 1) (supplied by the caller, who owns the
 * random number generator) selects the first token whose cumulative probability in that
 * order exceeds u times the nucleus mass. */
typedef struct spd_sample_cfg {
    float top_p; /* in (0, 1] */
    float tau;   /* > 0 */
} spd_sample_cfg;

/* One token of one pass.  The first call after spd_prefill samples from the prefix pass's
 * logits; every later call feeds the previously sampled token's embedding through the
 * transformer (one more cached position) and samples from the new logits.  out_token /
 * out_logprob: HOST, may be NULL (then the call does not synchronise); the log-probability
 * is that of the sampled token under the full-vocabulary softmax.  A pass and an SPD
 * generation with k > 1 cannot be interleaved on one context (SPD_ESTATE); spd_prefill
 * starts either. */
int spd_nucleus_step(spd_ctx *ctx, const spd_sample_cfg *sc, float u, int32_t *out_token, float *out_logprob);

/* Run only the sampler (not the transformer) on caller-supplied DEVICE logits float [vocab],
 * as if the forward pass had produced them; `first` != 0 starts a pass (as the first
 * spd_nucleus_step after spd_prefill does).  Does not touch the KV cache or the position.
 * Does not synchronise; read the result with spd_get_state / spd_get_nucleus_info. */
int spd_nucleus_sample(spd_ctx *ctx, const spd_sample_cfg *sc, float u, const float *dev_logits, int32_t first);

/* Size and probability mass of the nucleus of the most recent sampling call, and the sum
 * of the log-probabilities of the tokens sampled so far in this pass.  HOST outputs, any may
 * be NULL.  Synchronises. */
int spd_get_nucleus_info(spd_ctx *ctx, int32_t *out_size, float *out_mass, float *out_sum_logprob);

/* Current position (= number of cached positions) as tracked by the host. */
int spd_position(const spd_ctx *ctx, int32_t *out_pos);

/* Turn the captured-graph replay of spd_step on (default) or off (plain launches). */
int spd_set_graph(spd_ctx *ctx, int32_t enable);

/* The transformer forward of a timestep runs either as one persistent kernel ("fused": the
 * default wherever an instantiation exists for the model shape) or as one kernel per
 * matrix-vector product.  Both compute the same thing; spd_set_fused switches between them
 * (SPD_EINVAL when asked for a fused kernel the shape has none for), spd_get_fused tells
 * which one runs. */
int spd_set_fused(spd_ctx *ctx, int32_t enable);
int spd_get_fused(const spd_ctx *ctx, int32_t *out_enabled);

/* spd_prefill runs the prefix either one token at a time through the timestep's forward, or
 * ("dense": the default for bf16 models whose widths allow it, for prefixes of 8 tokens or
 * more; spd_commit uses the same pass) up to 1024 prefix tokens at a time as matrix-matrix
 * products on the matrix cores, reading the weights once per chunk.  Both fill the same cache
 * and leave the same logits up to fp32 rounding.  A dense pass exists for bf16 weights,
 * d_head <= 128, d_model <= 8192 and d_model, d_ffn, n_heads * d_head divisible by 128; it adds
 * 1024 rows of activations to spd_workspace_bytes.  spd_set_dense_prefill switches (SPD_EINVAL
 * when asked for a dense pass the model has none for). */
int spd_set_dense_prefill(spd_ctx *ctx, int32_t enable);
int spd_get_dense_prefill(const spd_ctx *ctx, int32_t *out_enabled);

/* Per-kernel timing for profiling runs: when enabled, spd_step launches kernels one by one
 * with a HIP event pair around each and accumulates the elapsed time per kernel class.
 * spd_get_kernel_timing fills HOST arrays of up to `cap` entries (class name pointers valid
 * for the ctx lifetime, total milliseconds, launch counts), sets *out_n, and synchronises. */
int spd_set_kernel_timing(spd_ctx *ctx, int32_t enable);
int spd_get_kernel_timing(spd_ctx *ctx, int32_t cap, const char **out_names, float *out_ms,
                          int64_t *out_launches, int32_t *out_n);

/* While kernel timing is on, every block of the fused forward kernel records a 100 MHz clock
 * stamp before and after each of its device-wide barriers (and at its end):
 * stamp[2i] = arrival at barrier i, stamp[2i+1] = release, i = 0 .. 5 n_layers (barrier 0
 * follows the input phase; each layer then has QKV, attention, O, gate/up, down).  Copies the
 * stamps of the most recent fused forward to HOST memory as [*out_blocks][*out_n] (the first
 * 512 blocks at most) with
 * *out_n = 2 (5 n_layers + 2); `cap` counts int64 elements of out_stamps.  SPD_ESTATE when
 * the model shape has no fused kernel. */
int spd_get_phase_clock(spd_ctx *ctx, int32_t cap, int64_t *out_stamps, int32_t *out_n,
                        int32_t *out_blocks);

/* ---- stand-alone operators (the kernels of one timestep, callable one at a time) ---- */

/* y = W x (+ residual), optionally with x first RMS-normalised (x * rsqrt(mean x^2 + eps) *
 * gain).  W is DEVICE [rows, cols] in `dtype`; x, residual, y are DEVICE float; gain is
 * DEVICE [cols] in `dtype` or NULL (no normalisation); residual may be NULL or equal y. */
int spd_op_gemv(int32_t dtype, const void *W, const void *gain, float eps, const float *x,
                const float *residual, float *y, int32_t rows, int32_t cols, void *hip_stream);
/* u = silu(Wg xn) * (Wu xn) with xn = RMS-normalised x (gain may be NULL: xn = x). */
int spd_op_swiglu(int32_t dtype, const void *Wg, const void *Wu, const void *gain, float eps,
                  const float *x, float *u, int32_t rows, int32_t cols, void *hip_stream);
/* Single-query attention over n_ctx cached positions: out[h] = softmax(q[h] . K / sqrt(d_head)) V
 * with K, V DEVICE [n_kv_heads, cap_ctx, d_head] in `dtype` (head-major, as the library's
 * cache, which is fp32 or fp16: SPD_DTYPE_FP16 is accepted here too), q and out DEVICE float
 * [n_heads, d_head]; `partials` is DEVICE scratch of spd_op_attention_scratch_bytes() bytes. */
size_t spd_op_attention_scratch_bytes(int32_t n_heads, int32_t d_head, int32_t cap_ctx);
int spd_op_attention(int32_t dtype, const float *q, const void *K, const void *V, float *out,
                     void *partials, int32_t n_heads, int32_t n_kv_heads, int32_t d_head,
                     int32_t n_ctx, int32_t cap_ctx, void *hip_stream);

/* spd_op_attention for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same computation with
 * the scratch in a static device array of SPD_STATIC_SCRATCH_BYTES inside the library instead
 * of a caller-supplied buffer.  The call allocates nothing.  Shapes whose
 * spd_op_attention_scratch_bytes(n_heads, d_head, cap_ctx) exceeds SPD_STATIC_SCRATCH_BYTES are
 * refused with SPD_EWORKSPACE before any GPU work.  Each GPU holds one such array for the life
 * of the process and every call on that GPU uses it: calls on one stream are ordered (each
 * clears the counters it needs with a fill kernel), calls that overlap on one GPU (other
 * streams, other threads) race and must be serialised by the caller.  Does not synchronise. */
#define SPD_STATIC_SCRATCH_BYTES (4u << 20)
int spd_op_attention_static(int32_t dtype, const float *q, const void *K, const void *V, float *out,
                            int32_t n_heads, int32_t n_kv_heads, int32_t d_head, int32_t n_ctx,
                            int32_t cap_ctx, void *hip_stream);

/* ---- test hooks for the error path of the persistent kernel's bounded waits ----
 * A wait of the persistent forward kernel that gives up (its grid was not co-resident) sets an
 * error word in the device-side draft state; every entry point that copies that state back
 * (spd_step, spd_generate, spd_commit, spd_nucleus_step, spd_get_state, spd_get_step_info,
 * spd_get_nucleus_info) then returns SPD_EHIP.  spd_test_state_layout gives the size of that
 * state in 32-bit words and the index of the error word; spd_test_state_status applies the
 * library's check to a HOST copy of the state filled by the caller (host only, no GPU);
 * spd_test_poke_err writes the device-side error word (a fill kernel on the ctx's stream, no
 * synchronisation) so that the getters' mapping can be seen without any wait ever failing:
 * spd_prefill clears it again. */
int spd_test_state_layout(size_t *out_words, size_t *out_err_word);
int spd_test_state_status(const int32_t *state_words, size_t n_words);
int spd_test_poke_err(spd_ctx *ctx, int32_t value);

const char *spd_last_error(const spd_ctx *ctx);
const char *spd_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPD_H */
