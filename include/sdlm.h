/*
 * sdlm.h - C ABI of the MI355X (gfx950) block-decode library for SDLM's Next
 * Sequence Prediction inference ("Sequential Diffusion Language Models").
 *
 * The library computes, entirely in hand-written HIP kernels, one decode step of
 * Longest Prefix Decoding (Sec. 3.2 and 3.4 of the paper):
 *
 *   - the block input X_T = [x_last, [m] x (D-1)] is appended after the cached
 *     prefix (block definition below the training objective, Sec. 3.2; Fig. 2(b));
 *   - a dense Qwen-2.5-shaped decoder (Sec. 4.1) runs on the block rows, which
 *     attend causally to the cache and bidirectionally inside the block (the
 *     attention-mask equation of Sec. 3.3, its operator read as OR);
 *   - per block position the arg-max token and its confidence are computed:
 *     softmax probability of the decoded token (Sec. 3.4 item (1)) or one minus
 *     the normalised entropy (Sec. 3.4 item (2));
 *   - gamma_tau = max({ j in 1..D : prod_{k<=j} p_k >= tau } U {1}) tokens are
 *     accepted (the gamma_tau equation, Sec. 3.4) and Decode() takes exactly those
 *     (the Decode equation, Sec. 3.2);
 *   - the cache only ever receives K/V of real, accepted tokens computed under
 *     causal attention: the tokens accepted in step t are fed in step t+1 as
 *     "pending" causal rows whose K/V land directly in their cache slots, next
 *     to the D block rows whose K/V are used inside the step and then dropped.
 *     This keeps the step a function of the token history alone (Sec. 3.2).
 *
 * Conventions
 *   Pointers marked [dev] are device (HBM) addresses, [host] are host addresses.
 *   The caller owns every buffer it passes in; the library allocates nothing on
 *   the device: all of its memory is the single workspace handed to sdlm_create.
 *   All work is enqueued on the HIP stream given to sdlm_create; outputs are
 *   valid once the caller has synchronised that stream.  Unless noted, calls do
 *   not synchronise.  Every call returns 0 on success or a negative sdlm_status;
 *   nothing throws or aborts across this boundary; sdlm_last_error() gives text.
 *   A context is not thread-safe.
 */
#ifndef SDLM_H
#define SDLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sdlm_ctx sdlm_ctx; /* opaque */

typedef enum {
    SDLM_OK = 0,
    SDLM_EINVAL = -1,    /* bad argument or unsupported shape */
    SDLM_ECAPACITY = -2, /* sequence would outgrow max_seq_len, page pool or workspace too small */
    SDLM_ESTATE = -3,    /* call out of order (commit without step, step without prefill, ...) */
    SDLM_EHIP = -4       /* a HIP runtime call failed */
} sdlm_status;

/* Shape of the decoder (Qwen-2.5 family: pre-norm RMSNorm, rotate-half RoPE, GQA, SwiGLU, untied LM head). */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rope_theta, rms_eps;
    float logit_scale;     /* logits = logit_scale * (x_hat . W_lm[v]) */
    int32_t dtype;         /* 0: fp32 weights, cache and arithmetic (debug / tiny); 1: bf16 weights and cache,
                              bf16 matrix-core inputs, fp32 accumulation, fp32 residual stream and softmax */
    int32_t mask_token_id; /* the id of [m]; its embedding is an ordinary row of the table */
    int32_t has_qkv_bias;
    int32_t block_causal;  /* 0: full mutual attention inside the block (the method, Sec. 3.3); 1: the ablation of
                              Sec. 4.4 "Causal Attention": block row k sees the block rows up to itself only */
} sdlm_model_cfg;

typedef struct {
    int32_t max_batch;   /* sequences decoded together, >= 1 */
    int32_t max_seq_len; /* most known tokens a sequence may reach; a step needs n_b + D <= max_seq_len, so that
                            accepting all D tokens still fits */
    int32_t block_D;     /* D: block size, 1..16 */
    int32_t kv_layout;   /* 0: contiguous (each sequence owns a fixed run of 16-token tiles sized for
                            max_seq_len); 1: paged (tiles handed out from a shared pool on demand) */
    int32_t page_size;   /* tokens per page; must be 16 */
    int32_t n_pages;     /* paged only: pages in the pool (per layer) */
    float tau;           /* acceptance threshold of gamma_tau */
    int32_t conf_fn;     /* 0: logit-value confidence; 1: entropy-normalised confidence */
    int32_t accept_rule; /* 0: cumulative product >= tau (the paper's rule); 1: each leading confidence >= tau */
    int32_t prefill_rows; /* rows per prefill pass (0: library default) */
} sdlm_run_cfg;

/*
 * Source weights, every matrix [out_features, in_features] row-major with in_features contiguous, element
 * type given by sdlm_model_cfg.dtype.  Per-layer entries are arrays of n_layers pointers.  A NULL entry in a
 * per-layer array (or a NULL global) leaves that tensor's packed copy untouched, so weights may be streamed in
 * over several calls.
 */
typedef struct {
    const void *embed, *lm_head, *final_norm; /* [V,h] [V,h] [h] */
    const void *const *attn_norm;             /* [h] */
    const void *const *wq, *const *wk, *const *wv; /* [Hq*d,h] [Hkv*d,h] [Hkv*d,h] */
    const void *const *wo;                    /* [h,Hq*d] */
    const void *const *bq, *const *bk, *const *bv; /* [Hq*d] [Hkv*d] [Hkv*d]; ignored unless has_qkv_bias */
    const void *const *ffn_norm;              /* [h] */
    const void *const *w_gate, *const *w_up;  /* [F,h] */
    const void *const *w_down;                /* [h,F] */
} sdlm_weights;

/* Bytes of device workspace a context with these settings needs (0 on invalid settings). */
size_t sdlm_workspace_bytes(const sdlm_model_cfg *m, const sdlm_run_cfg *r);

/*
 * Create a context inside `workspace` [dev] (256-byte aligned, at least sdlm_workspace_bytes()).  `hip_stream`
 * is a hipStream_t (NULL: the default stream).  Synchronises the stream once (tables are uploaded).
 * Errors: SDLM_EINVAL (shape not supported: head_dim not a multiple of 32 or > 256, n_q_heads not a multiple
 * of n_kv_heads, block_D outside 1..16, page_size != 16, ...), SDLM_ECAPACITY (workspace too small).
 */
int sdlm_create(const sdlm_model_cfg *m, const sdlm_run_cfg *r, void *workspace, size_t workspace_bytes,
                void *hip_stream, sdlm_ctx **out);

/*
 * Copy and repack weights into the workspace (matrix-core tile order for bf16).  The sources may be freed once
 * the stream has been synchronised.  on_device != 0: the pointers inside `w` are [dev]; 0: they are [host]
 * (staged through pageable copies; this synchronises).  `w` itself and its pointer arrays are [host].
 */
int sdlm_init_weights(sdlm_ctx *ctx, const sdlm_weights *w, int32_t on_device);

/*
 * Start `batch` sequences (1..max_batch) from their prompts and fill the cache with a causal forward over
 * each prompt (no block rows, no LM head).  ids_packed [host]: all prompts back to back; offsets [host]:
 * batch+1 entries, prompt b is ids_packed[offsets[b] .. offsets[b+1]).  Every prompt needs >= 1 token and
 * len + D <= max_seq_len.  Discards all earlier sequences.  Afterwards n_b = c_b = len_b.
 */
int sdlm_prefill(sdlm_ctx *ctx, int32_t batch, const int32_t *ids_packed, const int32_t *offsets);

/*
 * One block-decode step for every sequence.  Outputs, all [dev]:
 *   ids    [batch, D]  int32  arg-max token of each block position (lowest index on exact ties); the first
 *                             count[b] entries of row b are the accepted tokens (Decode), the rest are the
 *                             predictions that were not accepted;
 *   count  [batch]     int32  gamma_tau, 1..D;
 *   conf   [batch, D]  float  confidence per block position (may be NULL);
 *   logits [batch*D,V] float  the logits Z (may be NULL; costs a batch*D*V write).
 * The step publishes nothing: K/V of the pending tokens are written into cache slots that stay invisible
 * until sdlm_kv_commit, and the block rows' K/V live in per-step staging.  It may therefore be repeated.
 * Errors: SDLM_ESTATE before prefill; SDLM_ECAPACITY if n_b + D > max_seq_len for some sequence, i.e. if accepting
 * all D tokens would not fit (the host tracks an upper bound of each length and refreshes it with a stream
 * synchronisation only when the bound trips; the same refresh reports a page pool that ran out at the last commit).
 */
int sdlm_decode_step(sdlm_ctx *ctx, int32_t *ids, int32_t *count, float *conf, float *logits);

/*
 * sdlm_decode_step for callers that cannot allocate device memory for the step's partial results: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and errors as
 * sdlm_decode_step; the partial-result scratch of the step's kernels (split-k slabs of the projections, split-KV
 * partial results of the attention, per-vocabulary-block partials of the LM head; in fp32 mode the logits when
 * `logits` is NULL) lives in a 32 MiB array that is part of the library's code object instead of the workspace:
 * 16 MiB of slabs, 12 MiB of attention partials (both only bound how far the work is split, so a large model runs
 * with fewer splits) and 4 MiB for the LM head, which must hold batch x D rows: otherwise SDLM_ECAPACITY.  Calls
 * no hipMalloc / hipFree and creates no events or graphs (phase timing and graph replay do not apply to it).
 * Every GPU the library runs on holds one copy of the array until the process ends, and every context on that GPU
 * shares it: calls that overlap on one GPU (other streams, other contexts) race; calls in stream order do not, and
 * nothing in the array needs to start at zero (every partial result is written before it is read).  The device
 * current at sdlm_create is the one whose copy is used.  SDLM_EHIP if the array's address could not be obtained.
 */
int sdlm_decode_step_static(sdlm_ctx *ctx, int32_t *ids, int32_t *count, float *conf, float *logits);

/*
 * Replay the decode step as a HIP graph.  The launch sequence of sdlm_decode_step is fixed once the batch is known
 * (row counts, lengths and page tables live in device memory), so with enable != 0 the first sdlm_decode_step after
 * a prefill, or after the output pointers change, captures its launches on the context's stream and later calls
 * replay the captured graph: one submission instead of ~9 launches per layer, which is what bounds the step for small
 * batches.  Results are identical to the eager path.  The step runs eagerly regardless while any phase is being
 * timed (sdlm_profile) or a debug tap is set.  sdlm_verify_step and sdlm_kv_commit are always eager.
 * Errors: SDLM_ESTATE if the context was created on the null stream (which cannot be captured).
 */
int sdlm_graph(sdlm_ctx *ctx, int32_t enable);

/*
 * Second pass of a self-speculative step (Sec. 3.4, "Self-Speculative Decoding", Eq. 10); call it between
 * sdlm_decode_step, whose D arg-max tokens are the speculative tokens yhat^1..yhat^D, and sdlm_kv_commit.
 * Verification input j (j = 2..D) is the sequence extended by yhat^1..yhat^{j-1} followed by the mask tokens, i.e.
 * the input of an ordinary block step on that longer sequence; ytilde^j is the token that step would predict first
 * (input 1 is the first pass itself, so ytilde^1 = yhat^1).  All D-1 inputs of all sequences run as one batch of
 * rows through the same kernels as the step; they read the cache and write nothing to it.
 *   rule       0: gamma_verify = length of the longest prefix on which yhat and ytilde agree (at least 1);
 *              1: the equation as printed: the largest j with yhat^j == ytilde^j (at least 1).
 *   ids_tilde  [dev, batch x D] ytilde, or NULL.
 *   count      [dev, batch] gamma_verify, or NULL.  It also replaces the step's own count, so that a commit
 *              without overrides publishes yhat^1..yhat^{gamma_verify}.
 *   logits     [dev, batch x (D-1) x vocab] fp32 logits from which ytilde^2..ytilde^D were taken, or NULL.
 * Asynchronous on the context's stream.  Errors: SDLM_ESTATE without a preceding step, SDLM_EINVAL for an unknown
 * rule.  Every block size 1..16 is served; a sequence contributes (D-2) + (D-1) D rows to the pass (the causal rows
 * of the speculative tokens are shared by all inputs).
 */
int sdlm_verify_step(sdlm_ctx *ctx, int32_t rule, int32_t *ids_tilde, int32_t *count, float *logits);

/*
 * Publish the last step: the pending tokens' K/V become part of the cache (c_b = n_b) and the accepted tokens
 * become the next step's pending tokens (n_b += count_b); in the paged layout the page table grows to back
 * every position < n_b.  With both arguments NULL the step's own result is committed.  With ids_override
 * [dev, batch x D] and count_override [dev, batch] (1 <= count <= D; out-of-range counts are clamped and
 * reported through sdlm_get_lengths' return code, as are override ids outside the vocabulary, which are replaced by 0) the caller's tokens are committed instead: this is how a
 * verifier or a teacher-forced test drives the cache.  Errors: SDLM_ESTATE without a preceding step.
 */
int sdlm_kv_commit(sdlm_ctx *ctx, const int32_t *ids_override, const int32_t *count_override);

/*
 * Copy the per-sequence lengths to n [dev, batch] and c [dev, batch] (either may be NULL), then synchronise
 * and refresh the host's bounds.  Returns SDLM_ECAPACITY if a device-side guard (page pool exhausted) or
 * SDLM_EINVAL if a clamped override count was seen since the last call.
 */
int sdlm_get_lengths(sdlm_ctx *ctx, int32_t *n, int32_t *c);

/*
 * Debug taps.  The next sdlm_decode_step copies the named intermediate of layer `layer` into dst [dev]:
 *   0: residual stream entering the layer            float [R, hidden]
 *   1: attention output (before the O projection)    elem  [R, Hq*d]
 *   2: SwiGLU activation (input of the down proj.)   elem  [R, ffn]
 *   3: residual stream leaving the layer             float [R, hidden]
 *   4: normalised block rows entering the LM head    elem  [batch*D, hidden]   (layer ignored)
 *   5: rotated queries                               elem  [R, Hq*d]
 *   6: residual stream after the O projection        float [R, hidden]
 * "elem" is float in fp32 mode and bf16 in bf16 mode.  R is the step's packed row count: per sequence its
 * pending rows then its D block rows.  `which` < 0 clears all taps.  dst must hold max_rows rows.
 */
int sdlm_debug_tap(sdlm_ctx *ctx, int32_t layer, int32_t which, void *dst);

/*
 * Copy the packed row description of the last step: tok, pos, seq, kind [dev, max_rows each] (kind: -1 for a
 * pending row, else the block index 0..D-1) and n_rows [dev, 1].  Any pointer may be NULL.
 */
int sdlm_debug_rows(sdlm_ctx *ctx, int32_t *tok, int32_t *pos, int32_t *seq, int32_t *kind, int32_t *n_rows);

/*
 * Read cached K and V vectors of one (layer, sequence, kv head) for positions [pos0, pos0+count) into
 * k_out, v_out [dev, count x head_dim] as float.  Positions must be < n_b.  pos0 = -1 reads instead the first
 * `count` (<= D) entries of the sequence's staging tile: the K/V of the last step's block rows at that layer.
 */
int sdlm_debug_read_kv(sdlm_ctx *ctx, int32_t layer, int32_t seq, int32_t kv_head, int32_t pos0, int32_t count,
                       float *k_out, float *v_out);

/*
 * Host logic only (no GPU work): the launch shape the bf16 matrix-core GEMM takes for `rows` launch rows of which
 * `min_rows` certainly exist (0: unknown), an [n, k] weight matrix (k a multiple of 64) and an epilogue (0: plain fp32
 * store, 1: residual add, 2: SiLU(gate)*up, 3: LM head).  Outputs: rows and columns of a workgroup's tile (512 columns:
 * a workgroup of eight wavefronts, else four) and the number of splits along k.  For tests of the tile policy.  Errors: SDLM_EINVAL.
 */
int sdlm_debug_gemm_plan(int32_t epilogue, int32_t rows, int32_t min_rows, int32_t n, int32_t k, int32_t *tile_rows, int32_t *tile_cols,
                         int32_t *splits);

/* Rows the activation buffers are sized for (decode: batch * 2D; prefill pass size). */
int32_t sdlm_max_rows(const sdlm_ctx *ctx);

/*
 * Per-phase GPU time.  sdlm_profile(ctx, mask) makes every later step bracket each phase p whose bit (1 << p) is
 * set in `mask` with HIP events on the context's stream (-1: all phases, 0: none); sdlm_profile_read
 * synchronises, adds up the events recorded since the last read and
 * returns, for phase p in 0..SDLM_N_PHASES-1, total milliseconds in ms[p] and launches in launches[p] ([host]).
 */
enum { SDLM_PH_ROWS = 0, SDLM_PH_NORM, SDLM_PH_QKV, SDLM_PH_ROPE, SDLM_PH_ATTN, SDLM_PH_OPROJ, SDLM_PH_GATEUP,
       SDLM_PH_DOWN, SDLM_PH_LMHEAD, SDLM_PH_ACCEPT, SDLM_PH_ATTN_MERGE /* merge of the split-KV partials */, SDLM_N_PHASES };
int sdlm_profile(sdlm_ctx *ctx, int32_t mask);
/*
 * Sampling: bracket only every n-th launch of a selected phase (n >= 1, default 1), counted per phase from this call
 * on.  An event record between two kernels keeps them from running back to back, so timing every launch of a phase
 * that runs once per layer slows the step it measures; with n coprime to the layer count the samples rotate through
 * the layers.  sdlm_profile_read then reports the sampled launches only.  Errors: SDLM_EINVAL.
 */
int sdlm_profile_every(sdlm_ctx *ctx, int32_t n);
int sdlm_profile_read(sdlm_ctx *ctx, float *ms, int32_t *launches);

/* Which kernel family serves the GEMMs and the attention: "generic-fp32", "mfma-bf16", ... ([host] string). */
const char *sdlm_kernel_info(const sdlm_ctx *ctx);

const char *sdlm_last_error(const sdlm_ctx *ctx);
void sdlm_destroy(sdlm_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SDLM_H */
