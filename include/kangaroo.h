/*
 * libkangaroo — C ABI of the MI355X (gfx950) implementation of Kangaroo's batch-1
 * draft-and-verify decode loop (arXiv 2404.18911, "Kangaroo: Lossless Self-Speculative
 * Decoding via Double Early Exiting").
 *
 * Conventions for every call
 *   - "dev" pointers are device (HBM) addresses on the current HIP device; "host" pointers are
 *     ordinary host addresses.  The library never allocates or frees device memory: the caller
 *     owns the weight arena, the KV pool and the scratch area it binds, and the HIP stream.
 *   - Return value: KG_OK (0) or a negative kg_status.  kg_last_error() gives a message for the
 *     last failing call on that context.  A failing call leaves the sequence state unchanged,
 *     except after KG_EHIP (device error), after which the context must be reset.
 *   - A context is not thread-safe; calls on one context must not overlap.
 *   - Row counts per forward are limited to KG_MAX_ROWS (gamma + 1 <= 8).
 *
 * Call order:  kg_create -> kg_workspace_bytes -> kg_bind -> kg_load_tensor (all tensors)
 *              -> kg_prefill -> { kg_draft_step x (1..gamma) -> kg_verify -> kg_accept }*
 *              or kg_generate / kg_decode_plain, which run the whole loop.
 */
#ifndef KANGAROO_H
#define KANGAROO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KG_MAX_ROWS 8

typedef enum kg_status {
    KG_OK = 0,
    KG_EINVAL = -1, /* bad argument or configuration */
    KG_ESTATE = -2, /* call-order violation (e.g. verify before any draft step) */
    KG_ENOSPC = -3, /* the sequence would exceed max_seq, or a buffer is too small */
    KG_EHIP = -4,   /* a HIP runtime call failed; message holds the HIP error string */
    KG_ENOMEM = -5  /* host allocation failed */
} kg_status;

typedef struct kg_ctx kg_ctx; /* opaque */

/* Model and cache shape.  The target model M^b of Section 3 (Notation) is a LLaMA-style decoder
 * (Section 4.1 uses Vicuna): n_layers pre-norm blocks of RMSNorm, rotary multi-head attention,
 * SwiGLU feed-forward; exit_layer is the early-exit layer l of Section 3.1 (1 <= l <= n_layers). */
typedef struct kg_config {
    int n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int exit_layer;
    int dtype;          /* storage type of the weights: 0 = float32, 1 = bfloat16 */
    int kv_dtype;       /* storage type of the KV cache (rotated keys, values): 0 = float32, 1 = bfloat16,
                           2 = float16 (IEEE half); 1 and 2 need dtype = 1 */
    float rms_eps, rope_theta;
    int max_seq;        /* token capacity of the caches: prompt + generated + gamma_max + 1 */
    int gamma_max;      /* largest draft length gamma that will be used (<= KG_MAX_ROWS - 1) */
    int kv_page_tokens; /* tokens per KV page: a power of two in 16..128 */
    int adapter_kind;   /* architecture of the adapter A (Table 2), one of enum kg_adapter_kind; 0 = the paper's */
} kg_config;

/* The adapter architectures of Table 2's ablation.  Every one maps the early feature f to a hidden
 * state h that goes through the adapter's last RMSNorm and an LM head:
 *   KG_ADAPTER_ATTN       "Kangaroo": h = f + Wo.MHA(RMSNorm(f)); the target's LM head (67M at 7B)
 *   KG_ADAPTER_ATTN_HEAD  "Kangaroo + Head": the same, with an LM head of its own (198M)
 *   KG_ADAPTER_LAYER      "1-Layer Transformer": attention, then post norm and SwiGLU feed-forward
 *                         with their residuals, i.e. one more decoder block; the target's head (202M)
 *   KG_ADAPTER_MLP        "MLP Only": h = f + W2.silu(W1.RMSNorm(f)), two [d_model][d_model] maps,
 *                         no attention and no cache; own head (165M) */
typedef enum kg_adapter_kind {
    KG_ADAPTER_ATTN = 0, KG_ADAPTER_ATTN_HEAD = 1, KG_ADAPTER_LAYER = 2, KG_ADAPTER_MLP = 3
} kg_adapter_kind;

/* Tensors of the model.  Per-layer kinds take layer = 0..n_layers-1, the others layer = -1.
 * The adapter A of Section 3.1 / Figure 2 / Table 2 (row "Kangaroo") is one bias-free multi-head
 * attention (KG_A_WQ..KG_A_WO, each [d_model][d_model]) between two RMSNorm gain vectors, and
 * re-uses the target's LM head.  The kinds from KG_A_HEAD on belong to the other adapter
 * architectures of Table 2: a context takes exactly the adapter tensors its adapter_kind has
 * (loading another one is KG_EINVAL). */
typedef enum kg_tensor_kind {
    KG_EMBED = 0,       /* [vocab][d_model] */
    KG_LM_HEAD = 1,     /* [vocab][d_model] */
    KG_FINAL_NORM = 2,  /* [d_model] */
    KG_WQ = 3, KG_WK = 4, KG_WV = 5, KG_WO = 6, /* [d_model][d_model] */
    KG_WG = 7, KG_WU = 8,                        /* [d_ffn][d_model]   */
    KG_WD = 9,                                   /* [d_model][d_ffn]   */
    KG_NORM1 = 10, KG_NORM2 = 11,                /* [d_model] */
    KG_A_WQ = 12, KG_A_WK = 13, KG_A_WV = 14, KG_A_WO = 15,
    KG_A_NORM_IN = 16, KG_A_NORM_LAST = 17,
    KG_A_HEAD = 18,                              /* [vocab][d_model]: KG_ADAPTER_ATTN_HEAD, KG_ADAPTER_MLP */
    KG_A_NORM_POST = 19,                         /* [d_model]: KG_ADAPTER_LAYER */
    KG_A_WG = 20, KG_A_WU = 21,                  /* [d_ffn][d_model]: KG_ADAPTER_LAYER */
    KG_A_WD = 22,                                /* [d_model][d_ffn]: KG_ADAPTER_LAYER */
    KG_A_W1 = 23, KG_A_W2 = 24,                  /* [d_model][d_model]: KG_ADAPTER_MLP */
    KG_N_TENSOR_KINDS = 25
} kg_tensor_kind;

/* Decoding parameters.  gamma and eta are the maximum draft length and the confidence
 * threshold of Section 3.2 (the paper's setting: gamma = 6, eta = 0.6, Section 4.2); drafting
 * stops after a token whose top-1 probability is < eta (Eq. 4; eta = 0 gives fixed-step
 * drafting).  mode 0 accepts drafts while they equal the target's top-1 token; mode 1 is
 * speculative rejection sampling at the given temperature, which keeps the target's sampling
 * distribution.  Mode 1 uses one uniform number in [0,1) per (absolute token position, purpose):
 * purpose 0 draws the draft token of that position, 1 tests its acceptance, 2 draws a resampled /
 * bonus / first / plain token there.  With uniforms == NULL the kernels generate the number on the
 * device: Philox4x32-10 with key (seed mod 2^32, seed >> 32) and counter (position, purpose, 0, 0),
 * u = (first output word >> 8) * 2^-24; the stream of a request is then a function of (weights,
 * prompt, seed) alone, whatever the control flow.  With uniforms != NULL (host,
 * float[n_uniform_positions][3], indexed [position][purpose]) those numbers are used instead and
 * seed is ignored: a hook for tests that need to choose the numbers. */
typedef struct kg_params {
    int mode;
    float temperature;
    float eta;
    int gamma;
    const float *uniforms;
    int n_uniform_positions;
    uint64_t seed;
} kg_params;

/* Counters of one kg_generate / kg_decode_plain call.  s_hist[s] counts the rounds that emitted
 * s tokens (the list S of Section 3; compression rate, Eq. 1, is emitted_in_rounds / rounds).
 * bytes_*: algorithmic device traffic of the decode loop (Section 1: decoding is bound by reading the
 * weights): weight bytes streamed plus cached key / value bytes read, by what the forward belongs to:
 * draft = the self-draft model's steps (shallow layers, adapter, head), shallow = the shallow-only
 * passes (the stopped token's next early feature, Figure 2), verify = the remaining layers and the
 * head over the unit (or the whole model in plain decoding).  The prompt pass is not included.
 * There is no wall-clock for the shallow-only pass: it is launched ahead, inside the draft step, while
 * the host waits for that step's token, so its time is part of t_draft_s. */
typedef struct kg_stats {
    int rounds, drafted, accepted, emitted;
    int s_hist[KG_MAX_ROWS + 1];
    int draft_steps, verify_calls, plain_steps;
    double t_draft_s, t_verify_s, t_total_s; /* host wall-clock spent in each phase */
    double bytes_draft, bytes_shallow, bytes_verify;
} kg_stats;

/* Metrics of Section 3 from the counters of a run: compression rate CR = mean tokens emitted per
 * forward of the large model (Eq. 1), and the consistent token acceptance rate CTAR(w) = share of
 * rounds in which the first w drafts were all accepted, i.e. that emitted more than w tokens
 * (Eq. 2).  Both return KG_EINVAL for a run without rounds. */
int kg_stats_cr(const kg_stats *st, double *cr);
int kg_stats_ctar(const kg_stats *st, int w, double *ctar);

/* Create a context for a shape.  Host-only: no device is touched.  *out is NULL on failure. */
int kg_create(const kg_config *cfg, kg_ctx **out);

/* Bytes the caller must provide to kg_bind: the arena that will hold the re-tiled weights, the KV
 * pool (n_layers + 1 caches: one per decoder layer plus the adapter's), and scratch.
 * Layout of the KV pool, in elements of kv_dtype, row-major:
 *   [physical page][cache 0..n_layers][head][0 = keys, 1 = values][position in page][head_dim],
 * with ceil(max_seq / kv_page_tokens) pages; logical page i (positions i * kv_page_tokens ..) lives in
 * physical page perm[i] of kg_set_page_order (default i); keys are stored after the rotary embedding.
 * Between rounds (after kg_prefill or kg_accept, before the next kg_draft_step) only positions
 * below the committed length (kg_get_state: base; adapter_len for the adapter's cache) will ever be
 * read again: a caller may overwrite everything beyond them at that point. */
int kg_workspace_bytes(const kg_ctx *ctx, size_t *weight_bytes, size_t *kv_bytes, size_t *scratch_bytes);

/* Bind caller-owned device memory (256-byte aligned, at least the sizes above; all BORROWED until
 * kg_destroy) and the HIP stream (a hipStream_t, may be NULL for the default stream) every kernel
 * of this context is launched on.  Clears scratch and resets the sequence. */
int kg_bind(kg_ctx *ctx, void *weights_dev, size_t weight_bytes, void *kv_dev, size_t kv_bytes,
            void *scratch_dev, size_t scratch_bytes, void *hip_stream);

/* Load one tensor (Section 3.1: the target's weights and the adapter's; the exit layer was fixed at
 * kg_create).  src_dev is a row-major device array of n_elements values in the configured dtype;
 * it is copied into the arena in the library's tiled layout and may be freed when the call returns
 * (the call synchronises the stream). */
int kg_load_tensor(kg_ctx *ctx, int kind, int layer, const void *src_dev, size_t n_elements);

/* Optional: order in which physical KV pages are handed out (host, a permutation of 0..n-1 where
 * n = number of pages = ceil(max_seq / kv_page_tokens)).  Default is the identity.  Resets the
 * sequence. */
int kg_set_page_order(kg_ctx *ctx, const int32_t *perm_host, int n);

/* Run the full model and the adapter over the prompt (host, n >= 1 token ids): fills all caches
 * for positions 0..n-1 and returns the target model's next token, which becomes the pending
 * token of the first round.  Resets any previous sequence. */
int kg_prefill(kg_ctx *ctx, const kg_params *p, const int32_t *prompt_host, int n, int32_t *first_token);

/* One drafting step of the self-draft model M^s = A o M^b[:l] (Section 3.1): shallow layers on
 * the latest token, adapter (on two rows when a lagged feature is pending, Figure 2), shared LM
 * head with fused arg-max / log-sum-exp.  Outputs the draft token, its top-1 probability, and
 * *stop = 1 when drafting must end (confidence < eta, Eq. 4, or gamma drafts exist). */
int kg_draft_step(kg_ctx *ctx, const kg_params *p, int32_t *token, float *confidence, int *stop);

/* Compute the last draft's next early feature, then run the remaining layers M^b[l:] once over
 * [f_0..f_k] (Figure 2).  target_tokens (host, room for gamma+1) receives the target's greedy
 * token per row (mode 0) and *k_plus_1 the number of rows. */
int kg_verify(kg_ctx *ctx, const kg_params *p, int32_t *target_tokens, int *k_plus_1);

/* Acceptance (Section 3: the first rejected draft discards the rest) and cache rollback.
 * emitted (host, room for gamma+1) receives the 1..k+1 tokens of this round. */
int kg_accept(kg_ctx *ctx, const kg_params *p, int32_t *emitted, int *n_emitted);

/* prefill + rounds until max_new tokens are out (the first is the prefill's).  out: host, room for
 * max_new.  Produces exactly the stream the stepwise calls produce.  stats may be NULL. */
int kg_generate(kg_ctx *ctx, const kg_params *p, const int32_t *prompt_host, int n_prompt, int max_new,
                int32_t *out, int *n_out, kg_stats *stats);

/* Plain autoregressive decoding of the full model (Section 1), one token per forward. */
int kg_decode_plain(kg_ctx *ctx, const kg_params *p, const int32_t *prompt_host, int n_prompt, int max_new,
                    int32_t *out, int *n_out, kg_stats *stats);

/* One plain step after kg_prefill, after earlier plain steps, or after a kg_accept: feed `token` at
 * the next uncommitted position (the pending token's) through all layers and return the next token.
 * Lets a caller force the token stream.  After a plain step the adapter's cache is no longer in step
 * with the sequence: draft calls return KG_ESTATE until the next kg_prefill. */
int kg_plain_step(kg_ctx *ctx, const kg_params *p, int32_t token, int32_t *next_token);

/* Copy one row of the most recent logits to the host (float[vocab]).  which = 0: draft logits of
 * draft step `row` of the current round; which = 1: target logits of row `row` of the last
 * verify / prefill / plain step. */
int kg_read_logits(kg_ctx *ctx, int which, int row, float *host_out);

/* Copy the early feature f_row of the current round (float[d_model]) to the host: row = 0..KG_MAX_ROWS-1,
 * or row = -1 for the lagged feature (Figure 2: the early feature of the last accepted token that the
 * adapter has not seen yet; meaningful while kg_get_state reports lag = 1).  Other rows: KG_EINVAL. */
int kg_read_feature(kg_ctx *ctx, int row, float *host_out);

/* Copy the cached key and value vectors (float[d_model] each, widened from the cache type) of
 * cache `slot` (0..n_layers-1: decoder layers; n_layers: the adapter) at position pos. */
int kg_read_kv(kg_ctx *ctx, int slot, int pos, float *k_host, float *v_host);

/* Sequence state: committed tokens (`base`), tokens in the adapter's cache, lag flag, drafts so far. */
int kg_get_state(const kg_ctx *ctx, int *base, int *adapter_len, int *lag, int *n_drafts);

/* Per-kernel-class device timing, for bandwidth accounting (Section 1: decoding is bound by
 * reading the weights).  With profiling on, a pair of HIP events brackets every kernel launch of
 * the context's stream; elapsed times are summed when a call synchronises.  Classes: 0 = the
 * weight-streaming projections of the decode forwards (all linear layers and the LM head),
 * 1 = attention, 2 = the rest, 3 = the dense (MFMA) projections of the prompt pass, 4 = the fp32
 * contractions of the adapter's training step.
 * bytes[] is the algorithmic traffic of the launches: weight bytes for class 0, KV bytes read for
 * class 1; for classes 3 and 4 it holds floating-point operations (2 M N K per launch) instead.
 * kg_set_profiling resets the sums. */
typedef struct kg_profile {
    long long launches[5];
    double seconds[5];
    double bytes[5];
} kg_profile;
int kg_set_profiling(kg_ctx *ctx, int on);
int kg_get_profile(kg_ctx *ctx, kg_profile *out);

/* Drop the sequence state, keep bindings and weights. */
int kg_reset(kg_ctx *ctx);

const char *kg_last_error(const kg_ctx *ctx);
void kg_destroy(kg_ctx *ctx);

/*
 * Training of the adapter (Section 3.1 "Training Loss", Eq. 3; Section 4.1: AdamW), one step per
 * call on one token sequence, for every adapter architecture of kg_adapter_kind.  With the target model
 * frozen, the adapter is run over all n positions at once (causal attention over the earlier early
 * features) and
 *     loss = sum_t sum_v  - p_t[v] log q_t[v],   p_t = softmax(target logits at t), q_t = softmax(draft logits at t)
 * is differentiated with respect to every tensor of the adapter (Wq, Wk, Wv, Wo, g_in, g_last for
 * the paper's; an own LM head, the feed-forward tensors or the two linear maps for the others); AdamW
 * (decoupled weight decay on the matrices, none on the gains, bias-corrected moments) updates fp32 master copies, and the
 * adapter tensors the decode calls use are refreshed from them (matrices and gains re-rounded to bf16
 * where the model is bf16: decoding runs what a checkpoint in the model's type would hold).  All training arithmetic is fp32; keys and values inside the training graph are not
 * rounded to the cache's type.  The target model and its LM head are never updated.
 *
 *   kg_train_workspace_bytes / kg_train_bind: device workspace (256-byte aligned, BORROWED until
 *     kg_destroy) for sequences of up to max_tokens tokens (<= 2048 and <= max_seq); bind copies the
 *     loaded adapter tensors into the master copies and zeroes the AdamW moments and step count.
 *     All tensors must be loaded first; kg_bind, or loading an adapter tensor afterwards, drops the
 *     training binding (kg_train_step then returns KG_ESTATE until kg_train_bind is called again).
 *   kg_train_step: tokens_host[n], 1 <= n <= max_tokens.  *loss is Eq. 3 for the parameters before
 *     the update.  Drops the sequence state of the context (a new kg_prefill is needed to decode).
 *     It is kg_train_accumulate on a fresh gradient followed by kg_train_apply.
 *   kg_train_accumulate / kg_train_apply: a step over several sequences (Eq. 3 sums over all their
 *     positions): each accumulate call adds one sequence's gradient to the gradient block and returns
 *     that sequence's loss; apply performs the AdamW update with the accumulated gradient, refreshes
 *     the decode tensors and clears the count (KG_ESTATE when nothing was accumulated).
 *   kg_train_features / kg_train_accumulate_features: the frozen model's part of a step on its own.
 *     Several epochs over fixed sequences need the target model only once per sequence: features
 *     writes the early features F_dev [n][d_model] and the target logits Zt_dev [n][vocab] (fp32,
 *     caller-owned device memory) of a sequence; accumulate_features does what kg_train_accumulate
 *     does from such a pair instead of from tokens.
 *   kg_train_read: copy one buffer of the last step to the host (tests and monitoring):
 *     early features [n][d_model], target / draft logits [n][vocab], the gradient block and the
 *     parameter block, per-position losses [n].  n_floats must be the buffer's exact size.  A block
 *     holds the adapter's tensors row-major in this order: KG_ADAPTER_ATTN Wq, Wk, Wv, Wo, g_in, g_last
 *     (4 d^2 + 2 d floats); KG_ADAPTER_ATTN_HEAD the same, then the head [vocab][d]; KG_ADAPTER_LAYER the
 *     same, then g_post, Wg, Wu [d_ffn][d], Wd [d][d_ffn]; KG_ADAPTER_MLP W1, W2, g_in, g_last, head.
 */
typedef struct kg_train_params {
    float lr, beta1, beta2, eps, weight_decay;
} kg_train_params;
typedef enum kg_train_buffer {
    KG_TRAIN_FEATURES = 0, KG_TRAIN_TARGET_LOGITS = 1, KG_TRAIN_DRAFT_LOGITS = 2, KG_TRAIN_GRADIENTS = 3,
    KG_TRAIN_PARAMETERS = 4, KG_TRAIN_ROW_LOSSES = 5
} kg_train_buffer;
int kg_train_workspace_bytes(const kg_ctx *ctx, int max_tokens, size_t *bytes);
int kg_train_bind(kg_ctx *ctx, void *work_dev, size_t bytes, int max_tokens);
int kg_train_step(kg_ctx *ctx, const kg_train_params *hp, const int32_t *tokens_host, int n, double *loss);
int kg_train_accumulate(kg_ctx *ctx, const int32_t *tokens_host, int n, double *loss);
int kg_train_apply(kg_ctx *ctx, const kg_train_params *hp);
int kg_train_features(kg_ctx *ctx, const int32_t *tokens_host, int n, float *F_dev, float *Zt_dev);
int kg_train_accumulate_features(kg_ctx *ctx, const float *F_dev, const float *Zt_dev, int n, double *loss);
int kg_train_read(kg_ctx *ctx, int what, float *host_out, size_t n_floats);

/*
 * The dense contraction of the training step (the products with the LM head and the gradient
 * products of Eq. 3's chain rule), exposed for kernel-level tests: C[M][N] (+)= sum_k A(m,k) B(k,n)
 * in fp32 on the matrix units, A(m,k) = A_dev[m*sam + k*sak], B(k,n) = B_dev[k*sbk + n*sbn],
 * C row-major with leading dimension ldc >= N.  Launches on `hip_stream`, does not synchronise.
 */
int kg_op_gemm_f32(const float *A_dev, long sam, long sak, const float *B_dev, long sbk, long sbn, float *C_dev, long ldc,
                   int M, int N, int K, int accumulate, void *hip_stream);

/*
 * Stand-alone weight-streaming product Y[M][N] = X[M][K] . W^T used by every projection of the
 * decode forwards (Section 1: decoding is bound by reading the weights), exposed for kernel-level
 * tests and bandwidth measurements.
 *   kg_op_packed_bytes: bytes of the tiled form of a [N][K] matrix (N % 16 == 0, K % 8 == 0).
 *   kg_op_pack:   re-tile a row-major dev matrix (dtype 0 f32 / 1 bf16) into packed_dev.
 *   kg_op_linear: x_dev float[M][K], y_dev float[M][N]; work_dev >= kg_op_work_bytes(K) bytes of
 *                 device scratch; M <= KG_MAX_ROWS.  Launches on `hip_stream`, does not synchronise.
 */
size_t kg_op_packed_bytes(int dtype, int N, int K);
/* Position (0 .. KS-1) of k-step ks among the KS = ceil(K / 32) weight tiles of one 16-row tile in
 * the packed bf16 form: the tiles are stored in the order the projection workgroup reads them (its
 * eight waves own contiguous k ranges and walk them in step).  Host arithmetic only, no GPU: the
 * tests check that it is a permutation for every KS.  Returns -1 unless 0 <= ks < KS. */
int kg_op_tile_pos(int ks, int KS);
size_t kg_op_work_bytes(int K);
int kg_op_pack(int dtype, const void *src_dev, int N, int K, void *packed_dev, void *hip_stream);
int kg_op_linear(int dtype, const void *packed_dev, int N, int K, const float *x_dev, int M, float *y_dev,
                 void *work_dev, void *hip_stream);

/*
 * The one-row product y[N] = W . x[K] of kg_op_linear (bf16 tiles from kg_op_pack, x and y fp32 on the
 * device) computed on the vector ALUs instead of the matrix units: the same launch shape and memory
 * stream, another arithmetic unit.  It exists for the A/B measurement behind the choice of the matrix
 * units for the weight-streaming projections (Section 1: the projections are bound by reading the
 * weights, so the unit that multiplies should not matter; measured, it does not).  K % 16 == 0.
 * Launches on `hip_stream`, does not synchronise.
 */
int kg_op_linear_valu(const void *packed_dev, int N, int K, const float *x_dev, float *y_dev, void *hip_stream);

/*
 * kg_op_linear for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same product, same kernels
 * and bit-identical results; the activation staging area is a static device array inside the library
 * (KG_OP_STATIC_MAX_K * KG_MAX_ROWS * 4 bytes = 512 KB per GPU, held until the process ends) instead of
 * work_dev.  Allocates nothing (no hipMalloc / hipFree, no memset node: the area is cleared by a
 * kernel), launches on `hip_stream`, does not synchronise.  The device address of the array is looked
 * up on the first call on each device (the current device must be the one the pointers live on).
 * Errors: KG_EINVAL as kg_op_linear, or a device ordinal >= KG_OP_STATIC_MAX_DEVICES; KG_ENOSPC for
 * K > KG_OP_STATIC_MAX_K; KG_EHIP.  Every call on one GPU shares that GPU's array: calls that overlap
 * on one GPU (different streams or threads) race; calls ordered on one stream do not.
 */
#define KG_OP_STATIC_MAX_K 16384
#define KG_OP_STATIC_MAX_DEVICES 64
int kg_op_linear_static(int dtype, const void *packed_dev, int N, int K, const float *x_dev, int M, float *y_dev,
                        void *hip_stream);

/*
 * The generator of sampling mode on its own (kernel-level tests): out_dev[i] = first output word of
 * Philox4x32-10 for key (seed mod 2^32, seed >> 32) and counter (pos0 + i, purpose, 0, 0), i < n.
 * Launches on `hip_stream`, does not synchronise.
 */
int kg_op_philox_words(uint64_t seed, uint32_t pos0, uint32_t purpose, int n, uint32_t *out_dev, void *hip_stream);

/*
 * Measured ceiling for a weight stream (Section 1: decoding is bound by reading the weights): one
 * launch that reads `bytes` bytes (16-byte aligned dev pointer) with no dependencies between the
 * loads and keeps nothing.  work_dev: 4096 bytes of device scratch (XOR of what was read, so the
 * loads cannot be dropped).  Launches on `hip_stream`, does not synchronise; the caller times it.
 * KG_EINVAL for a NULL / misaligned pointer or fewer than 16 bytes.
 */
int kg_op_stream_read(const void *src_dev, size_t bytes, void *work_dev, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KANGAROO_H */
