/*
 * templora.h -- C ABI of the MI355X (gfx950) Temp-Lora chunk-update library.
 *
 * The library implements the inference-time training step of Temp-Lora
 * (arXiv 2401.11504): the training line of Algorithm 1 (the module Theta_k is
 * trained to produce the newest chunk from the tokens before it), i.e. one
 * forward + backward pass of a chunk of tokens through a frozen
 * Llama2-style decoder (Section 3, "Baselines") whose q, k, v, o, gate, up and
 * down projections carry a temporary LoRA module (Section 2; rank / alpha from
 * Section 3, "Setup"), followed by one AdamW step on the LoRA factors only.
 * The module's life cycle follows Algorithm 1: created at k = 0 (tl_lora_init),
 * trained once per chunk and epoch (tl_chunk_update), destroyed at the end
 * (tl_discard).  The frozen weights are never written.
 *
 * General conventions
 *   - Every function returns a tl_status and never throws or aborts.  Outputs
 *     are written only when TL_OK is returned.  tl_last_error() gives a
 *     human-readable message for the calling thread's last failure.
 *   - "device" pointers are HIP device memory on the GPU that was current when
 *     the model was created; "host" pointers are ordinary process memory.
 *   - All device work is enqueued on the HIP stream given to tl_model_create
 *     (a hipStream_t passed as void*; NULL = the default stream).  Calls that
 *     return host values synchronise that stream before returning.
 *   - Matrices are row-major.  W is [d_out, d_in]; A is [r, d_in]; B is
 *     [d_out, r]; activations are [tokens, width].
 *   - Projection index ("proj"): 0 q, 1 k, 2 v, 3 o, 4 gate, 5 up, 6 down.
 *   - A handle must not be used from two threads at once.
 *   - There is no CPU fallback: without a gfx950 device every call that would
 *     compute returns TL_ERR_DEVICE.
 */
#ifndef TEMPLORA_H
#define TEMPLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tl_model tl_model; /* frozen decoder: shapes + library-owned packed copies of the weights */
typedef struct tl_lora tl_lora;   /* temporary module: A, B (fp32 master + bf16 shadows), moments, step */

typedef enum {
    TL_OK = 0,
    TL_ERR_ARG = -1,         /* null pointer, bad enum value, bad size */
    TL_ERR_SHAPE = -2,       /* unsupported dimensions (see tl_model_cfg) */
    TL_ERR_TOKEN_RANGE = -3, /* a token id is < 0 or >= vocab */
    TL_ERR_WINDOW = -4,      /* n_tokens > max_tokens, n_tokens < 2 or n_ctx >= n_tokens */
    TL_ERR_NONFINITE = -5,   /* the loss (or a LoRA gradient) came out NaN/Inf; see tl_chunk_update */
    TL_ERR_DEVICE = -6,      /* HIP error, or no gfx950 device */
    TL_ERR_DISCARDED = -7,   /* the module was already discarded */
    TL_ERR_OOM = -8          /* device allocation failed */
} tl_status;

/* Decoder dimensions.  Supported: d_model == n_heads * d_head, d_head in {64, 128},
 * d_model, d_ffn and vocab multiples of 8, vocab >= 0 (0 = no embedding / lm_head:
 * only tl_layer_step may be used), max_tokens >= 2.  max_tokens is the window the
 * caller promises never to exceed in one call (chunk size plus conditioning
 * prefix, cf. the constraint L_X + Delta <= W of Section 2). */
typedef struct {
    int32_t n_layers, d_model, n_heads, d_head, d_ffn, vocab, max_tokens;
    float rms_eps;   /* RMSNorm epsilon (Llama2: 1e-5) */
    float rope_base; /* RoPE base (Llama2: 10000) */
} tl_model_cfg;

/* LoRA + optimizer hyper-parameters (Section 3 "Setup": alpha = 64, rank = 64,
 * learning rate 5e-5; the learning rate itself is a per-call argument so that
 * the caller can apply the paper's warm-up over the first chunks).
 * rank must be a multiple of 8 and <= 256. */
typedef struct {
    int32_t rank;
    float alpha;        /* output scale s = alpha / rank */
    float beta1, beta2; /* AdamW moment decay (0.9, 0.999) */
    float eps;          /* AdamW epsilon, added after the bias-corrected square root */
    float weight_decay; /* decoupled weight decay (0) */
    float a_init_std;   /* A ~ N(0, a_init_std^2) from a counter-based generator; B = 0 */
    uint64_t seed;      /* seed of that generator and of the dropout masks */
    float dropout;      /* LoRA dropout probability p in [0, 1) (Setup: 0.05; 0 = off), see below */
} tl_lora_cfg;

/*
 * LoRA dropout (Section 3 "Setup").  It acts on the input of the low-rank branch only and only in
 * tl_chunk_update / tl_chunk_train / tl_layer_step (tl_chunk_loss and the generation side run without it):
 *     Y = X W^T + s ((D o X) A^T) B^T,   D[t, c] = 0 with probability p, else 1 / (1 - p).
 * One mask per projection group input: group 0 = q|k|v (their common input), 1 = o, 2 = gate|up, 3 = down.
 * The mask is a pure function of (seed, step, layer, group, t, c), step = the optimizer step counter when the
 * pass starts, so that a caller (or a checker) can reproduce it:
 *     mix64(z): z += 0x9E3779B97F4A7C15; z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9;
 *               z = (z ^ z >> 27) * 0x94D049BB133111EB; return z ^ z >> 31        (64-bit wrap-around)
 *     key  = mix64(seed ^ mix64(2^63 | step << 16 | layer << 3 | group))
 *     kept = (mix64(key + t * d_in + c) >> 32) >= floor(p * 2^32)
 */

/* Number of device pointers tl_model_create expects: 9 per layer + 3. */
#define TL_PTRS_PER_LAYER 9
#define TL_N_WEIGHT_PTRS(n_layers) (TL_PTRS_PER_LAYER * (n_layers) + 3)

/*
 * Build a frozen decoder (the LM Theta of Algorithm 1).
 *   weight_ptrs: host array of TL_N_WEIGHT_PTRS(n_layers) device pointers:
 *     [9*l + p], p = 0..6 : projection p of layer l, bf16 [d_out, d_in]
 *     [9*l + 7], [9*l + 8]: RMSNorm gains before attention / before the MLP, fp32 [d_model]
 *     [9*L + 0]           : token embedding, bf16 [vocab, d_model]   (ignored if vocab == 0)
 *     [9*L + 1]           : final RMSNorm gain, fp32 [d_model]        (ignored if vocab == 0)
 *     [9*L + 2]           : lm_head, bf16 [vocab, d_model]            (ignored if vocab == 0)
 *   The buffers are only READ, and only during this call: the library keeps its
 *   own packed copies (q|k|v and gate|up stacked, plus a transposed copy of every
 *   matrix for the backward pass), so the caller may release its buffers after
 *   the call returns.  Nothing the caller owns is ever written.
 *   hip_stream: the stream all later work on this model runs on.
 * Errors: TL_ERR_ARG, TL_ERR_SHAPE, TL_ERR_DEVICE, TL_ERR_OOM; *out untouched on error.
 */
tl_status tl_model_create(const tl_model_cfg* cfg, const void* const* weight_ptrs, void* hip_stream,
                          tl_model** out);

/* Free the model's device memory.  Modules created on it must be discarded first
 * (or are invalid afterwards). NULL is accepted. */
tl_status tl_model_destroy(tl_model* model);

/*
 * Create the temporary module (Algorithm 1's initialisation: the module counter k starts at 0).  Allocates
 * A, B, gradients, moments, bf16 shadows and all activation workspaces for
 * max_tokens tokens.  A is drawn N(0, a_init_std^2), B = 0, moments 0, step 0.
 * Errors: TL_ERR_ARG, TL_ERR_SHAPE (rank), TL_ERR_OOM, TL_ERR_DEVICE.
 */
tl_status tl_lora_init(tl_model* model, const tl_lora_cfg* cfg, tl_lora** out);

/*
 * One training step on one chunk (Algorithm 1, "Train Theta_k"; one call per
 * chunk and epoch, the module state is carried from call to call).
 *   tokens   : host, int32[n_tokens], copied during the call.  The first n_ctx
 *              tokens are conditioning only (the preceding L_T tokens X_T of
 *              Section 2); the remaining ones are the chunk.
 *   Position t predicts token t+1; it carries loss iff t+1 >= max(n_ctx, 1).
 *   loss_out : host, mean negative log-likelihood over the *n_targets_out target
 *              positions (so perplexity = exp(loss)).
 *   lr       : AdamW learning rate of this step.
 * On success the step counter advances and A, B, moments are updated.  A bad
 * token id, a window violation or a non-finite loss (TL_ERR_NONFINITE) leave the
 * module state exactly as it was: the loss kernel leaves its verdict in device
 * memory and every optimizer launch of the call reads it before it writes.  The
 * optimizer step of a layer is applied as soon as that layer's gradients are
 * complete, while the layers below are still in their backward pass; so a
 * gradient entry that is not finite although the loss was (TL_ERR_NONFINITE as
 * well: the step of the layer it appeared in and of every layer below is
 * skipped, the step counter does not advance) and a device error during the
 * backward pass (TL_ERR_DEVICE) leave the layers above already stepped.
 */
tl_status tl_chunk_update(tl_lora* lora, const int32_t* tokens, int32_t n_tokens, int32_t n_ctx, float lr,
                          float* loss_out, int32_t* n_targets_out);

/* Same forward + loss without backward or update (Algorithm 1's Theta_k used as
 * a scorer: perplexity of a chunk under the current module). */
tl_status tl_chunk_loss(tl_lora* lora, const int32_t* tokens, int32_t n_tokens, int32_t n_ctx, float* loss_out,
                        int32_t* n_targets_out);

/*
 * The whole module update for one chunk: Algorithm 1's "Train Theta_k" with the
 * Section 3 "Setup" recipe (n epochs, linear learning-rate warm-up) and the batch
 * sizes of Table 5 (a chunk of Delta tokens trained in Delta / batch steps per epoch).
 *   tokens  : host int32[n_tokens]; the LAST n_chunk tokens are the chunk, whatever
 *             precedes them is text the stream already holds (conditioning only).
 *   The chunk is cut into consecutive pieces of cfg->batch tokens (the last may be
 *   shorter; batch = 0 or >= n_chunk means one piece).  Each piece is one training
 *   sample: the up to cfg->n_ctx_max tokens before the piece (L_T; earlier pieces
 *   of the same chunk included) as conditioning, loss on the piece only; one
 *   AdamW step per piece, pieces in order, the whole pass repeated cfg->epochs times.
 *   The rate of each step is tl_warmup_lr(cfg->lr, step counter, cfg->warmup_steps).
 *   losses_out : host fp32[epochs * ceil(n_chunk / batch)] or NULL: the loss of each step, in order.
 *   n_steps_out: steps completed (also written when a later step fails), or NULL.
 * All samples are validated before the first step (TL_ERR_ARG, TL_ERR_WINDOW: a sample
 * longer than max_tokens or without a target, TL_ERR_TOKEN_RANGE): then nothing
 * changes.  A non-finite loss in step i returns TL_ERR_NONFINITE with the first i
 * steps applied.
 */
typedef struct {
    int32_t n_ctx_max;    /* L_T (Setup: 1024) */
    int32_t batch;        /* tokens per optimizer step; 0 = the whole chunk */
    int32_t epochs;       /* n (Setup: 2) */
    int32_t warmup_steps; /* optimizer steps of linear warm-up, counted over the module's life; 0 = none.
                             Setup warms up over the first 2 chunks: 2 * epochs * pieces. */
    float lr;             /* peak learning rate (Setup: 5e-5) */
} tl_train_cfg;
tl_status tl_chunk_train(tl_lora* lora, const int32_t* tokens, int32_t n_tokens, int32_t n_chunk,
                         const tl_train_cfg* cfg, float* losses_out, int32_t* n_steps_out);

/* Linear warm-up (Setup): the rate of the optimizer step with 0-based index `step`
 * is lr * min(1, (step + 1) / warmup_steps); lr itself if warmup_steps <= 0. */
float tl_warmup_lr(float lr, int64_t step, int32_t warmup_steps);

/* Destroy the module (Algorithm 1, last line: Theta_k <- Theta).  Frees all its
 * device memory; the handle stays valid only for tl_lora_free and makes every
 * other call return TL_ERR_DISCARDED.  The base model is untouched by design. */
tl_status tl_discard(tl_lora* lora);

/* ---- generation side (Algorithm 1, the token loop between two updates; Section 2, "cache reuse" / recomputation) ----
 * Greedy decoding with the module applied, over a key/value cache owned by the module.  The cache holds the
 * rotated keys and the values of every layer for positions 0 .. kv_length-1 (positions count from the start of the
 * window handed to tl_prefill).  It is (re)built by tl_prefill and extended by tl_decode_step; every
 * tl_chunk_update / tl_chunk_loss / tl_layer_step invalidates it, which is the paper's default of recomputing the
 * cache with the updated module after each chunk (call tl_prefill on the last L_X tokens); tl_cache_reuse changes that.
 *
 * tl_prefill: tokens host int32[n_tokens], 1 <= n_tokens <= max_tokens.  Runs the LoRA-adapted forward pass over the
 * window, fills the cache, and returns in *next_token the greedy continuation (index of the largest last-position
 * logit; the lowest index wins among equal logits).  logits_out: host fp32[vocab] for the last position, or NULL.
 * tl_decode_step: appends `token` at position kv_length and returns the next greedy token (and its logits).
 * Errors: TL_ERR_ARG (null pointer; decode without a cache), TL_ERR_WINDOW (n_tokens out of range; cache full),
 * TL_ERR_TOKEN_RANGE, TL_ERR_SHAPE (vocab = 0), TL_ERR_DISCARDED, TL_ERR_DEVICE.  Outputs written only on TL_OK. */
tl_status tl_prefill(tl_lora* lora, const int32_t* tokens, int32_t n_tokens, int32_t* next_token, float* logits_out);
tl_status tl_decode_step(tl_lora* lora, int32_t token, int32_t* next_token, float* logits_out);
tl_status tl_kv_length(tl_lora* lora, int32_t* n_out);

/*
 * Algorithm 1 as one call (the cascaded deployment of Section 3, "Efficiency": generation pauses while the module is
 * updated).  Starting from `prompt` (host int32[n_prompt], n_prompt >= 1), repeat: take the most recent cfg->window
 * tokens of the text so far as X (L_X), rebuild the cache with the current module, decode greedily until the chunk
 * holds cfg->chunk tokens (Delta), then tl_chunk_train on that chunk with the up to cfg->train.n_ctx_max tokens
 * before it (L_T) as conditioning.  Stops after n_new tokens; a last, incomplete chunk is not trained on.  The module
 * stays alive afterwards (the caller discards it, Algorithm 1's last line).
 *   tokens_out : host int32[n_new], the generated tokens.
 *   losses_out : host fp32[(n_new / chunk) * epochs * ceil(chunk / batch)] or NULL: the loss of every training step.
 *   n_steps_out: training steps made, or NULL.
 * Needs window + chunk <= max_tokens and n_ctx_max + batch <= max_tokens (TL_ERR_WINDOW otherwise, before anything
 * runs).  Other errors as tl_prefill / tl_decode_step / tl_chunk_train; what was generated and trained before an
 * error stays.
 */
typedef struct {
    int32_t window;      /* L_X */
    int32_t chunk;       /* Delta */
    tl_train_cfg train;  /* L_T, batch, epochs, warm-up, learning rate */
} tl_generate_cfg;
tl_status tl_generate(tl_lora* lora, const int32_t* prompt, int32_t n_prompt, int32_t n_new, const tl_generate_cfg* cfg,
                      int32_t* tokens_out, float* losses_out, int32_t* n_steps_out);

/* Cache reuse (Section 2: after an update, keep the key/value states instead of recomputing them with the updated
 * module).  on != 0: the cache moves to buffers of its own (allocated on the first call: n_layers * max_tokens *
 * 3 d_model bf16) and survives tl_chunk_update / tl_chunk_train / tl_chunk_loss / tl_layer_step; tl_decode_step then
 * attends over keys and values of the earlier module for the positions cached before the update and uses the updated
 * module for everything it computes itself.  tl_prefill still rebuilds the whole cache with the current module (the
 * paper's default, and what the caller does when the window is full).  on == 0 (the initial state): back to the
 * default, the cache is dropped.  Errors: TL_ERR_ARG, TL_ERR_DISCARDED, TL_ERR_OOM, TL_ERR_DEVICE. */
tl_status tl_cache_reuse(tl_lora* lora, int32_t on);

/* Release the (discarded or not) handle itself. NULL is accepted. */
tl_status tl_lora_free(tl_lora* lora);

/* ---- inspection surface used by parity tests (not part of the paper's method) ---- */

typedef enum {
    TL_FACTOR_A = 0, TL_FACTOR_B = 1,   /* fp32 master values */
    TL_GRAD_A = 2, TL_GRAD_B = 3,       /* gradients of the last tl_chunk_update / tl_layer_step */
    TL_M_A = 4, TL_M_B = 5,             /* AdamW first moments */
    TL_V_A = 6, TL_V_B = 7              /* AdamW second moments */
} tl_which;

/* Copy one tensor of (layer, proj) to host fp32.  n must equal r*d_in (A-like) or d_out*r (B-like). */
tl_status tl_get_factor(tl_lora* lora, int32_t layer, int32_t proj, int32_t which, float* host_out, size_t n);
/* Overwrite A or B (which = TL_FACTOR_A / TL_FACTOR_B) from host fp32; refreshes the bf16 shadows. */
tl_status tl_set_factor(tl_lora* lora, int32_t layer, int32_t proj, int32_t which, const float* host_in, size_t n);
/* Optimizer step counter (number of successful updates so far). */
tl_status tl_get_step(tl_lora* lora, int64_t* step_out);
/* Per-position negative log-likelihood of the last update/loss call: host fp32[n], n = that call's n_tokens
 * (0 at non-target positions). */
tl_status tl_get_nll(tl_lora* lora, float* host_out, size_t n);
/* Gradient of the last update's loss w.r.t. the hidden state entering layer `boundary`
 * (boundary = n_layers: the state entering the final RMSNorm): host fp32[n_tokens * d_model]. */
tl_status tl_get_dh(tl_lora* lora, int32_t boundary, float* host_out, size_t n);
/* The gradient at boundary 0 (the embedding output) reaches no trainable parameter: the embedding is frozen
 * (Section 2: only the module is trained) and dA, dB of layer 0 do not need it.  By default an update therefore
 * leaves out dX of layer 0's q|k|v projections and the backward of its first RMSNorm, and tl_get_dh(.., 0, ..)
 * returns TL_ERR_ARG.  on != 0 makes the following updates compute it (parity checks); every other output of the
 * update is bit-identical either way. */
tl_status tl_keep_input_grad(tl_lora* lora, int32_t on);

/* ---- measurement hooks (not part of the paper's method) ----
 * While enabled, every launch of the frozen-weight GEMM kernel (the LoRA-adapted projections forward and their
 * dX backward, lm_head forward and backward) made by tl_chunk_update / tl_chunk_loss / tl_layer_step is bracketed
 * by two HIP events on the model's stream.  tl_profile_read synchronises, returns the summed elapsed time of
 * those launches in milliseconds, their number, and the floating-point operations they performed
 * (2 M N (K + K2) per launch), and clears the counters.  On the generation side (tl_decode_step) the bracketed
 * launches are the matrix-vector products that stream a frozen matrix (four per layer and the lm_head), with
 * 2 N (K + r) operations each, i.e. N (K + r) bf16 elements = 2 N (K + r) bytes read per launch. */
tl_status tl_profile_enable(tl_lora* lora, int32_t on);
tl_status tl_profile_read(tl_lora* lora, double* ms_total, int64_t* launches, double* flop_total);

/*
 * One decoder layer alone: forward from a given hidden state, backward from a
 * given upstream gradient, gradients of that layer's 7 LoRA pairs, and
 * (apply_adamw != 0) one AdamW step on them with learning rate lr.
 *   h_in, dh_out : device fp32 [n_tokens, d_model] (read)
 *   h_out, dh_in : device fp32 [n_tokens, d_model] (written)
 * Positions are 0..n_tokens-1.  Errors as tl_chunk_update.
 */
tl_status tl_layer_step(tl_lora* lora, int32_t layer, const float* h_in, const float* dh_out, int32_t n_tokens,
                        float* h_out, float* dh_in, float lr, int32_t apply_adamw);

/*
 * A single LoRA-adapted linear layer in fp32 (no model needed):
 *   Y = X W^T + s (X A^T) B^T;  dX = dY W + dH A, dH = s dY B;  dA = dH^T X;  dB = s dY^T (X A^T);
 *   then (apply_adamw != 0) the first AdamW step (zero moments, step 1) giving A_new, B_new.
 * All pointers device fp32: X [T, d_in], W [d_out, d_in], A [r, d_in], B [d_out, r], dY [T, d_out] (read);
 * Y [T, d_out], dX [T, d_in], dA [r, d_in], dB [d_out, r], A_new, B_new (written; A_new/B_new may be NULL
 * when apply_adamw == 0).  Synchronises the stream before returning.
 */
tl_status tl_linear_step(const float* X, const float* W, const float* A, const float* B, const float* dY,
                         int32_t T, int32_t d_in, int32_t d_out, int32_t r, float s, float lr, float beta1,
                         float beta2, float eps, float weight_decay, int32_t apply_adamw, float* Y, float* dX,
                         float* dA, float* dB, float* A_new, float* B_new, void* hip_stream);

/*
 * tl_linear_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as tl_linear_step, but the scratch that call
 * takes from hipMalloc (H = X A^T and dH, fp32 [T, r] each, and with apply_adamw the 2 r (d_in + d_out) moments) lives
 * in a buffer of 2^20 floats (4 MiB) that is part of the library's image: every GPU the library runs on holds one
 * until the process ends, and this call performs no allocation or release of any kind.
 * TL_ERR_SHAPE if 2 T r (+ 2 r (d_in + d_out)), each part rounded up to 64 floats, exceeds 2^20 floats.
 * All calls on one GPU share that buffer: it holds the previous call's values on entry (the call clears what it needs
 * zeroed), and two calls that overlap in time on one GPU race -- the caller serialises them.
 */
tl_status tl_linear_step_static(const float* X, const float* W, const float* A, const float* B, const float* dY,
                                int32_t T, int32_t d_in, int32_t d_out, int32_t r, float s, float lr, float beta1,
                                float beta2, float eps, float weight_decay, int32_t apply_adamw, float* Y, float* dX,
                                float* dA, float* dB, float* A_new, float* B_new, void* hip_stream);

/* ---- single kernels, exposed for per-kernel parity tests and timing ----
 * All pointers are device memory; work is enqueued on hip_stream and NOT synchronised.
 * bf16 buffers are passed as uint16_t*. */

/* C[M,N] = alpha * (A[M,K] B[N,K]^T + A2[M,K2] B2[N,K2]^T) (+ R[M,N] if R != NULL), bf16 MFMA, fp32 accumulate.
 * A2/B2 may be NULL (K2 = 0).  c_f32 != 0: C and R are fp32, else C is bf16 and R must be NULL.
 * lda/ldb/lda2/ldb2/ldc are row strides in elements; K, K2, lda, ldb, lda2, ldb2 multiples of 8.
 * Tile shape, contraction split and (for many-tile shapes whose last round of workgroups would be poorly filled)
 * a split into two launches over two column ranges are chosen as in the update path.
 * workspace: NULL, or device fp32 scratch of workspace_elems floats for the partial results of a split contraction
 * (without it no shape is split; a split of s ways uses s * M * N floats; contents are undefined afterwards). */
tl_status tl_k_gemm_nt(const uint16_t* A, int32_t lda, const uint16_t* B, int32_t ldb, int32_t M, int32_t N,
                       int32_t K, const uint16_t* A2, int32_t lda2, const uint16_t* B2, int32_t ldb2, int32_t K2,
                       float alpha, const float* R, void* C, int32_t ldc, int32_t c_f32, float* workspace,
                       size_t workspace_elems, void* hip_stream);
/* Which tile configuration tl_k_gemm_nt uses for dense operands of these sizes with a workspace of workspace_elems
 * floats (0 = none): its name ("128x128", "256x128", "256x128-split", "256x192", "256x256", "reg-128x128",
 * "reg-128x64", "64x64", "64x64-split", "reg-64x64", "reg-64x64-split") into name_out (host, name_cap bytes), the
 * contraction split and the number of launches (2 = two column ranges; the name is then the first range's).  Host
 * only, nothing is launched: the kernel tests use it to show that their shapes reach every configuration. */
tl_status tl_k_gemm_nt_plan(int32_t M, int32_t N, int32_t K, int32_t K2, size_t workspace_elems, char* name_out,
                            size_t name_cap, int32_t* n_split_out, int32_t* n_launches_out);

/* C[Mo,No] (fp32) = alpha * P[T,Mo]^T Q[T,No]  (contraction over the token dimension; dA and dB). */
tl_status tl_k_gemm_tn(const uint16_t* P, int32_t ldp, const uint16_t* Q, int32_t ldq, int32_t T, int32_t Mo,
                       int32_t No, float alpha, float* C, int32_t ldc, void* hip_stream);

/* y (bf16) = h * rsqrt(mean(h^2) + eps) * g ; h fp32 [T, d], g fp32 [d]. */
tl_status tl_k_rmsnorm_fwd(const float* h, const float* g, int32_t T, int32_t d, float eps, uint16_t* y,
                           void* hip_stream);
/* dh_out (fp32) = dres + RMSNorm backward of dy (bf16) at h; optional bf16 copy of dh_out (may be NULL). */
tl_status tl_k_rmsnorm_bwd(const uint16_t* dy, const float* h, const float* g, const float* dres, int32_t T,
                           int32_t d, float eps, float* dh_out, uint16_t* dh_out_bf16, void* hip_stream);
/* In-place RoPE on x bf16 [T, n_heads, d_head] with row stride ld elements; sign = +1 forward, -1 backward. */
tl_status tl_k_rope(uint16_t* x, int32_t ld, int32_t T, int32_t n_heads, int32_t d_head, float base, int32_t pos0,
                    int32_t sign, void* hip_stream);
/* The same through the (cos, sin) table the chunk path uses: `table` (device, 16-byte aligned, table_elems >=
 * (pos0 + T) * d_head floats, caller-owned scratch) is filled with the angles of positions 0 .. pos0 + T - 1 and the
 * rotation then reads it.  TL_ERR_SHAPE if the table is too small or misaligned. */
tl_status tl_k_rope_table(uint16_t* x, int32_t ld, int32_t T, int32_t n_heads, int32_t d_head, float base,
                          int32_t pos0, int32_t sign, float* table, size_t table_elems, void* hip_stream);
/* a = silu(g) * u, gu bf16 [T, 2f] = [gate | up], a bf16 [T, f]. */
/* y = D o x for one projection group input (bf16 [T, d_in]), D as defined with tl_lora_cfg.dropout. */
tl_status tl_k_dropout(const uint16_t* x, int32_t T, int32_t d_in, float p, uint64_t seed, int64_t step,
                       int32_t layer, int32_t group, uint16_t* y, void* hip_stream);
tl_status tl_k_swiglu_fwd(const uint16_t* gu, int32_t T, int32_t f, uint16_t* a, void* hip_stream);
/* One-token kernels of the generation side.
 * tl_k_gemv: y[N] = alpha * (W[N,K] x[K] + sum_j lora_b[n,j] lora_h[(n / rows_per_group) r + j]) (+ resid[n]).
 *   W, x, lora_b bf16; lora_h fp32 (already scaled); lora_b may be NULL.  y_f32 != 0: y and resid fp32, else y bf16
 *   and resid must be NULL.  K, ldw multiples of 8.
 * tl_k_attention_decode: o[n_heads * d_head] (bf16) = softmax(q K^T / sqrt(d_head)) V per head, q one row, K and V
 *   rows 0 .. n_keys-1 with row stride ld (elements), every key visible.  workspace: NULL, or device fp32 scratch of
 *   workspace_elems floats: with it the keys are cut into up to 32 ranges of >= 128 keys, one workgroup per (head,
 *   range) and a second launch that merges them (n_heads * ranges * (d_head + 2) floats are used); without it one
 *   workgroup per head reads the whole cache.
 * tl_k_argmax: index of the largest of n fp32 values, lowest index among equals; out is a device int32. */
tl_status tl_k_gemv(const uint16_t* W, int32_t ldw, const uint16_t* x, int32_t N, int32_t K, const uint16_t* lora_b,
                    const float* lora_h, int32_t r, int32_t rows_per_group, float alpha, const float* resid, void* y,
                    int32_t y_f32, void* hip_stream);
/* y fp32 [N] = W x with x formed inside the launch: mode 1, x = bf16(RMSNorm(h) * gain) of the fp32 row h[K];
 * mode 2, x = bf16(silu(g) * u) of the bf16 row gu = g[K] | u[K].  x_out (bf16 [K]) receives x if not NULL. */
tl_status tl_k_gemv_pre(const uint16_t* W, int32_t ldw, int32_t N, int32_t K, int32_t mode, const float* h,
                        const float* gain, float eps, const uint16_t* gu, uint16_t* x_out, float* y, void* hip_stream);
tl_status tl_k_attention_decode(const uint16_t* q, const uint16_t* k, const uint16_t* v, int32_t ld, int32_t n_keys,
                                int32_t n_heads, int32_t d_head, uint16_t* o, float* workspace, size_t workspace_elems,
                                void* hip_stream);
tl_status tl_k_argmax(const float* x, int32_t n, int32_t* out, void* hip_stream);
/* dgu bf16 [T, 2f] from da bf16 [T, f] and gu. */
tl_status tl_k_swiglu_bwd(const uint16_t* da, const uint16_t* gu, int32_t T, int32_t f, uint16_t* dgu,
                          void* hip_stream);
/* Causal attention forward: q, k, v, o bf16 [T, n_heads, d_head] with row strides ldq (shared by q, k, v)
 * and ldo; lse fp32 [n_heads, T] = log-sum-exp of the scaled scores of each row. */
tl_status tl_k_attention_fwd(const uint16_t* q, const uint16_t* k, const uint16_t* v, int32_t ldq, int32_t T,
                             int32_t n_heads, int32_t d_head, uint16_t* o, int32_t ldo, float* lse,
                             void* hip_stream);
/* Causal attention backward: dq, dk, dv (row stride ldq) from do (row stride ldo), q, k, v, o, lse.
 * delta is fp32 scratch [n_heads, T]. */
tl_status tl_k_attention_bwd(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* o,
                             const uint16_t* d_o, const float* lse, int32_t ldq, int32_t ldo, int32_t T,
                             int32_t n_heads, int32_t d_head, uint16_t* dq, uint16_t* dk, uint16_t* dv,
                             float* delta, void* hip_stream);
/* Fused softmax cross-entropy over fp32 logits [T, V] with int32 labels [T] and a target mask given by
 * [first_target, T-1): nll fp32 [T]; dlogits bf16 [T, V] = (softmax - onehot) / n_targets on target rows,
 * 0 elsewhere (dlogits may be NULL: loss only).  loss_sum[0] (fp32) receives sum of nll over targets. */
tl_status tl_k_cross_entropy(const float* logits, const int32_t* labels, int32_t T, int32_t V,
                             int32_t first_target, int32_t n_targets, float* nll, uint16_t* dlogits,
                             float* loss_sum, void* hip_stream);
/* Fused AdamW over n fp32 elements; writes p, m, v in place and a bf16 copy of p (shadow may be NULL). */
tl_status tl_k_adamw(float* p, const float* g, float* m, float* v, uint16_t* shadow, size_t n, int64_t step,
                     float lr, float beta1, float beta2, float eps, float weight_decay, void* hip_stream);
/* h fp32 [T, d] = E[tok[t]] (bf16 rows widened). */
tl_status tl_k_embed(const uint16_t* E, const int32_t* tokens, int32_t T, int32_t d, float* h, void* hip_stream);

const char* tl_last_error(void);
/* Library version string. */
const char* tl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TEMPLORA_H */
