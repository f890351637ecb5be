/*
 * dllm.h -- C ABI of the MI355X (gfx950) SlowFast-sampling library.
 *
 * One denoising step of a masked-diffusion LLM (Section 3.1 of the paper:
 * the mask predictor's full-sequence forward, eq. 2; greedy decode, eq. 3;
 * confidence, the equation of "Low-Confidence Remasking") followed by the
 * SlowFast selection rule (Section 3.3, eqs. 6 and 9, Algorithm 1), plus the
 * stage controller and decode loop of Algorithm 1.
 *
 * Conventions
 *   - Every function returns DLLM_OK (0) or a negative dllm_status.  Nothing
 *     throws across this boundary.  A textual reason for the last failure of a
 *     handle is kept in the handle (dllm_last_error); for handle-free functions
 *     it is kept per thread (dllm_last_error(NULL)).
 *   - "dev" pointers are HIP device memory on the device that was current at
 *     dllm_create; "host" pointers are ordinary host memory.
 *   - All device work is enqueued on the HIP stream given at dllm_create (or
 *     passed to the handle-free functions).  Calls return without waiting
 *     unless stated otherwise.  The library creates no streams of its own.
 *   - The caller owns tokens / mask / prev_pred / commit lists / weights and
 *     keeps them alive while work that uses them is in flight.  The library
 *     owns its workspace (activations, logits, per-position predictions).
 *   - Matrices are row-major bf16.  A linear map is stored as W[N][K] and
 *     applied as y = x W^T.
 *   - Positions are absolute, 0-based, over prompt + generated region.  A span
 *     [s, e] is inclusive at both ends; the generated region is
 *     [gen_start, gen_end).
 */
#ifndef DLLM_H
#define DLLM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DLLM_OK = 0,
    DLLM_EINVAL = -1,    /* bad argument: null pointer, shape, range                 */
    DLLM_ENOMEM = -2,    /* device or host allocation failed                         */
    DLLM_EHIP = -3,      /* a HIP runtime call or kernel launch failed               */
    DLLM_ECAPACITY = -4, /* commit list capacity smaller than the step's window      */
    DLLM_ESTATE = -5     /* call not valid in the handle's current state             */
} dllm_status;

enum { DLLM_STAGE_SLOW = 0, DLLM_STAGE_FAST = 1, DLLM_STAGE_IDLE = 2 };

#define DLLM_MAX_BATCH 64

typedef struct dllm_handle dllm_handle; /* opaque, owned by the library */

/* Shape of the mask predictor.  The paper only calls it a bidirectional
 * Transformer (Section 3.1); the operator stack is LLaDA-style: pre-norm
 * RMSNorm, rotate-half RoPE on q and k, non-causal multi-head attention with
 * scale 1/sqrt(head_dim), SwiGLU feed-forward, untied vocabulary projection,
 * no biases.  Requires n_heads * head_dim == d_model, head_dim in {64, 128},
 * d_model % 8 == 0, d_ffn % 8 == 0, vocab % 8 == 0, 0 <= mask_id < vocab,
 * 1 <= max_batch <= DLLM_MAX_BATCH, 1 <= max_seq <= 8192. */
typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab, mask_id;
    float rms_eps, rope_theta;
    int32_t max_batch, max_seq;
} dllm_config;

/* Device pointers to bf16 weights; the library reads them in place and never
 * copies or frees them.  Per-layer members are host arrays of n_layers device
 * pointers (the arrays themselves are copied at create).
 * (dllm_create also makes panel-major copies of the projection matrices for its own use, see "Panel-major
 * layout" below; the caller's arrays stay in use for shapes those copies do not serve and must stay alive.)
 *   embed      [vocab][d_model]     token embedding ([MASK] has its own row)
 *   lm_head    [vocab][d_model]
 *   final_norm [d_model]
 *   attn_norm  [d_model]            gain of the norm before attention
 *   wqkv       [3 d_model][d_model] rows: q features | k features | v features,
 *                                   each head-major (h * head_dim + j)
 *   wo         [d_model][d_model]
 *   ffn_norm   [d_model]
 *   w_gate_up  [2 d_ffn][d_model]   rows: gate | up
 *   w_down     [d_model][d_ffn] */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *attn_norm, *const *wqkv, *const *wo, *const *ffn_norm, *const *w_gate_up, *const *w_down;
} dllm_weights;

/* What one step needs to know about one sequence (Section 3.3).
 *   slow stage: the window is [s_cycle, gen_end - 1]; the step commits the
 *     top_k (= k_slow) most confident masked positions of the window
 *     ("Cautious Decoding") and reports e_cand (eq. 6).
 *   fast stage: the window is [s_cycle, e_cycle]; the step commits every masked
 *     position of the window whose confidence exceeds tau_high_conf (eq. 9),
 *     or, if there is none, the top_k (= k_fast) most confident ones
 *     ("Fallback Top-k Refinement").
 *   idle: the sequence rides along in the forward; nothing is selected.
 *   conv_mode 0: Algorithm 1 as printed.  1: a position joins the fast set only
 *     if its prediction equals prev_pred (Convergence Principle, Section 3.2).
 * Ranking is by (higher confidence, then lower position); thresholds are
 * strict ">"; every comparison is made on binary32 confidences. */
typedef struct {
    int32_t stage;
    int32_t s_cycle, e_cycle;
    int32_t top_k;
    float tau_min_conf, tau_high_conf;
    int32_t conv_mode;
    int32_t gen_start, gen_end;
} dllm_stage_params;

/* Result of a step, all members dev pointers, caller-allocated.
 *   n_commit       [B]            committed positions of this step
 *   pos, tok, conf [B][capacity]  the commits, ascending position
 *   e_cand         [B]            eq. 6 over the window, -1 if no masked position
 *                                 of the window exceeds tau_min_conf
 *   first_masked   [B]            leftmost masked position of the window before
 *                                 the commit, -1 if none
 *   n_masked_after [B]            masked positions left in the whole sequence
 * capacity must be >= the longest window of the batch. */
typedef struct {
    int32_t capacity;
    int32_t *n_commit;
    int32_t *pos, *tok;
    float *conf;
    int32_t *e_cand, *first_masked, *n_masked_after;
} dllm_commit_list;

/* Inputs of Algorithm 1 ("Require" line) plus the k_slow / k_fast the paper
 * leaves open. */
typedef struct {
    int32_t max_steps; /* N */
    int32_t k_max, w_hist;
    int32_t k_slow, k_fast;
    int32_t conv_mode;
    float sigma2_stable, tau_min_conf, tau_high_conf;
    int32_t out_of_span_cache; /* 0 / 1: Section 3.3's Out-of-Span Caching in the fast stage: the first step of
                                  a fast stage is a complete prediction; masked positions right of e_cycle whose
                                  confidence there is below tau_min_conf are not recomputed (their keys/values
                                  are reused) in the later steps of that stage */
    int32_t prompt_cache_interval; /* K_p >= 0.  0: off.  Otherwise the long-interval prompt caching of dLLM-Cache,
                                      which the paper combines its sampler with (Section 4.2), in its simplest form:
                                      every K_p-th step (from step 0) is a complete forward that refreshes all cached
                                      keys/values; in the steps between, the prompt positions are not recomputed */
    int32_t response_cache_interval; /* K_r >= 0.  0: off.  Otherwise the short-interval response caching of that
                                        scheme, in the same simplest form: every K_r-th step (from step 0) recomputes
                                        the whole response; in the steps between, the response positions outside the
                                        range the step rates ([s_cycle, end] in the slow stage, [s_cycle, e_cycle] in
                                        the fast stage) are not recomputed.  The first step of a fast stage with
                                        out_of_span_cache stays a complete forward.  The scheme's value-based choice
                                        of positions to refresh in between is not part of this library */
} dllm_decode_params;

/* One record per denoising step of dllm_decode. */
typedef struct {
    int32_t n_slow, n_fast, n_idle; /* sequences in each stage during the step */
    int32_t n_commit;               /* tokens committed by the step, whole batch */
    float ms;                       /* device time of the step (HIP events)      */
} dllm_step_stat;

/* Validates the configuration, records the weight pointers and allocates the
 * workspace for max_batch x max_seq on the current device (the bf16 logits
 * buffer, max_batch x max_seq x vocab, and the key/value cache of the cached
 * steps are allocated by the first call that needs them).  `hip_stream` is a
 * hipStream_t (NULL = the default stream).  Synchronous. */
int dllm_create(const dllm_config *cfg, const dllm_weights *w, void *hip_stream, dllm_handle **out);
void dllm_destroy(dllm_handle *h);
const char *dllm_last_error(const dllm_handle *h);

/* One denoising step on a batch (Section 3.1 eqs. 2-5 + Section 3.3):
 * forward over all B*L positions, greedy decode and confidence at the masked
 * positions of each window, selection, and the transition
 *   tokens[pos] <- prediction, mask[pos] <- 0            at committed positions
 *   prev_pred[i] <- prediction                           at every masked position of the window
 * Committed tokens are never re-masked.  Logits never leave the library.
 *   tokens    dev int32 [B][L]  in/out; every id must lie in [0, vocab).  The ids live on the device,
 *                               so the host cannot check them before enqueueing: an id outside the range
 *                               is never used as an index (its position gets an all-zero embedding) and
 *                               raises a flag that dllm_decode / dllm_decode_low_confidence (after every
 *                               step) and dllm_sync_status turn into DLLM_EINVAL
 *   mask      dev uint8 [B][L]  in/out, 1 = [MASK]
 *   prev_pred dev int32 [B][L]  in/out, -1 = no previous prediction
 *   sp        host [B]
 *   out       host struct of dev pointers
 * Errors (nothing is enqueued): null pointers, B or L out of range, a window
 * outside [gen_start, gen_end), e_cycle < s_cycle in the fast stage, top_k < 1,
 * capacity below the longest window.  A sequence without masked positions in
 * its window is not an error: n_commit = 0. */
int dllm_step(dllm_handle *h, int32_t B, int32_t L, int32_t *tokens, uint8_t *mask, int32_t *prev_pred,
              const dllm_stage_params *sp, const dllm_commit_list *out);

/* Waits for the handle's stream and reports what only the device could see: DLLM_EINVAL if a step or
 * forward since the last report read a token id outside [0, vocab) (Section 3.1: the state y^(k) is a
 * sequence over the vocabulary; see `tokens` above), else DLLM_OK.  Reporting clears the condition. */
int dllm_sync_status(dllm_handle *h);

/* Where the greedy decode and the confidence (Section 3.1, eq. 3 and the confidence it defines)
 * of dllm_step / dllm_step_cached / the decode calls are computed.  enable != 0 (the default):
 * inside the vocabulary projection, on its accumulators after the rounding to bf16; the logits
 * are never written, each wave leaves (max, sum of exp, argmax) of its column slice per row and a
 * merge kernel combines the slices.  enable == 0: the projection writes bf16 logits
 * (dllm_debug_logits can read them) and a separate kernel reads them back.  Both take argmax and
 * maximum over the same bf16 values, so predictions are identical; the confidences differ by the
 * order of an fp32 sum.  Takes effect from the next step. */
int dllm_set_fused_selector(dllm_handle *h, int32_t enable);

/* dllm_step with out-of-span caching (Section 3.3, "Out-of-Span Caching"; Algorithm 1, fast
 * phase: "cache features for position i").  The features kept per position are its keys (after
 * the rotary embedding) and values in every layer.  Per sequence, cache_mode is
 *   DLLM_CACHE_OFF      nothing special for this sequence
 *   DLLM_CACHE_REFRESH  first step of a fast stage: a complete prediction whose confidences
 *                       cover [s_cycle, gen_end), so that the caller can pick the positions to
 *                       cache (the paper: masked, right of e_cycle, confidence < tau_min_conf;
 *                       read them with dllm_debug_rows); selection stays inside [s_cycle, e_cycle]
 *   DLLM_CACHE_REUSE    later steps of the stage: positions with skip[b][i] != 0 are not
 *                       recomputed; all others are, attend to the cached keys/values of the
 *                       skipped ones, and refresh their own cache rows
 * REFRESH widens the rated range only in the fast stage; REUSE may skip any position outside the
 * sequence's window (prompt caching skips the prompt).  In any step with a sequence in REFRESH or REUSE the
 * keys/values of every recomputed position of the batch are written to the cache (allocated on
 * first use: n_layers x max_batch x max_seq x 3 d_model bf16).
 *   cache_mode  host int32 [B]
 *   skip        host uint8 [B][L], may be NULL when no sequence is in REUSE; read before the
 *               call returns; a skipped position must lie outside the positions the step rates
 * Errors beyond dllm_step's: DLLM_ESTATE when positions are skipped before any step filled the
 * cache; DLLM_EINVAL for a skipped position inside the window, or a model whose d_model is
 * not a multiple of 64 (the cached path uses the fused QKV + RoPE kernel only). */
#define DLLM_CACHE_OFF 0
#define DLLM_CACHE_REFRESH 1
#define DLLM_CACHE_REUSE 2
int dllm_step_cached(dllm_handle *h, int32_t B, int32_t L, int32_t *tokens, uint8_t *mask, int32_t *prev_pred,
                     const dllm_stage_params *sp, const int32_t *cache_mode, const uint8_t *skip,
                     const dllm_commit_list *out);

/* Full SlowFast decode (Algorithm 1) of B sequences that share gen_start and
 * gen_end = L: alternates exploratory (slow) and accelerated (fast) stages per
 * sequence until no [MASK] is left or max_steps steps were taken.  The stage
 * controller runs on the host and reads a few integers per sequence back after
 * every step, so this call is synchronous.  tokens / mask as in dllm_step.
 *   steps_taken host out, number of forward passes
 *   stats       host out, nullable, up to stats_capacity records */
int dllm_decode(dllm_handle *h, int32_t B, int32_t L, int32_t gen_start, int32_t *tokens, uint8_t *mask,
                const dllm_decode_params *p, int32_t *steps_taken, dllm_step_stat *stats, int32_t stats_capacity);

/* The baseline sampler the method is measured against (Section 3.1, "Low-Confidence
 * Remasking", optionally "Semi-Autoregressive"): the generated region [gen_start, L) is
 * cut into blocks of block_len positions that are denoised left to right with
 * n_steps / (number of blocks) steps each; after the j-th of a block's N_b steps the
 * block holds floor(block_len * j / N_b) unmasked tokens, the newly unmasked ones being
 * the most confident masked positions of the block (ties: lower position).  A step
 * whose target a sequence already meets commits nothing there; a step no sequence
 * needs runs no forward pass.  Uses the same step kernels as dllm_decode (the
 * slow-stage rule with top_k from the schedule and the block as window).
 *   block_len   <= 0 means one block over the whole region; must divide L - gen_start
 *   n_steps     a positive multiple of the number of blocks
 * Other arguments, synchronisation and errors as dllm_decode. */
int dllm_decode_low_confidence(dllm_handle *h, int32_t B, int32_t L, int32_t gen_start, int32_t *tokens,
                               uint8_t *mask, int32_t n_steps, int32_t block_len, int32_t *steps_taken,
                               dllm_step_stat *stats, int32_t stats_capacity);

/* Test and measurement hooks: device pointers into the workspace, valid until
 * the next call on the handle.  logits: bf16 [B*L][vocab] of the last forward
 * (after dllm_step only the rows inside each sequence's window are defined:
 * the vocabulary projection skips rows the selector does not read; and none
 * are written by a step while the fused selector is on: DLLM_ESTATE if no
 * call on the handle has written logits yet);
 * pred / conf: int32 / float [B*L] of the last row phase (defined at the
 * masked positions of each window only). */
int dllm_debug_logits(dllm_handle *h, const void **logits);
/* Test hook: the library reads its DLLM_GEMM_* / DLLM_NO_FUSED_ROPE environment switches (kernel and
 * tile selection for tests and tuning) once per process and keeps the launch plan it finds for every
 * product shape; this reads them again and drops the kept plans.  Not for use while another thread is
 * inside the library with work that depends on the old values. */
void dllm_debug_reload_env(void);
/* Measurement hook (runs on the host only): the launch plan the library uses for the product
 * C[M][N] = A[M][K] W[N][K]^T with a given epilogue: 0 bf16 output, 1 gate/up + SwiGLU (N counts gate and
 * up rows), 2 fp32 split-K slabs (O and down projection; split_limit = most slabs allowed, 8 in a step at
 * up to 4096 rows), 3 / 4 QKV + rotary embedding for head_dim 64 / 128, 5 vocabulary projection with the
 * greedy decode.  out8 (host): tile rows, tile columns, K depth of a pipeline stage, pipeline stages, wave
 * grid rows, wave grid columns, K splits, 1 for the asynchronous-copy kernel / 0 for the register-staged one. */
int dllm_debug_gemm_plan(int32_t epilogue, int32_t M, int32_t N, int32_t K, int32_t split_limit, int32_t *out8);
int dllm_debug_rows(dllm_handle *h, const int32_t **pred, const float **conf);
/* Measurement hook: the sustained rate of the bf16 matrix instruction itself (the practical ceiling of the
 * projections: with random operands the chip's power limit sets it well below the nominal peak).  Enqueues one
 * kernel on hip_stream in which each of `workgroups` workgroups of four waves executes iters * 8 instructions
 * v_mfma_f32_32x32x16_bf16 on operands held in registers (32768 flop each, so a launch performs
 * workgroups * 4 * iters * 8 * 32768 flop); the caller times it.  operands (device): n_operands >= 1 pieces of
 * 16 bytes holding the bf16 values to multiply, read once per wave; sink (device): workgroups * 256 floats that
 * receive the accumulator sums.  workgroups and iters in [1, 2^20].  Returns DLLM_EINVAL for a null pointer or a
 * count out of range, DLLM_EHIP if the launch fails. */
int dllm_debug_mfma_rate(void *hip_stream, const void *operands, int32_t n_operands, float *sink,
                         int32_t workgroups, int32_t iters);

/* Measurement hook for the kernel that carries the most flops of a step, the
 * gate/up projection GEMM with the SwiGLU epilogue (one launch per layer):
 * between begin and end every such launch is bracketed by a HIP event pair on
 * the handle's stream, up to max_launches pairs.  dllm_profile_end waits for
 * the stream, returns the summed device time of the bracketed launches and
 * their number, and switches the hook off. */
int dllm_profile_begin(dllm_handle *h, int32_t max_launches);
int dllm_profile_end(dllm_handle *h, float *total_ms, int32_t *launches);

/* Forward only (eq. 2): fills the logits workspace for tokens dev int32 [B][L]. */
int dllm_forward(dllm_handle *h, int32_t B, int32_t L, const int32_t *tokens);

/* The selector alone, on logits the caller provides (eq. 3, the confidence
 * equation, Section 3.3): row phase over the masked positions of each window,
 * then selection and the transition of dllm_step.
 *   logits dev bf16 [B][L][V]; pred / conf dev [B][L] outputs (written at the
 *   masked positions of each window); the rest as in dllm_step.
 * `hip_stream` as in dllm_create.  Requires 0 <= mask_id < V, B <= DLLM_MAX_BATCH,
 * L <= 8192. */
int dllm_select(void *hip_stream, const void *logits, int32_t B, int32_t L, int32_t V, int32_t mask_id,
                int32_t *tokens, uint8_t *mask, int32_t *prev_pred, const dllm_stage_params *sp,
                int32_t *pred, float *conf, const dllm_commit_list *out);

/* ---- building blocks, exposed for per-kernel parity tests and timing -------
 * All pointers dev; all enqueue on `hip_stream`; shapes are validated.        */

/* C[M][N] (bf16) = A[M][K] (bf16) * W[N][K]^T, fp32 accumulation.  K % 8 == 0. */
int dllm_op_linear(void *hip_stream, const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K);
/* out[M][f] = silu(A Wg^T) * (A Wu^T) with W = [gate | up] rows, [2f][K]. */
int dllm_op_linear_swiglu(void *hip_stream, const void *A, const void *W, void *out, int32_t M, int32_t f,
                          int32_t K);
/* Panel-major layout.  Inside a step the library keeps the operands of its projections "panel-major": a
 * matrix X[rows][K] (K % 32 == 0) stored as [K / 32][panel_rows][32], i.e. panel p holds elements
 * [32 p, 32 p + 32) of every row and the 64-byte pieces of consecutive rows follow each other.  A tile's
 * K-stage is then one contiguous block and every request to the L2 a whole 128-byte line (measured: tile
 * copies at 115 instead of 65 GB/s per CU from the L2, 6.3 instead of 4.4 TB/s from HBM).  dllm_create
 * makes panel-major copies of the projection weights whose reduction length is a multiple of 64 (so a
 * handle holds those weights twice: 15 GB more at the LLaDA-8B shape) unless the environment variable
 * DLLM_NO_PACK is set; the two calls below expose the layout for tests and timing.
 *
 * dst (bf16 [K / 32][rows][32]) = src (bf16 [rows][K]). */
int dllm_op_pack_panels(void *hip_stream, const void *src, void *dst, int64_t rows, int32_t K);
/* dllm_op_linear (swiglu == 0) or dllm_op_linear_swiglu (swiglu != 0, N counts gate + up rows) with operands in
 * either layout: a_panel_rows 0 = A row-major [M][K], else A panel-major with that many rows per panel (>= M,
 * A points at the first used row inside panel 0); w_panels != 0 = W panel-major [K / 32][N][32]; c_panel_rows
 * (SwiGLU only, (N / 2) % 32 == 0) likewise for the output.  DLLM_EINVAL if a panel-major operand is given for
 * a shape the asynchronous-copy kernel does not take (K % 64 != 0). */
int dllm_op_linear_panels(void *hip_stream, const void *A, const void *W, void *C, int32_t M, int32_t N, int32_t K,
                          int32_t swiglu, int32_t a_panel_rows, int32_t w_panels, int32_t c_panel_rows);
/* x (fp32 [M][d], in/out) += sum of n_partials fp32 [M][d] slabs (0 to 8);
 * h (bf16 [M][d]) = RMSNorm(x) * gain. */
int dllm_op_add_rmsnorm(void *hip_stream, float *x, const float *partials, int32_t n_partials,
                        const void *gain, void *h, int32_t M, int32_t d, float eps);
/* In-place RoPE on the q and k thirds of qkv bf16 [B*L][3*H*dh]. */
int dllm_op_rope(void *hip_stream, void *qkv, int32_t B, int32_t L, int32_t H, int32_t dh, float theta);
/* Fused QKV projection + RoPE (Section 3.1's bidirectional transformer block; rotary embedding
 * as in LLaDA): qkv bf16 [B*L][3*H*dh] = A[B*L][H*dh] * W[3*H*dh][H*dh]^T with the q and k thirds
 * rotated in fp32 before the single bf16 rounding; row r has position r % L.  `table` is scratch
 * the caller provides, float [L][dh/2][2] dev, filled with (cos, sin) by this call.
 * DLLM_EINVAL if the fused kernel does not cover the shape (dh not 64/128, (H*dh) % 64 != 0). */
int dllm_op_linear_qkv_rope(void *hip_stream, const void *A, const void *W, void *qkv, float *table,
                            int32_t B, int32_t L, int32_t H, int32_t dh, float theta);
/* dllm_op_linear_qkv_rope for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same product, same
 * kernels and bit-identical output, but the rotary table lives in a 4 MiB array built into the library
 * (one copy per GPU, resident until the process ends) instead of caller-provided scratch; the call
 * allocates nothing on the device.  Limit: L * dh / 2 <= 524288 table entries, i.e. L <= 8192 at
 * head_dim 128 and L <= 16384 at head_dim 64 (DLLM_EINVAL beyond, nothing enqueued).  Every call on a GPU
 * rewrites that GPU's one table: calls that may overlap on the same GPU (different streams or threads,
 * unless every one of them uses the same L, dh and theta) race and must be serialised by the caller.
 * Other arguments and errors as dllm_op_linear_qkv_rope. */
int dllm_op_linear_qkv_rope_static(void *hip_stream, const void *A, const void *W, void *qkv, int32_t B, int32_t L,
                                   int32_t H, int32_t dh, float theta);
/* Non-causal attention: qkv bf16 [B*L][3*H*dh] -> out bf16 [B*L][H*dh]. */
int dllm_op_attention(void *hip_stream, const void *qkv, void *out, int32_t B, int32_t L, int32_t H, int32_t dh);

#ifdef __cplusplus
}
#endif
#endif /* DLLM_H */
