/*
 * tfm.h - C boundary of the MI355X (gfx950) mixed-precision Transformer training step.
 *
 * The library implements one path of the paper (fairseq, arXiv 1904.01038): the single-GPU training step of a
 * Transformer encoder-decoder or decoder-only language model (Applications: machine translation; language
 * modeling) with
 *   - loss = criterion(model, batch)                     (Design, Criterions)
 *   - half-precision forward/backward, full-precision parameter update, dynamic loss scaling: the loss is scaled
 *     right after the forward pass, the gradients are unscaled before the update
 *                                                         (Implementation, Mixed precision)
 *   - gradients accumulated over several sub-batches before one update ("delayed updates")
 *                                                         (Implementation, Multi-GPU training)
 *   - an optimiser that updates the parameters from the gradients (Design, Optimizers); here Adam.
 *
 * General rules
 *   - Every function returns 0 on success and a negative TFM_E* code on failure.  Nothing throws, aborts or
 *     prints.  tfm_last_error() gives a human-readable message for the last failure on a context.
 *   - "host" pointers are ordinary CPU memory owned by the caller and may be reused as soon as the call returns.
 *     "device" pointers are HIP device memory owned by the caller.  The library allocates no device memory:
 *     parameters, optimiser state, gradients and activations all live in the caller's workspace.
 *   - One context = one HIP stream = one caller thread at a time.  Work is enqueued on the context's stream;
 *     calls that return results to the host (an `out` struct, tfm_get_*) synchronise that stream.
 *   - Inputs are validated on the host before anything is enqueued: a call that fails with TFM_EINVAL leaves
 *     parameters, gradients and scaler state untouched.
 *   - Same context state + same inputs => bit-identical results (no floating-point atomics anywhere).
 */
#ifndef TFM_H
#define TFM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TFM_OK        0
#define TFM_EINVAL   -1   /* bad config / shape / token id outside [0, vocab) / length out of range / over capacity */
#define TFM_ENOMEM   -2   /* workspace too small */
#define TFM_EHIP     -3   /* a HIP runtime call failed (message holds the HIP error string) */
#define TFM_ESTATE   -4   /* call not allowed in this state, e.g. tfm_apply_update with no accumulated sub-batch */
#define TFM_ESCALE   -5   /* the loss scale fell below min_loss_scale */

#define TFM_FP32 0
#define TFM_FP16 1
#define TFM_BF16 2

typedef struct tfm_ctx tfm_ctx;   /* opaque; created by tfm_create, released by tfm_destroy */

typedef struct {
  int32_t enc_layers;       /* 0 = decoder-only language model (src must then be NULL)                      */
  int32_t dec_layers;       /* >= 1                                                                          */
  int32_t d_model;          /* model width d; multiple of 8                                                  */
  int32_t n_heads;          /* d_model % n_heads == 0; head width d_h = d_model / n_heads <= 128             */
  int32_t d_ffn;            /* feed-forward inner width F; multiple of 8                                     */
  int32_t vocab;            /* V; one shared embedding table, output projection tied to it, no output bias   */
  int32_t pad_id, eos_id;   /* padding id (ignored everywhere) and end-of-sentence id                        */
  int32_t max_sentences;    /* capacity: sentences per sub-batch                                             */
  int32_t max_len;          /* capacity: longest source or target sentence                                   */
  int32_t max_tokens;       /* capacity: non-pad tokens per sub-batch on either side                         */
  int32_t precision;        /* TFM_FP32 | TFM_FP16 (dynamic loss scaling) | TFM_BF16 (scale fixed at its initial value) */
  int32_t pre_norm;         /* 0: LayerNorm after each residual sum; 1: before each sub-layer + a final one  */
  float   dropout;          /* on embeddings and on each sub-layer output before the residual sum; [0, 1)    */
  float   attn_dropout;     /* on the attention weights, after the softmax; [0, 1)                           */
  float   relu_dropout;     /* on the feed-forward hidden activations, after the ReLU; [0, 1)                */
  float   label_smoothing;  /* eps in q = (1-eps) onehot + eps/V                                             */
  float   adam_beta1, adam_beta2, adam_eps;
  float   weight_decay;     /* L2 form: weight_decay * w joins the unscaled (and clipped) gradient; 0 = off  */
  float   clip_norm;        /* 0 = off; else the unscaled gradient is scaled down to this L2 norm            */
  float   init_loss_scale;  /* a power of two; use 1 for fp32/bf16                                           */
  int32_t scale_window;     /* clean updates after which the scale doubles                                   */
  float   min_loss_scale;   /* tfm_apply_update reports TFM_ESCALE below this                                */
  uint64_t seed;            /* dropout seed; parameters are set by the caller                                */
  /* Adaptive input embeddings and adaptive softmax (Applications, language modeling); decoder-only models with
   * label_smoothing = 0.  n_cutoffs = 0: one flat tied table.  Otherwise the vocabulary (sorted by frequency) is
   * the head [0, cutoffs[0]) plus n_cutoffs tail clusters [cutoffs[i-1], cutoffs[i]), the last ending at vocab; tail
   * cluster i has a table "embed.i" [V_i, d_model / adaptive_factor^i] and a projection "embed.i.proj"
   * [d_model, d_model / adaptive_factor^i], both shared by the input and the output side, and "embed" holds the
   * head's cutoffs[0] tokens followed by one output row per tail cluster.  The matrix-core kernels serve tables
   * whose row counts (cutoffs[0] + n_cutoffs, every V_i) and widths are multiples of 8; other sizes run on the
   * generic kernels. */
  int32_t n_cutoffs;        /* 0 .. 3 */
  int32_t cutoffs[3];
  int32_t adaptive_factor;  /* >= 1 when n_cutoffs > 0 */
} tfm_config;

typedef struct {
  double  loss_sum;         /* sum over non-pad target tokens of the label-smoothed loss, nats, NOT scaled   */
  double  nll_sum;          /* same for the plain negative log-likelihood                                    */
  int64_t ntokens;          /* non-pad target tokens of this sub-batch                                       */
  int32_t overflow;         /* 1 if this sub-batch produced a non-finite gradient value                      */
  float   loss_scale;       /* scale that was applied                                                        */
} tfm_step_out;

typedef struct {
  int32_t skipped;          /* 1: overflow in the window, nothing was updated                                */
  float   loss_scale_after;
  int32_t clean_steps;      /* clean updates since the last overflow or growth                               */
  int64_t num_updates;      /* optimiser steps taken so far                                                  */
  float   grad_norm;        /* L2 norm of the unscaled, token-normalised gradient (NaN when skipped)         */
  int64_t ntokens_total;    /* target tokens in the window                                                   */
} tfm_update_out;

/* Bytes of device workspace tfm_create needs for this configuration. */
int tfm_workspace_bytes(const tfm_config* cfg, size_t* bytes);

/* Create a context.  dev_workspace: device memory, 256-byte aligned, at least tfm_workspace_bytes() long, owned
 * by the caller and kept alive until tfm_destroy; its contents are initialised here (parameters and optimiser
 * state zero).  hip_stream: a hipStream_t (NULL = the default stream). */
int tfm_create(const tfm_config* cfg, void* dev_workspace, size_t bytes, void* hip_stream, tfm_ctx** out);
void tfm_destroy(tfm_ctx* ctx);                      /* does not free the workspace */
const char* tfm_last_error(const tfm_ctx* ctx);      /* ctx may be NULL: message of the last failed tfm_create */

/* Parameters: addressed by index, identified by name (tfm_param_info); the index order is the library's memory order and
 * carries no meaning of its own (the key/value projections "dec.<l>.cross.wkv" / ".bkv" of all decoder layers are stored
 * back to back, ahead of the decoder's other parameters, so that one product serves every layer).  Matrices are
 * row-major W[out, in] (y = x W^T + b). */
int tfm_num_params(const tfm_ctx* ctx, int32_t* n);
int tfm_param_info(const tfm_ctx* ctx, int32_t i, char name[64], int64_t shape[2]);   /* shape[1] = 0 for vectors */
int tfm_set_param(tfm_ctx* ctx, int32_t i, const float* host, int64_t n);  /* sets the fp32 master and the half copy */
int tfm_get_param(tfm_ctx* ctx, int32_t i, float* host, int64_t n);        /* fp32 master                             */
/* Accumulated gradient of the current window as fp32, still multiplied by the loss scale, not token-normalised. */
int tfm_get_grad(tfm_ctx* ctx, int32_t i, float* host, int64_t n);
/* Adam moments (which = 0: first, 1: second). */
int tfm_get_adam(tfm_ctx* ctx, int32_t i, int32_t which, float* host, int64_t n);
int tfm_set_adam(tfm_ctx* ctx, int32_t i, int32_t which, const float* host, int64_t n);
/* tfm_get_scaler fills its outputs and then returns TFM_ESCALE if the scale is below min_loss_scale; tfm_set_scaler
 * with a scale at or above the minimum clears that condition. */
int tfm_get_scaler(tfm_ctx* ctx, float* loss_scale, int32_t* clean_steps, int64_t* num_updates);
int tfm_set_scaler(tfm_ctx* ctx, float loss_scale, int32_t clean_steps, int64_t num_updates);

/* One sub-batch: forward, loss (scaled right after the forward pass), backward; gradients are added to the
 * window's accumulator (Implementation, Mixed precision; Multi-GPU training).
 *   src, tgt        host, int32, row-major [B, Ls] and [B, Lt], right-padded with pad_id.  src = NULL (and
 *                   src_lens = NULL, Ls = 0) for the decoder-only model.
 *   src_lens,tgt_lens host, int32 [B], 1 <= len <= L*.  Positions beyond len are ignored.
 *   The decoder is fed eos followed by the target without its last token (teacher forcing); the loss runs over
 *   all tgt_lens[b] target tokens.
 *   out             host, may be NULL: then nothing is copied back and the call does not synchronise.
 * With out != NULL the call returns TFM_ESCALE (out is filled, the sub-batch has been accumulated) if an earlier
 * unsynchronised tfm_apply_update left the loss scale below min_loss_scale. */
int tfm_train_step(tfm_ctx* ctx, const int32_t* src, const int32_t* tgt, const int32_t* src_lens,
                   const int32_t* tgt_lens, int32_t B, int32_t Ls, int32_t Lt, tfm_step_out* out);

/* End of the window: inf/nan scan; on overflow skip, halve the scale; else unscale, normalise by the window's
 * target tokens, optional clipping, Adam step in fp32 on the master weights, refresh the half copy; the scale
 * doubles after scale_window clean updates.  Clears the accumulator.  Returns TFM_ESCALE (out is filled) when the
 * scale has fallen below min_loss_scale; the condition ends as soon as the scale is back at or above it (growth, or
 * tfm_set_scaler).  out may be NULL: no synchronisation, and a too-small scale is then reported by the next
 * tfm_train_step with out != NULL, tfm_apply_update with out != NULL or tfm_get_scaler. */
int tfm_apply_update(tfm_ctx* ctx, float lr, tfm_update_out* out);

/* The backward pass enqueues weight-gradient GEMMs and bias column sums on a second stream that the context owns
 * (non-blocking, default priority), ordered against hip_stream with events and joined before tfm_train_step's
 * inf/nan scan, so callers see one stream's semantics.  on = 0 puts everything on hip_stream; the results are
 * bit-identical either way.  Default: on. */
int tfm_set_overlap(tfm_ctx* ctx, int32_t on);

/* Test hook: the NEXT tfm_train_step multiplies its loss scale by mult (forces an overflow with 1e6 or inf). */
int tfm_debug_set_loss_multiplier(tfm_ctx* ctx, float mult);

/* Profiling: when on, every kernel launch is bracketed by HIP events on the context's stream and its duration is
 * added to its class.  tfm_profile_read synchronises and returns, per class, launches, total milliseconds and the
 * algorithmic flops and bytes the launches were credited with.  Classes: see TFM_PROF_*. */
#define TFM_PROF_GEMM      0
#define TFM_PROF_ATTENTION 1
#define TFM_PROF_NORM      2   /* residual + dropout + LayerNorm forward and backward, bias column sums */
#define TFM_PROF_LOSS      3
#define TFM_PROF_EMBED     4
#define TFM_PROF_OPTIM     5   /* inf/nan scan, accumulation, Adam */
#define TFM_PROF_CLASSES   6
typedef struct { int64_t launches; double ms; double flops; double bytes; } tfm_prof_entry;
int tfm_profile_enable(tfm_ctx* ctx, int32_t on);
int tfm_profile_read(tfm_ctx* ctx, tfm_prof_entry out[TFM_PROF_CLASSES], int32_t reset);

/* ---- measurement aids: what this device sustains, to print beside the published peaks -------------------------------
 * tfm_probe_mfma: a register-only loop of 32x32x16 matrix-core instructions (dtype TFM_FP16 or TFM_BF16) on every
 * compute unit; *tflops receives the rate.  scratch: device memory, at least 2048 bytes per compute unit (256 CUs:
 * 512 KiB), written with throw-away values.  tfm_probe_copy: a copy kernel of `bytes` (a multiple of 16, both pointers
 * 16-byte aligned, no overlap; at most 2^31 x 4 KiB) in the fastest form found on this device - one 16-byte non-temporal load
 * and store per thread, no loop - timed over 10 launches; *gbs receives (bytes read + bytes written) per second.  Both block until the measurement is done. */
int tfm_probe_mfma(int32_t dtype, void* scratch, size_t scratch_bytes, double* tflops, void* stream);
int tfm_probe_copy(void* dst, const void* src, size_t bytes, double* gbs, void* stream);
/* tfm_probe_fetch: the rate at which compute units pull data in: one 16-wavefront block per compute unit re-reads its own
 * region of region_bytes (a multiple of 16 KiB) with 16-byte loads.  64 KiB regions stay in the XCDs' L2 caches (the GEMMs'
 * operand-tile path when panels are shared inside an XCD); 512 KiB regions (128 MiB in all) are served by the memory side
 * through the fabric (the path of every panel's first touch in an XCD).  buf: device memory (contents irrelevant, read only
 * except for 16 KiB at its end), at least compute units x region_bytes + 16 KiB, else TFM_ENOMEM.  Blocks until done. */
int tfm_probe_fetch(const void* buf, size_t bytes, size_t region_bytes, double* gbs_per_cu, double* gbs_total, void* stream);

/* ---- single operations on caller-owned device buffers (used by the kernel-level parity tests) ---------------
 * dtype: TFM_FP32 / TFM_FP16 / TFM_BF16 for every tensor argument unless stated.  stream: hipStream_t or NULL.  */

/* C[M,N] = epilogue(op(A) op(B)).  form 0 "NT": A[M,K], B[N,K];  1 "NN": A[M,K], B[K,N];  2 "TN": A[K,M], B[K,N].
 * lda/ldb/ldc are row strides in elements.  epilogue: + bias[N] (may be NULL), ReLU if relu != 0, multiply by
 * (mask[m,n] > 0) if mask != NULL (row stride ldc), + residual[m,n] if residual != NULL (row stride ldc; must not
 * overlap C). */
int tfm_op_gemm(int32_t dtype, int32_t form, int32_t M, int32_t N, int32_t K, const void* A, int32_t lda,
                const void* B, int32_t ldb, void* C, int32_t ldc, const void* bias, int32_t relu,
                const void* mask, const void* residual, void* stream);

/* Same as tfm_op_gemm with a caller-owned fp32 device workspace.  With it the "TN" form without epilogue may split K
 * across blocks when the output has few tiles (weight gradients); partial tiles are added in a fixed order, so the
 * result stays reproducible.  workspace may be NULL (then identical to tfm_op_gemm).
 * Two more epilogue steps, as the feed-forward layer with dropout on its hidden activations needs them: drop_p > 0
 * applies inverted dropout after bias and ReLU (element m * N + n of the counter-based generator with key drop_key,
 * kept values multiplied by 1 / (1 - drop_p)); with mask, the kept elements are also multiplied by mask_scale (pass 1
 * otherwise). */
int tfm_op_gemm_ws(int32_t dtype, int32_t form, int32_t M, int32_t N, int32_t K, const void* A, int32_t lda,
                   const void* B, int32_t ldb, void* C, int32_t ldc, const void* bias, int32_t relu,
                   const void* mask, const void* residual, void* workspace, size_t workspace_bytes, uint64_t drop_key,
                   float drop_p, float mask_scale, void* stream);

/* Grouped weight gradients, the form every linear layer's backward pass ends in (accumulated gradients of Implementation,
 * Multi-GPU training, are sums of exactly these): for i < n (n <= 48), C_i[M_i, N_i] = A_i^T B_i with A_i[K_i, M_i],
 * B_i[K_i, N_i], and, where colsum[i] != NULL, colsum[i][m] = sum over k of A_i[k, m] (the bias gradient), all in ONE
 * launch.  dims: host int32 [n][6] = M, N, K, lda, ldb, ldc (row strides in elements); A, B, C, colsum: host arrays of
 * n device pointers (colsum itself may be NULL).  dtype TFM_FP16 or TFM_BF16 only; M, N and the strides multiples of 8,
 * pointers 16-byte aligned, else TFM_EINVAL and nothing is launched.  Outputs must not overlap inputs or each other. */
int tfm_op_wgrad_grouped(int32_t dtype, int32_t n, const int32_t* dims, const void* const* A, const void* const* B,
                         void* const* C, void* const* colsum, void* stream);

/* Multi-head attention over packed sentences.  q rows of sentence b are q_off[b]..q_off[b+1], keys/values
 * k_off[b]..k_off[b+1] (device int32 [B+1]).  Head h uses columns h*dh..(h+1)*dh.  o = softmax(q k^T/sqrt(dh)
 * [+ causal mask]) v; lse (device fp32 [H, q_off[B]]) receives the row log-sum-exp of the scaled scores.
 * drop_p > 0: inverted dropout on the attention weights; weight (packed query row i, head h, key j of the sentence)
 * uses element ((i * H + h) << 16) + j of the counter-based generator with key drop_key.  The backward call must be
 * given the same key and probability.
 * groups (device int32 [(n_groups + 1) * 4], 16-byte aligned, or NULL with n_groups = 0): optional packing of short
 * sentences.  Entry g is {first sentence, first query row, first key row, 0} of group g, the closing entry {B, total_q,
 * total_k, 0}; a group is a run of at most 16 consecutive sentences whose query rows and whose key rows each number at most
 * 64.  When max_lq and max_lk are both at most 64 and drop_p = 0, one block then serves a whole group (the products run
 * over the group's 64-row tiles and a weight counts only inside a sentence); otherwise the table is ignored.  The results
 * do not depend on it. */
int tfm_op_attention_fwd(int32_t dtype, const void* q, int32_t ldq, const void* k, int32_t ldk, const void* v,
                         int32_t ldv, void* o, int32_t ldo, float* lse, const int32_t* q_off, const int32_t* k_off,
                         int32_t B, int32_t H, int32_t dh, int32_t max_lq, int32_t max_lk, int32_t total_q,
                         int32_t causal, uint64_t drop_key, float drop_p, const int32_t* groups, int32_t n_groups,
                         void* stream);
int tfm_op_attention_bwd(int32_t dtype, const void* q, int32_t ldq, const void* k, int32_t ldk, const void* v,
                         int32_t ldv, const void* o, int32_t ldo, const void* d_o, int32_t lddo, const float* lse,
                         void* dq, int32_t lddq, void* dk, int32_t lddk, void* dv, int32_t lddv,
                         const int32_t* q_off, const int32_t* k_off, int32_t B, int32_t H, int32_t dh,
                         int32_t max_lq, int32_t max_lk, int32_t total_q, int32_t total_k, int32_t causal,
                         uint64_t drop_key, float drop_p, const int32_t* groups, int32_t n_groups, void* stream);

/* s = x + dropout(y) (y may be NULL: s = x), n = gamma * (s - mean)/sqrt(var + 1e-5) + beta.  [rows, d], contiguous.
 * s_out may be NULL.  mean, rstd: device fp32 [rows].  gamma/beta in `dtype`.  dropout: keep bits from (key, p). */
int tfm_op_residual_layernorm_fwd(int32_t dtype, const void* x, const void* y, const void* gamma, const void* beta,
                                  void* s_out, void* n_out, float* mean, float* rstd, int32_t rows, int32_t d,
                                  uint64_t drop_key, float p, void* stream);
/* ds = add + LayerNorm-backward(dn) (add may be NULL); ds_drop = dropout-backward(ds) if p > 0 (else untouched);
 * dgamma/dbeta [d]; dbias [d] = column sums of dropout-backward(ds) (may be NULL).  scratch: device fp32, at least
 * tfm_op_layernorm_bwd_scratch(rows, d) bytes. */
size_t tfm_op_layernorm_bwd_scratch(int32_t rows, int32_t d);
int tfm_op_layernorm_bwd(int32_t dtype, const void* dn, const void* add, const void* s, const float* mean,
                         const float* rstd, const void* gamma, void* ds, void* ds_drop, void* dgamma, void* dbeta,
                         void* dbias, int32_t rows, int32_t d, uint64_t drop_key, float p, void* scratch,
                         void* stream);

/* Fused log-softmax + label-smoothed cross-entropy, forward and backward, in place: z[rows, V] (row stride V) is
 * overwritten with scale * (softmax(z) - q), q = (1-eps) onehot(label) + eps/V.  loss_rows / nll_rows: device
 * fp32 [rows], unscaled, nats. */
int tfm_op_loss(int32_t dtype, void* z, const int32_t* labels, float* loss_rows, float* nll_rows, int32_t rows,
                int32_t V, float eps, float scale, void* stream);

/* Adam on a flat fp32 range with gradient g (dtype gdtype) pre-multiplied by 1/inv_scale:
 * gg = g * grad_mult + weight_decay * w; m = b1 m + (1-b1) gg; v = b2 v + (1-b2) gg^2;
 * w -= lr * (m/bc1) / (sqrt(v/bc2) + eps); half copy (dtype hdtype, may be NULL) = w. */
int tfm_op_adam(float* w, float* m, float* v, const void* g, int32_t gdtype, void* half_copy, int32_t hdtype,
                int64_t n, float lr, float beta1, float beta2, float eps, float weight_decay, float grad_mult,
                float bc1, float bc2, void* stream);

/* result[0] = 1.0f if any element of x[n] is non-finite else 0; result[1] = sum of squares (fp32 device [2]). */
int tfm_op_scan(int32_t dtype, const void* x, int64_t n, float* result, void* scratch, void* stream);
size_t tfm_op_scan_scratch(int64_t n);

/* tfm_op_scan for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same kernels and the same result, bit for bit, with the per-block
 * partial results kept in a 16 KiB device array that the library holds on every GPU it runs on until the process ends.
 * The call allocates and frees nothing.  x (device, `dtype`, n elements, n a multiple of 8) and result (device fp32 [2])
 * are the caller's.  n above TFM_SCAN_NOALLOC_MAX_N returns TFM_EINVAL; tfm_last_error(NULL) then names the limit, or
 * the HIP error for TFM_EHIP.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race on it and must be serialised by the caller.  Nothing needs clearing between calls: every
 * launch overwrites the entries it later reads. */
#define TFM_SCAN_NOALLOC_MAX_N ((int64_t)1 << 31)
int tfm_op_scan_noalloc(int32_t dtype, const void* x, int64_t n, float* result, void* stream);

/* Dropout keep bits of (key, p) for elements [0, n): out[i] = 1 or 0 (device uint8). */
int tfm_op_dropout_mask(uint64_t key, float p, uint8_t* out, int64_t n, void* stream);
/* Host helper: the 64-bit key of a dropout site (stream 0 encoder / 1 decoder; layer -1 = embedding;
 * sub 0 self-attention, 1 cross-attention, 2 feed-forward) at a training step. */
uint64_t tfm_dropout_key(uint64_t seed, uint64_t step, int32_t stream, int32_t layer, int32_t sub);

/* ---- Incremental decoding (Implementation, Inference) ------------------------------------------------------
 * Step-wise prediction over a per-row key/value cache: a step feeds ONE new token per row and returns the
 * distribution over the next one.  Rows are sentences x beam, row = sentence * beam + slot.  The decoder borrows the
 * context's parameters (their current half/fp32 model copy), stream and encoder buffers during tfm_decoder_begin and
 * keeps its own copy of everything a step needs afterwards (projected source keys/values, source offsets).  A batch
 * stays valid only while the context's parameters do: after any tfm_train_step, tfm_apply_update or tfm_set_param on
 * the context, tfm_decoder_step returns TFM_ESTATE until tfm_decoder_begin starts a batch again.  Dropout is off.
 * The search itself (which beams continue, length penalty, stopping) is the caller's: it passes, per row, the token to
 * feed and the row whose history this row continues.  Models with adaptive inputs / an adaptive softmax (n_cutoffs > 0) are
 * decoded the same way: the returned log-probabilities are log p_head(token) for a head token and log p_head(cluster entry) +
 * log p_cluster(token) for a token of a tail cluster (Applications, language modeling). */
typedef struct tfm_decoder tfm_decoder;

/* max_rows: sentences x beam; max_steps <= config.max_len: positions a hypothesis may reach; max_src_tokens: source
 * tokens of a batch (ignored for a decoder-only model); topk in [1, 16]: candidates returned per row and step. */
int tfm_decoder_workspace_bytes(const tfm_ctx* ctx, int32_t max_rows, int32_t max_steps, int32_t max_src_tokens,
                                int32_t topk, size_t* bytes);
/* dev_workspace: device memory, 256-byte aligned, owned by the caller, alive until tfm_decoder_destroy. */
int tfm_decoder_create(tfm_ctx* ctx, void* dev_workspace, size_t bytes, int32_t max_rows, int32_t max_steps,
                       int32_t max_src_tokens, int32_t topk, tfm_decoder** out);
void tfm_decoder_destroy(tfm_decoder* dec);

/* Start a batch of B sentences with `beam` rows each: runs the encoder once over the sources (host int32
 * [B, Ls] right-padded, lengths [B]; both NULL for a decoder-only model) and projects its output to every decoder
 * layer's cross-attention keys and values; empties the caches. */
int tfm_decoder_begin(tfm_decoder* dec, const int32_t* src, const int32_t* src_lens, int32_t B, int32_t Ls,
                      int32_t beam);

/* Step t = 0, 1, ...: row r consumes token prev[r] at position t (t = 0: the caller passes eos); its history is
 * the one row parent[r] had after the previous step (same sentence; NULL = every row continues itself).
 * prev, parent: host int32 [rows].  Outputs, host, [rows, topk]: the topk largest log-probabilities of the next
 * token (fp32, natural log, computed from the logits in the compute dtype), best first, equal values in ascending
 * id order, and their token ids.  Synchronises. */
int tfm_decoder_step(tfm_decoder* dec, const int32_t* prev, const int32_t* parent, float* top_logp,
                     int32_t* top_id);

/* Test access: log-probabilities over the whole vocabulary of the last step, host fp32 [rows, vocab]. */
int tfm_decoder_get_logprobs(tfm_decoder* dec, float* host, int64_t n);

/* ---- Steps on either side of the training step (host code, host pointers) --------------------------------- */

/* Inverse-square-root learning-rate schedule (Components, Learning Rate Schedulers; the schedule of the
 * Transformer paper it cites): update t = 1, 2, ... gets
 *   t <= warmup:  init_lr + (peak_lr - init_lr) * t / warmup        (linear warm-up)
 *   t >  warmup:  peak_lr * sqrt(warmup / t)
 * With init_lr = 0 and peak_lr = (d_model * warmup)^-1/2 this is d_model^-1/2 * min(t^-1/2, t * warmup^-3/2).
 * warmup = 0 means no warm-up: peak_lr / sqrt(max(t, 1)).  Returns NaN for t < 0 or warmup < 0. */
double tfm_lr_inverse_sqrt(int64_t t, int64_t warmup, double peak_lr, double init_lr);

/* Cyclical learning-rate schedule with warm restarts (Components, Learning Rate Schedulers: "cyclical schedulers
 * based on warm restarts", the cosine schedule of the work cited there).  Update t = 1, 2, ...:
 *   t <= warmup:  init_lr + (max_lr - init_lr) * t / warmup         (linear warm-up; warmup = 0: none)
 *   afterwards cycle i = 0, 1, ... lasts T_i = period * t_mult^i updates and runs
 *                 min_lr + (max_lr * shrink^i - min_lr) * (1 + cos(pi * T_cur / T_i)) / 2,
 * T_cur = updates since the cycle began (0 at its first update, which therefore runs at the cycle's maximum).
 * period > 0, t_mult >= 1 (need not be integers); returns NaN otherwise or for t < 0, warmup < 0. */
double tfm_lr_cosine_restarts(int64_t t, int64_t warmup, double max_lr, double min_lr, double period, double t_mult,
                              double shrink, double init_lr);

/* Token-capped batches of sentences of similar length (Implementation, Batching).  Sentences are ordered by
 * (max(src_len, tgt_len), index) ascending and cut greedily: a batch takes the next sentence while
 * (sentences + 1) * (longest sentence so far in the batch, counting the candidate) <= max_tokens and
 * sentences < max_sentences.  If multiple > 1, a batch that closed with at least `multiple` sentences keeps the
 * largest multiple of `multiple` and hands the rest to the next batch; no sentence is dropped.
 *   src_lens   host int32 [n] or NULL (language model: only tgt_lens counts)
 *   tgt_lens   host int32 [n], every length >= 1 and <= max_tokens, else TFM_EINVAL
 *   order      host int64 [n]      out: sentence indices, batch after batch
 *   batch_begin host int64 [n + 1] out: batch b is order[batch_begin[b] .. batch_begin[b+1]); entries after
 *              n_batches are not written
 * The content of every batch is a pure function of the lengths, so it stays the same from epoch to epoch. */
int tfm_batch_by_length(const int32_t* src_lens, const int32_t* tgt_lens, int64_t n, int32_t max_tokens,
                        int32_t max_sentences, int32_t multiple, int64_t* order, int64_t* batch_begin,
                        int64_t* n_batches);

/* The order in which an epoch visits the batches (Implementation, Batching: batches are shuffled every epoch).
 * perm (host int64 [n_batches]) receives a permutation of 0..n_batches-1 that depends only on (seed, epoch):
 * a Fisher-Yates shuffle, i = n-1 down to 1, swapping position i with position r_i mod (i + 1), where r_i is the
 * 64-bit splitmix64 finaliser of seed + 0x9E3779B97F4A7C15 * (epoch * 2^32 + i + 1). */
int tfm_shuffle_batches(int64_t n_batches, uint64_t seed, uint64_t epoch, int64_t* perm);

#ifdef __cplusplus
}
#endif
#endif
