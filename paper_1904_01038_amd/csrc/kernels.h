// Host-side launchers of the gfx950 kernels.  Every launcher only enqueues work on the given stream; none of them
// allocates or synchronises.  `dt` is a tfm::DType; all tensor arguments of one call share it unless noted.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace tfm {

// Device-resident state of one context: the loss scaler, the optimiser step counter and per-call results.  It is
// read and written by kernels so that a training step needs no host round trip.
struct DevState {
  float loss_scale;          // S
  int clean_steps;           // clean updates since the last overflow or growth
  long long num_updates;     // optimiser steps taken
  int window_overflow;       // OR of the sub-batch overflow flags of the current window
  int scale_too_small;       // sticky: S fell below the configured minimum
  // last tfm_train_step
  double loss_sum, nll_sum;
  int step_overflow;
  float step_scale;
  // last scan
  float scan_flag;           // 1.0 if a non-finite value was seen
  double scan_sumsq;         // sum of squares of the scanned buffer
  // last tfm_apply_update
  int skipped;
  float grad_norm;
  float grad_mult;           // 1/(S*N) * clip coefficient
  float bc1, bc2;            // 1 - beta^t
};

struct GemmArgs {
  int dt;
  int form;                  // 0 NT, 1 NN, 2 TN
  int M, N, K;
  const void* A; int lda;
  const void* B; int ldb;
  void* C; int ldc;
  const void* bias;          // [N] or null
  int relu;
  const void* mask;          // [M, N] stride ldc or null: multiply by (mask > 0)
  const void* residual;      // [M, N] stride ldc or null: added last (must not alias C)
  void* splitk_ws = nullptr; // optional fp32 workspace that allows split-K for small weight-gradient outputs
  size_t splitk_ws_bytes = 0;
  // Inverted dropout on the result (after bias and ReLU, before mask and residual): element m * N + n is kept when its
  // counter-based bit says so (see common.h) and multiplied by 1 / (1 - drop_p).  drop_p = 0: off.
  uint64_t drop_key = 0;
  float drop_p = 0.f;
  float mask_scale = 1.f;    // with mask: the kept elements are also multiplied by this (the dropout scale of the masked layer)
  // Deferred split-K reduction (host pointer or null).  If given and the launch splits the contraction, the fp32 partial
  // results [splits][M][N] stay in splitk_ws, nothing is written to C, bias is NOT applied, and *deferred_splits = splits:
  // the caller's next kernel adds them up (see launch_splitk_layernorm_fwd).  Otherwise *deferred_splits = 0 and C is complete.
  int* deferred_splits = nullptr;
};
void launch_gemm(hipStream_t s, const GemmArgs& a);
bool gemm_mfma_supported(const GemmArgs& a);
void launch_gemm_naive(hipStream_t s, const GemmArgs& a);
void launch_gemm_mfma(hipStream_t s, const GemmArgs& a);      // requires gemm_mfma_supported(a)
// C[m, n] = bias[n] + sum over s of partial[s][m][n] (fixed order): the second half of a split-K product whose reduction was
// deferred (2-byte types only)
void launch_splitk_reduce(hipStream_t s, int dt, const float* partial, int splits, int M, int N, void* C, int ldc, const void* bias);

// Grouped weight gradients (half precision): one launch computes C_i[M_i, N_i] = A_i^T B_i over K_i rows for every job and,
// where colsum is set, colsum_i[M_i] = the column sums of A_i (the bias gradient that goes with the weight gradient).
struct WgradJob {
  int M, N, K;
  const void* A; int lda;                // [K, M]
  const void* B; int ldb;                // [K, N]
  void* C; int ldc;                      // [M, N]
  void* colsum;                          // [M] or null
};
constexpr int WGRAD_GROUP_MAX = 48;      // jobs per launch
bool wgrad_group_supported(int dt, const WgradJob& j);
void launch_wgrad_grouped(hipStream_t s, int dt, const WgradJob* jobs, int n);   // n <= WGRAD_GROUP_MAX, every job supported

struct AttnArgs {
  int dt;
  const void *q, *k, *v; int ldq, ldk, ldv;
  void* o; int ldo;                      // forward: written; backward: read
  float* lse;                            // [H, total_q]
  const int *q_off, *k_off;              // device [B+1]
  int B, H, dh, max_lq, max_lk, total_q, total_k, causal;
  // backward only
  const void* d_o; int lddo;
  void *dq, *dk, *dv; int lddq, lddk, lddv;
  // Inverted dropout on the attention weights: weight (query row i of the packed stream, head h, key j of the sentence)
  // uses element ((i * H + h) << 16) + j of the counter-based generator (see common.h); drop_p = 0: off.  Forward and
  // backward regenerate the same bits from the key.
  uint64_t drop_key = 0;
  float drop_p = 0.f;
  // Optional packing of short sentences: device int32 [(n_groups + 1) * 4], 16-byte aligned, entry g = {first sentence, first
  // query row, first key row, 0} of group g and a closing entry {B, total query rows, total key rows, 0}.  A group is a run of
  // at most 16 consecutive sentences whose query rows and whose key rows each number at most 64.  Used by the one-chunk kernels
  // when every sentence fits 64 rows and the attention weights have no dropout; null: off.
  const int* groups = nullptr;
  int n_groups = 0;
};
void launch_attention_fwd(hipStream_t s, const AttnArgs& a);
void launch_attention_bwd(hipStream_t s, const AttnArgs& a);
bool attention_mfma_supported(const AttnArgs& a, bool bwd);
void launch_attention_fwd_mfma(hipStream_t s, const AttnArgs& a);
void launch_attention_bwd_mfma(hipStream_t s, const AttnArgs& a);
void launch_attention_fwd_naive(hipStream_t s, const AttnArgs& a);
void launch_attention_bwd_naive(hipStream_t s, const AttnArgs& a);

// The same as launch_residual_layernorm_fwd with y = bias + sum over `splits` fp32 slices partial[s][rows][d] (in that order)
// and no dropout: the reduction of a split-K product fused with the residual connection and LayerNorm that follow it.
void launch_splitk_layernorm_fwd(hipStream_t s, int dt, const void* x, const float* partial, int splits, const void* bias,
                                 const void* gamma, const void* beta, void* s_out, void* n_out, int rows, int d);
void launch_residual_layernorm_fwd(hipStream_t s, int dt, const void* x, const void* y, const void* gamma,
                                   const void* beta, void* s_out, void* n_out, float* mean, float* rstd, int rows,
                                   int d, uint64_t key, float p);
size_t layernorm_bwd_scratch_bytes(int rows, int d);
// The backward kernel leaves per-block partial column sums in `scratch`; a second, tiny kernel adds them in a fixed order
// into dgamma / dbeta / dbias (dbias may be null: then it is not formed).  With `defer` set that second kernel is NOT
// launched: the job is described there instead, scratch must stay untouched until launch_ln_reduce_batched has run it,
// and many such jobs go into one launch.
struct LnReduceJob { const float* partial; int np; int slots; void *dgamma, *dbeta, *dbias; };
constexpr int LN_REDUCE_MAX = 64;        // jobs per launch (more are split over several)
void launch_layernorm_bwd(hipStream_t s, int dt, const void* dn, const void* add, const void* sres, const float* mean,
                          const float* rstd, const void* gamma, void* ds, void* ds_drop, void* dgamma, void* dbeta,
                          void* dbias, int rows, int d, uint64_t key, float p, void* scratch, LnReduceJob* defer = nullptr);
void launch_ln_reduce_batched(hipStream_t s, int dt, const LnReduceJob* jobs, int n, int d);
size_t colsum_scratch_bytes(int rows, int n);
void launch_colsum(hipStream_t s, int dt, const void* x, int ld, int rows, int n, void* out, void* scratch);

// z[rows, V] in place; scale = (scale_ptr ? *scale_ptr : 1) * mult; if step_scale_out != null the applied scale is
// stored there.
void launch_loss(hipStream_t s, int dt, void* z, const int* labels, float* loss_rows, float* nll_rows, int rows, int V,
                 float eps, const float* scale_ptr, float mult, float* step_scale_out);
// sums[0] = sum loss_rows, sums[1] = sum nll_rows (double, single block, fixed order)
void launch_sum_rows(hipStream_t s, const float* loss_rows, const float* nll_rows, int rows, double* sums);

// ids[r] >= 0: row ids[r] of E; ids[r] = -1-k: row k of alt (both d wide)
void launch_embed_fwd(hipStream_t s, int dt, const void* E, const int* ids, const int* pos, const float* pe, void* out,
                      int rows, int d, uint64_t key, float p, const void* alt = nullptr);
// ---- adaptive inputs / adaptive softmax: row movers (index lists from the host) ----------------------------------------
void launch_gather_rows(hipStream_t s, int dt, const void* src, int ld_src, const int* idx, void* dst, int width, int n);
void launch_gather_dx(hipStream_t s, int dt, const void* dx, const int* idx, void* dst, int d, int n, float scale, uint64_t key, float p);
void launch_scatter_add_rows(hipStream_t s, int dt, void* dst, int ld_dst, const int* idx, const void* src, int width, int n);
void launch_scatter_add_f32(hipStream_t s, float* a, float* b, const int* idx, const float* sa, const float* sb, int n);
// virt[r][col0 + j] = z[r][j] + (entry >= 0 ? head[r][entry] - lse[r] : 0), j < width, r < rows (decoding with an adaptive softmax)
void launch_adaptive_virtual(hipStream_t s, int dt, const void* z, int ldz, int width, void* virt, int ldv, int col0, const void* head, int ldh,
                             int entry, const float* lse, int rows);
void launch_segsum_add_rows(hipStream_t s, int dt, void* dst, const void* src, int width, const int* tok, const int* beg, const int* end,
                            const int* entries, int n_seg);
// Adds sqrt(d) * dropout-backward(dx) of every occurrence of a token to its row of the embedding gradient.
// The host supplies occurrence lists cut into segments (see embed.hip); an entry is (stream << 30) | row.
constexpr int EMB_SEG = 32;
struct EmbedBwdArgs {
  int dt; void* gE; float* partial;                  // partial: fp32 [rows of multi-segment tokens, d]
  const int *seg_tok, *seg_beg, *seg_end, *seg_dst;  // per segment: token, entry range, partial row or -1
  const int* entries; int n_seg;
  const int *mt_tok, *mt_row0, *mt_n; int n_multi;   // per multi-segment token: token, first partial row, count
  const void *dx0, *dx1; int d; uint64_t key0, key1; float p;
};
void launch_embed_bwd(hipStream_t s, const EmbedBwdArgs& a);

size_t scan_scratch_bytes(int64_t n);
// flag/sumsq of x[n] -> result[0], result[1] (fp32) and, if st != null, st->scan_flag / scan_sumsq and
// st->step_overflow / window_overflow (|=).  If acc != null: acc = x (acc_mode 1) or acc += x (acc_mode 2), fp32.
void launch_scan(hipStream_t s, int dt, const void* x, int64_t n, float* result, DevState* st, float* acc, int acc_mode,
                 void* scratch);
void launch_convert(hipStream_t s, int src_dt, const void* src, int dst_dt, void* dst, int64_t n);

struct AdamArgs {
  float *w, *m, *v; const void* g; int gdt; void* half_copy; int hdt; int64_t n;
  float lr, beta1, beta2, eps;
  float weight_decay;        // L2 form: weight_decay * w joins the unscaled gradient
  const DevState* st;        // if non-null: skip flag, grad_mult, bc1, bc2 come from the device state
  float grad_mult, bc1, bc2;
};
void launch_adam(hipStream_t s, const AdamArgs& a);
// One-thread kernel: the loss-scale state machine and the Adam step scalars.
void launch_scaler_update(hipStream_t s, DevState* st, long long ntokens, float clip_norm, float beta1, float beta2,
                          int scale_window, float min_scale, int dynamic);
void launch_dropout_mask(hipStream_t s, uint64_t key, float p, uint8_t* out, int64_t n);

// ---- incremental decoding ---------------------------------------------------------------------------------------------
void launch_ancestry(hipStream_t s, const int* anc_old, int* anc_new, const int* parent, int rows, int max_steps, int t);
void launch_cache_append(hipStream_t s, int dt, const void* qkv, void* Kc, void* Vc, int rows, int d, int max_steps, int t);
struct DecodeAttnArgs {
  int dt;
  const void* q; int ldq;                // [rows, ldq], head h at column h * dh
  const void *k, *v;                     // self: caches [rows][max_steps][row_stride]; cross: [src tokens][row_stride]
  int row_stride;                        // elements between consecutive positions (d for the caches, 2d for fused K|V)
  void* o; int ldo;
  const int* anc;                        // self-attention: ancestry table [rows][max_steps]; null selects cross-attention
  const int* src_off;                    // cross-attention: [sentences + 1] row offsets into k / v
  int rows, H, dh, beam, t, max_steps;
  int n_max;                             // upper bound on the positions any row attends to (sizes the LDS buffers)
  // Self-attention only, optional: the step's new keys and values [rows, ld_new] (head h at column h * dh), not yet in the
  // caches.  The kernel then takes position t from here and stores it at position t of the row's own cache lines (k and v
  // must be writable), which saves the separate append.  Honoured only where decode_attention_appends() says so.
  const void *k_new = nullptr, *v_new = nullptr;
  int ld_new = 0;
  // Optional: the query projection left as q_splits fp32 slices [q_splits][rows][H * dh] of a split-K product, without its bias
  // (q_bias [H * dh] or null).  The kernel adds them up while it loads the query; q must then be a writable [rows, ldq] buffer,
  // which receives the sum only where the kernel cannot do that (see launch_decode_attention).
  const float* q_partial = nullptr;
  int q_splits = 0;
  const void* q_bias = nullptr;
};
void launch_decode_attention(hipStream_t s, const DecodeAttnArgs& a);
bool decode_attention_appends(const DecodeAttnArgs& a);   // would this launch append k_new / v_new to the caches itself?
// per row: log-sum-exp and the k (<= 16) largest logits as log-probabilities, best first, ties by ascending id
void launch_row_topk(hipStream_t s, int dt, const void* z, int ldz, int rows, int V, int k, float* top_logp, int* top_id,
                     float* lse);
void launch_logprob_rows(hipStream_t s, int dt, const void* z, int ldz, const float* lse, float* out, int rows, int V);

uint64_t dropout_site_key(uint64_t seed, uint64_t step, int stream, int layer, int sub);

// message tfm_last_error(NULL) returns on this thread (entry points that have no context to hold it)
void set_global_error(const char* msg);

}  // namespace tfm
