// C boundary and step scheduler of the training step: configuration checks, carving of the caller's workspace,
// host-side ingest (packing the padded batch into an un-padded token stream), and the static forward/backward/
// update kernel schedule.  No device memory is allocated here; one small pinned host buffer stages the token ids.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/tfm.h"
#include "kernels.h"
#include "common.h"

using namespace tfm;

namespace {

thread_local char g_create_error[256] = "";

struct Param {
  std::string name;
  int64_t rows, cols;      // cols = 0 for vectors
  int64_t off;             // element offset in the flat buffers
  int64_t numel() const { return cols ? rows * cols : rows; }
};

enum Kind { SELF = 0, CROSS = 1, FFN = 2 };

struct Block {
  Kind kind;
  int layer;
  int w_a, b_a;            // wqkv | wq | w1
  int w_kv, b_kv;          // cross-attention only
  int w_o, b_o;            // wo | w2
  int ln_g, ln_b;
  void* inter;             // qkv [R,3d] | q [R,d] | h [R,F]
  void* kv;                // cross: [R,2d] over source rows
  void* ctx;               // attention output [R,d]
  float* lse;              // [H,R]
  // Backward: the gradients the block's weight gradients are formed from.  Each block keeps its own, so the weight
  // gradients of many blocks can be deferred and computed together (see flush_wgrads).
  void* dy;                // [R,d]: gradient w.r.t. the sub-layer output (after dropout-backward)
  void* dint;              // gradient w.r.t. inter: [R,3d] | [R,d] | [R,F]
  void* dkv;               // cross: [R,2d] over source rows
};

struct Stream {
  int id;                  // 0 encoder, 1 decoder
  std::vector<Block> blocks;
  std::vector<void*> resid, norm;          // K+1 each
  std::vector<float*> mean, rstd;          // K+1 each
  int lnf_g = -1, lnf_b = -1;
  int *ids = nullptr, *pos = nullptr, *off = nullptr;   // device
  int rows = 0, max_len = 0;               // current batch
};

struct Arena {
  char* base;
  size_t off = 0;
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

constexpr int STAGE_SLOTS = 4;

// Adaptive input embeddings / adaptive softmax (language model).  Cluster 0 is the head, clusters 1..n the tails.
struct Adaptive {
  int n = 0;                               // tail clusters (0: flat vocabulary)
  int lo[4], hi[4], width[4];              // token range and embedding width per cluster
  int E[4], P[4];                          // parameter indices of a tail cluster's table and projection
  int v0;                                  // rows of "embed": the head's tokens plus one row per tail cluster
  int vmax;                                // largest tail cluster
  // device buffers
  void *Xc[4], *dXc[4], *U[4], *dU[4];     // [R, width]: gathered narrow rows (input side), their gradient; projected states
  void *Y, *dY, *Hc, *dHc;                 // [R, d]: projected inputs, their gradient; gathered states, their gradient
  void* tmpP[4];                           // [d, width]: the output side's projection gradient until the input side adds its own
  float *tail_loss, *tail_nll;             // [R]
  int *in_idx, *in_tok, *out_idx, *out_lab, *sg_tok, *sg_beg, *sg_end, *sg_ent;   // [R] each, filled per step
  // this step's counts (host)
  int in_cnt[4], in_off[4], out_cnt[4], out_off[4], sg_cnt[4], sg_off[4];
  int cluster_of(int id) const {
    int c = 0;
    while (c < n && id >= hi[c]) ++c;
    return c;
  }
};

struct ProfRec { int cls; hipEvent_t a, b; double flops, bytes; };

}  // namespace

struct tfm_ctx {
  tfm_config cfg;
  hipStream_t stream;
  // Weight gradients and bias column sums have no consumer before the end of the backward pass, so they run on a
  // second stream beside the chain of input gradients and fill the compute units that chain leaves idle.
  hipStream_t side;
  bool overlap;
  std::vector<hipEvent_t> sync_ev;                  // ordering events, handed out in sequence within a step
  size_t sync_used;
  // Deferred weight gradients: queued while the chain of input gradients runs, launched as grouped GEMMs (one launch
  // for the tiles of many projections) on the side stream.
  std::vector<WgradJob> wq;
  std::vector<double> wq_flops;
  long wq_tiles;
  long wq_flush_tiles;                              // flush once this many 128x128 tiles are queued
  // Deferred reductions of the LayerNorm backward kernels' partial column sums: each launch keeps its partials in its own
  // slice of ln_pool, and one batched kernel adds them up at the next flush.
  std::vector<LnReduceJob> lnq;
  char* ln_pool;
  size_t ln_slice;
  int ln_slices, ln_next;
  // Cross-attention keys and values of all decoder layers: one [rows, layers * 2d] activation (layer l's keys at column
  // l * 2d, its values at l * 2d + d) written by one product with the stacked weights, and its gradient likewise.
  int kv_w0, kv_b0;                                 // first stacked weight / bias parameter (-1: no encoder)
  void *kv_all, *dkv_all;
  int ld_kv;                                        // layers * 2d
  hipEvent_t kv_ready;                              // side-stream mark after that product (null: it ran on the main stream)
  // The Adam step also runs on the side stream, cut into chunks in the order the forward pass first touches the
  // parameters (the flat order), so the next sub-batch's forward pass starts while later layers are still being
  // updated: it waits chunk by chunk.  Every other entry point first waits for the whole update.
  struct Chunk { int64_t off, n; int last_param; };
  std::vector<Chunk> chunks;
  std::vector<int> chunk_of;                        // parameter index -> chunk
  std::vector<hipEvent_t> adam_ev;                  // one per chunk
  bool adam_pending;
  int adam_waited;                                  // chunks the main stream already waits for
  char err[256];
  int dt;                  // compute dtype
  size_t esz;              // its size
  std::vector<Param> params;
  int64_t P;               // padded flat length
  float *W, *M, *V, *G;    // fp32 master, Adam moments, window accumulator
  void *Wh, *g;            // model copy and sub-batch gradient in compute dtype (Wh == W in fp32 mode)
  DevState* st;
  Stream enc, dec;
  int R;                   // row capacity
  // scratch
  void *demb[2];           // gradient w.r.t. the embedding output of the encoder / decoder stream
  void *y, *dcur, *dsA, *dsB, *dctx, *dmem, *logits;
  float *loss_rows, *nll_rows, *pe;
  void *red_scratch, *scan_scratch, *splitk_ws;
  void *red_scratch_side, *splitk_ws_side;          // the side stream's own reduction scratch
  size_t splitk_bytes;
  int *labels, *uentries, *ibase;                   // device ints (ibase = start of the int block)
  int *seg_tok, *seg_beg, *seg_end, *seg_dst, *mt_tok, *mt_row0, *mt_n;
  int* grp[3];                                      // sentence groups for the packed attention kernels (4 ints per entry): encoder self, decoder self, cross
  float* emb_partial;
  size_t int_block_ints;
  Adaptive ad;
  std::vector<std::pair<int, int>> ad_pairs;
  // host staging
  int* stage[STAGE_SLOTS];
  hipEvent_t stage_ev[STAGE_SLOTS];
  bool stage_used[STAGE_SLOTS];
  int stage_next;
  std::vector<int> count;  // counting sort over the vocabulary
  std::vector<int> uniq, ustart;
  // window state (host mirror of what the host itself decides)
  int window_mb;
  long long window_tokens;
  uint64_t train_steps;
  float next_mult;
  // Bumped by everything that changes the parameters or re-uses the encoder buffers (tfm_train_step, tfm_apply_update,
  // tfm_set_param): a decoder remembers the value its batch began under and refuses to continue under another.
  uint64_t generation;
  // profiling
  bool prof;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> ev_pool;
  tfm_prof_entry prof_acc[TFM_PROF_CLASSES];
  float prof_overhead_ms;  // elapsed time of an empty event pair, subtracted from every bracket
};

namespace {

int fail(tfm_ctx* c, int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(c ? c->err : g_create_error, 256, fmt, ap);
  va_end(ap);
  return code;
}

}  // namespace
namespace tfm {
void set_global_error(const char* msg) { snprintf(g_create_error, sizeof(g_create_error), "%s", msg ? msg : ""); }
}  // namespace tfm
namespace {

#define HIP_TRY(c, expr)                                                                          \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return fail(c, TFM_EHIP, "%s: %s", #expr, hipGetErrorString(e_));        \
  } while (0)

int add_param(std::vector<Param>& ps, int64_t& off, const std::string& name, int64_t rows, int64_t cols, bool pad = true) {
  Param p{name, rows, cols, off};
  off += pad ? (p.numel() + 255) / 256 * 256 : p.numel();
  ps.push_back(p);
  return (int)ps.size() - 1;
}

void build_params(const tfm_config& c, std::vector<Param>& ps, int64_t& P, Stream& enc, Stream& dec, int* kv_w0, int* kv_b0) {
  const int d = c.d_model, F = c.d_ffn;
  int64_t off = 0;
  add_param(ps, off, "embed", c.n_cutoffs ? c.cutoffs[0] + c.n_cutoffs : c.vocab, d);
  {
    int width = d;
    for (int i = 1; i <= c.n_cutoffs; ++i) {
      width /= c.adaptive_factor;
      const int lo = c.cutoffs[i - 1], hi = i < c.n_cutoffs ? c.cutoffs[i] : c.vocab;
      add_param(ps, off, "embed." + std::to_string(i), hi - lo, width);
      add_param(ps, off, "embed." + std::to_string(i) + ".proj", d, width);
    }
  }
  auto ln = [&](const std::string& pre, int& g, int& b) {
    g = add_param(ps, off, pre + ".g", d, 0);
    b = add_param(ps, off, pre + ".b", d, 0);
  };
  auto self_block = [&](const std::string& pre, int layer) {
    Block b{};
    b.kind = SELF; b.layer = layer; b.w_kv = b.b_kv = -1;
    b.w_a = add_param(ps, off, pre + ".self.wqkv", 3 * d, d);
    b.b_a = add_param(ps, off, pre + ".self.bqkv", 3 * d, 0);
    b.w_o = add_param(ps, off, pre + ".self.wo", d, d);
    b.b_o = add_param(ps, off, pre + ".self.bo", d, 0);
    ln(pre + ".ln_self", b.ln_g, b.ln_b);
    return b;
  };
  auto cross_block = [&](const std::string& pre, int layer) {
    Block b{};
    b.kind = CROSS; b.layer = layer;
    b.w_a = add_param(ps, off, pre + ".cross.wq", d, d);
    b.b_a = add_param(ps, off, pre + ".cross.bq", d, 0);
    b.w_kv = *kv_w0 + layer;
    b.b_kv = *kv_b0 + layer;
    b.w_o = add_param(ps, off, pre + ".cross.wo", d, d);
    b.b_o = add_param(ps, off, pre + ".cross.bo", d, 0);
    ln(pre + ".ln_cross", b.ln_g, b.ln_b);
    return b;
  };
  auto ffn_block = [&](const std::string& pre, int layer) {
    Block b{};
    b.kind = FFN; b.layer = layer; b.w_kv = b.b_kv = -1;
    b.w_a = add_param(ps, off, pre + ".ffn.w1", F, d);
    b.b_a = add_param(ps, off, pre + ".ffn.b1", F, 0);
    b.w_o = add_param(ps, off, pre + ".ffn.w2", d, F);
    b.b_o = add_param(ps, off, pre + ".ffn.b2", d, 0);
    ln(pre + ".ln_ffn", b.ln_g, b.ln_b);
    return b;
  };
  enc.id = 0; dec.id = 1;
  for (int i = 0; i < c.enc_layers; ++i) {
    const std::string pre = "enc." + std::to_string(i);
    enc.blocks.push_back(self_block(pre, i));
    enc.blocks.push_back(ffn_block(pre, i));
  }
  if (c.enc_layers && c.pre_norm) ln("enc.ln_final", enc.lnf_g, enc.lnf_b);
  *kv_w0 = *kv_b0 = -1;
  if (c.enc_layers) {
    // The key/value projections of every decoder layer's cross-attention read the same encoder output: their weights lie
    // back to back (no padding between them) as one [layers * 2d, d] matrix, their biases as one vector, so that one
    // product serves all layers.  (2 d d and 2 d elements keep every slice 32-byte aligned since d is a multiple of 8.)
    for (int i = 0; i < c.dec_layers; ++i) {
      const int p = add_param(ps, off, "dec." + std::to_string(i) + ".cross.wkv", 2 * d, d, false);
      if (i == 0) *kv_w0 = p;
    }
    off = (off + 255) / 256 * 256;
    for (int i = 0; i < c.dec_layers; ++i) {
      const int p = add_param(ps, off, "dec." + std::to_string(i) + ".cross.bkv", 2 * d, 0, false);
      if (i == 0) *kv_b0 = p;
    }
    off = (off + 255) / 256 * 256;
  }
  for (int i = 0; i < c.dec_layers; ++i) {
    const std::string pre = "dec." + std::to_string(i);
    dec.blocks.push_back(self_block(pre, i));
    if (c.enc_layers) dec.blocks.push_back(cross_block(pre, i));
    dec.blocks.push_back(ffn_block(pre, i));
  }
  if (c.pre_norm) ln("dec.ln_final", dec.lnf_g, dec.lnf_b);
  P = off;
}

int validate(const tfm_config& c, char* msg) {
#define BAD(...) do { snprintf(msg, 256, __VA_ARGS__); return TFM_EINVAL; } while (0)
  if (c.enc_layers < 0 || c.enc_layers > 64 || c.dec_layers < 1 || c.dec_layers > 64) BAD("layer counts out of range");
  if (c.d_model < 8 || c.d_model > 2048 || c.d_model % 8) BAD("d_model must be a multiple of 8 in [8, 2048]");
  if (c.n_heads < 1 || c.d_model % c.n_heads) BAD("d_model must be divisible by n_heads");
  if (c.d_model / c.n_heads > 128) BAD("head width above 128");
  if (c.d_ffn < 8 || c.d_ffn % 8) BAD("d_ffn must be a multiple of 8");
  if (c.vocab < 4 || c.vocab > (1 << 24)) BAD("vocab out of range");
  if (c.pad_id < 0 || c.pad_id >= c.vocab || c.eos_id < 0 || c.eos_id >= c.vocab) BAD("pad/eos id outside the vocabulary");
  if (c.max_sentences < 1 || c.max_sentences > 65535) BAD("max_sentences out of range");
  if (c.max_len < 1 || c.max_len > 4096) BAD("max_len out of range");
  if (c.max_tokens < 1 || c.max_tokens > (1 << 20)) BAD("max_tokens out of range");
  if ((int64_t)c.max_tokens * c.vocab > ((int64_t)1 << 33)) BAD("max_tokens * vocab too large");
  if (c.precision < 0 || c.precision > 2) BAD("precision must be 0, 1 or 2");
  if (c.pre_norm != 0 && c.pre_norm != 1) BAD("pre_norm must be 0 or 1");
  if (!(c.dropout >= 0.f && c.dropout < 1.f)) BAD("dropout must be in [0, 1)");
  if (!(c.attn_dropout >= 0.f && c.attn_dropout < 1.f)) BAD("attn_dropout must be in [0, 1)");
  if (!(c.relu_dropout >= 0.f && c.relu_dropout < 1.f)) BAD("relu_dropout must be in [0, 1)");
  if (!(c.label_smoothing >= 0.f && c.label_smoothing < 1.f)) BAD("label_smoothing must be in [0, 1)");
  if (!(c.adam_beta1 >= 0.f && c.adam_beta1 < 1.f && c.adam_beta2 >= 0.f && c.adam_beta2 < 1.f && c.adam_eps > 0.f)) BAD("bad Adam constants");
  if (!(c.clip_norm >= 0.f)) BAD("clip_norm must be >= 0");
  if (!(c.weight_decay >= 0.f) || !std::isfinite(c.weight_decay)) BAD("weight_decay must be >= 0");
  if (!(c.init_loss_scale > 0.f) || !std::isfinite(c.init_loss_scale)) BAD("init_loss_scale must be positive");
  if (c.scale_window < 1) BAD("scale_window must be >= 1");
  if (!(c.min_loss_scale >= 0.f)) BAD("min_loss_scale must be >= 0");
  if (c.n_cutoffs < 0 || c.n_cutoffs > 3) BAD("n_cutoffs must be 0 .. 3");
  if (c.n_cutoffs > 0) {
    if (c.enc_layers != 0) BAD("adaptive inputs / adaptive softmax are for the decoder-only language model");
    if (c.label_smoothing != 0.f) BAD("the adaptive softmax is trained on the plain likelihood: label_smoothing must be 0");
    if (c.adaptive_factor < 1) BAD("adaptive_factor must be >= 1");
    int prev = 0, width = c.d_model;
    for (int i = 0; i < c.n_cutoffs; ++i) {
      if (c.cutoffs[i] <= prev || c.cutoffs[i] >= c.vocab) BAD("cutoffs must ascend inside (0, vocab)");
      prev = c.cutoffs[i];
      if (width % c.adaptive_factor) BAD("d_model must be divisible by adaptive_factor^i for every tail cluster");
      width /= c.adaptive_factor;
      if (width < 4 || width % 4) BAD("a tail cluster's width must be a multiple of 4");
    }
    if (c.pad_id >= c.cutoffs[0] || c.eos_id >= c.cutoffs[0]) BAD("pad and eos must lie in the head");
  }
#undef BAD
  return TFM_OK;
}

// Carves every buffer out of the workspace.  With ctx->... pointers null-based (base == nullptr) it only sizes.
size_t carve(tfm_ctx* c, char* base) {
  const tfm_config& cf = c->cfg;
  const size_t R = (size_t)cf.max_tokens, d = cf.d_model, F = cf.d_ffn, H = cf.n_heads, esz = c->esz;
  Arena a{base};
  c->W = (float*)a.take(c->P * 4);
  c->M = (float*)a.take(c->P * 4);
  c->V = (float*)a.take(c->P * 4);
  c->G = (float*)a.take(c->P * 4);
  c->g = a.take(c->P * esz);
  c->Wh = c->dt == F32 ? (void*)c->W : a.take(c->P * esz);
  c->st = (DevState*)a.take(sizeof(DevState));
  c->ld_kv = cf.enc_layers ? cf.dec_layers * 2 * (int)d : 0;
  c->kv_all = cf.enc_layers ? a.take(R * c->ld_kv * esz) : nullptr;
  c->dkv_all = cf.enc_layers ? a.take(R * c->ld_kv * esz) : nullptr;
  for (Stream* s : {&c->enc, &c->dec}) {
    const size_t K = s->blocks.size();
    if (K == 0) continue;
    s->resid.assign(K + 1, nullptr); s->norm.assign(K + 1, nullptr);
    s->mean.assign(K + 1, nullptr); s->rstd.assign(K + 1, nullptr);
    for (size_t k = 0; k <= K; ++k) {
      s->resid[k] = a.take(R * d * esz);
      s->norm[k] = a.take(R * d * esz);
      s->mean[k] = (float*)a.take(R * 4);
      s->rstd[k] = (float*)a.take(R * 4);
    }
    for (Block& b : s->blocks) {
      if (b.kind == SELF) { b.inter = a.take(R * 3 * d * esz); b.ctx = a.take(R * d * esz); b.lse = (float*)a.take(H * R * 4); b.dint = a.take(R * 3 * d * esz); }
      else if (b.kind == CROSS) {
        b.inter = a.take(R * d * esz); b.ctx = a.take(R * d * esz); b.lse = (float*)a.take(H * R * 4);
        b.dint = a.take(R * d * esz);
        b.kv = c->kv_all ? (char*)c->kv_all + (size_t)b.layer * 2 * d * esz : nullptr;
        b.dkv = c->dkv_all ? (char*)c->dkv_all + (size_t)b.layer * 2 * d * esz : nullptr;
      } else { b.inter = a.take(R * F * esz); b.dint = a.take(R * F * esz); }
      b.dy = a.take(R * d * esz);
    }
  }
  const size_t wide = std::max(3 * d, F);
  c->y = a.take(R * d * esz);
  c->dcur = a.take(R * d * esz);
  c->demb[0] = a.take(R * d * esz);
  c->demb[1] = a.take(R * d * esz);
  c->dsA = a.take(R * d * esz);
  c->dsB = a.take(R * d * esz);
  c->dctx = a.take(R * d * esz);
  c->dmem = a.take(R * d * esz);
  {
    Adaptive& ad = c->ad;
    ad.n = cf.n_cutoffs;
    ad.v0 = cf.vocab;
    ad.vmax = 0;
    int width = (int)d;
    for (int k = 0; k <= ad.n; ++k) {
      ad.lo[k] = k ? cf.cutoffs[k - 1] : 0;
      ad.hi[k] = k < ad.n ? cf.cutoffs[k] : cf.vocab;
      ad.width[k] = width;
      if (k) { ad.E[k] = 2 * k - 1; ad.P[k] = 2 * k; ad.vmax = std::max(ad.vmax, ad.hi[k] - ad.lo[k]); }   // parameters 1, 2, 3, 4, ...
      width = cf.adaptive_factor > 0 ? width / cf.adaptive_factor : width;
    }
    if (ad.n) ad.v0 = cf.cutoffs[0] + ad.n;
  }
  // logits: [R, vocab], or for the adaptive softmax the head's [R, v0] followed by room for one tail cluster at a time
  c->logits = a.take(R * (size_t)(c->ad.n ? c->ad.v0 + c->ad.vmax : cf.vocab) * esz + 256);   // (+ the tail region's alignment)
  if (c->ad.n) {
    Adaptive& ad = c->ad;
    for (int k = 1; k <= ad.n; ++k) {
      const size_t w = ad.width[k];
      ad.Xc[k] = a.take(R * w * esz); ad.dXc[k] = a.take(R * w * esz); ad.U[k] = a.take(R * w * esz); ad.dU[k] = a.take(R * w * esz);
      ad.tmpP[k] = a.take(d * w * esz);
    }
    ad.Y = a.take(R * d * esz); ad.dY = a.take(R * d * esz); ad.Hc = a.take(R * d * esz); ad.dHc = a.take(R * d * esz);
    ad.tail_loss = (float*)a.take(R * 4); ad.tail_nll = (float*)a.take(R * 4);
  }
  c->loss_rows = (float*)a.take(R * 4);
  c->nll_rows = (float*)a.take(R * 4);
  c->pe = (float*)a.take((size_t)cf.max_len * d * 4);
  const size_t red = std::max(layernorm_bwd_scratch_bytes((int)R, (int)d), colsum_scratch_bytes((int)R, (int)wide));
  c->red_scratch = a.take(red);
  c->ln_slice = (layernorm_bwd_scratch_bytes((int)R, (int)d) + 255) & ~(size_t)255;
  c->ln_slices = (int)(c->enc.blocks.size() + c->dec.blocks.size()) + 2;      // one LayerNorm backward per block, plus final norms
  c->ln_pool = (char*)a.take(c->ln_slice * c->ln_slices);
  c->red_scratch_side = a.take(colsum_scratch_bytes((int)R, (int)wide));
  c->scan_scratch = a.take(scan_scratch_bytes(c->P));
  c->splitk_bytes = c->dt == F32 ? 0 : (size_t)8 * 128 * 128 * 128 * sizeof(float);   // 8 slices of up to 128 tiles
  c->splitk_ws = c->splitk_bytes ? a.take(c->splitk_bytes) : nullptr;
  c->splitk_ws_side = c->splitk_bytes ? a.take(c->splitk_bytes) : nullptr;
  // one block of ints, filled by a single host-to-device copy per step:
  // enc ids, pos [R each], off [B+1]; dec ids, pos, off; labels [R]; occurrence entries [2R];
  // segments: tok, beg, end, dst [NS each]; multi-segment tokens: tok, row0, n [NM each]
  const size_t Bc = (size_t)cf.max_sentences + 1;
  const size_t NS = 2 * R + 2 * R / EMB_SEG + 2, NM = 2 * R / EMB_SEG + 2;
  c->emb_partial = (float*)a.take((2 * NM) * d * sizeof(float));
  c->int_block_ints = 2 * (2 * R + Bc) + R + 2 * R + 4 * NS + 3 * NM + (c->ad.n ? 8 * R : 0) + 12 * Bc + 4;
  c->ibase = (int*)a.take(c->int_block_ints * 4);
  int* p = c->ibase;
  auto nxt = [&](size_t n) { int* r = base ? p : nullptr; p += n; return r; };
  c->enc.ids = nxt(R); c->enc.pos = nxt(R); c->enc.off = nxt(Bc);
  c->dec.ids = nxt(R); c->dec.pos = nxt(R); c->dec.off = nxt(Bc);
  c->labels = nxt(R);
  c->uentries = nxt(2 * R);
  c->seg_tok = nxt(NS); c->seg_beg = nxt(NS); c->seg_end = nxt(NS); c->seg_dst = nxt(NS);
  c->mt_tok = nxt(NM); c->mt_row0 = nxt(NM); c->mt_n = nxt(NM);
  if (c->ad.n) {
    Adaptive& ad = c->ad;
    ad.in_idx = nxt(R); ad.in_tok = nxt(R); ad.out_idx = nxt(R); ad.out_lab = nxt(R);
    ad.sg_tok = nxt(R); ad.sg_beg = nxt(R); ad.sg_end = nxt(R); ad.sg_ent = nxt(R);
  }
  // (the last 12 * Bc ints of the block, moved up to a 16-byte boundary: the kernels read whole entries)
  p += (4 - ((p - c->ibase) & 3)) & 3;
  for (int k = 0; k < 3; ++k) c->grp[k] = nxt(4 * Bc);
  return (a.off + 255) & ~(size_t)255;
}

// ---- profiling wrapper -------------------------------------------------------------------------------------------------
template <typename F>
void run(tfm_ctx* c, int cls, double flops, double bytes, F&& launch, hipStream_t stream) {
  if (!c->prof) { launch(); return; }
  auto get_ev = [&]() {
    if (!c->ev_pool.empty()) { hipEvent_t e = c->ev_pool.back(); c->ev_pool.pop_back(); return e; }
    hipEvent_t e; hipEventCreate(&e); return e;
  };
  ProfRec r{cls, get_ev(), get_ev(), flops, bytes};
  hipEventRecord(r.a, stream);
  launch();
  hipEventRecord(r.b, stream);
  c->recs.push_back(r);
}
template <typename F>
void run(tfm_ctx* c, int cls, double flops, double bytes, F&& launch) { run(c, cls, flops, bytes, launch, c->stream); }

// ---- ordering between the two streams -----------------------------------------------------------------------------------
hipEvent_t mark(tfm_ctx* c, hipStream_t on) {
  if (c->sync_used == c->sync_ev.size()) {
    hipEvent_t e = nullptr;
    // (ordering between two streams of one device: a device-scope release is enough and far cheaper than the default,
    // which makes the work visible to the host as well)
    hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventReleaseToDevice);
    c->sync_ev.push_back(e);
  }
  hipEvent_t e = c->sync_ev[c->sync_used++];
  hipEventRecord(e, on);
  return e;
}
// what has been enqueued on `from` so far happens before what is enqueued on `to` from now on
inline void order(tfm_ctx* c, hipStream_t from, hipStream_t to) { hipStreamWaitEvent(to, mark(c, from), 0); }
inline hipStream_t wstream(tfm_ctx* c) { return c->overlap ? c->side : c->stream; }
// main -> side: the operands of the weight-gradient work enqueued next are ready
inline void side_begin(tfm_ctx* c) { if (c->overlap) order(c, c->stream, c->side); }
// main waits for a side mark
inline void main_wait(tfm_ctx* c, hipEvent_t& e) {
  if (c->overlap && e) hipStreamWaitEvent(c->stream, e, 0);
  e = nullptr;
}

void prof_collect(tfm_ctx* c) {
  for (ProfRec& r : c->recs) {
    float ms = 0.f;
    hipEventElapsedTime(&ms, r.a, r.b);
    ms -= c->prof_overhead_ms;
    if (ms < 0.f) ms = 0.f;
    tfm_prof_entry& e = c->prof_acc[r.cls];
    e.launches += 1; e.ms += ms; e.flops += r.flops; e.bytes += r.bytes;
    c->ev_pool.push_back(r.a); c->ev_pool.push_back(r.b);
  }
  c->recs.clear();
}

// main stream: the pending Adam update of parameter pi (and of everything before it in flat order) has finished
inline void need(tfm_ctx* c, int pi) {
  if (!c->adam_pending) return;
  const int ch = c->chunk_of[pi];
  if (ch >= c->adam_waited) {
    hipStreamWaitEvent(c->stream, c->adam_ev[ch], 0);
    c->adam_waited = ch + 1;
    if (c->adam_waited == (int)c->chunks.size()) c->adam_pending = false;
  }
}
inline void adam_join(tfm_ctx* c) { if (c->adam_pending) need(c, (int)c->params.size() - 1); }

// ---- small helpers over the flat parameter buffers ----------------------------------------------------------------------
inline void* wh(tfm_ctx* c, int i) { return (char*)c->Wh + c->params[i].off * c->esz; }
inline void* gr(tfm_ctx* c, int i) { return (char*)c->g + c->params[i].off * c->esz; }

void gemm(tfm_ctx* c, int form, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C, int ldc,
          const void* bias = nullptr, int relu = 0, const void* mask = nullptr, const void* residual = nullptr, bool side = false,
          uint64_t drop_key = 0, float drop_p = 0.f, float mask_scale = 1.f, int* deferred_splits = nullptr) {
  if (deferred_splits) *deferred_splits = 0;
  if (M <= 0 || N <= 0) return;
  GemmArgs a{c->dt, form, M, N, K, A, lda, B, ldb, C, ldc, bias, relu, mask, residual};
  a.drop_key = drop_key; a.drop_p = drop_p; a.mask_scale = mask_scale; a.deferred_splits = deferred_splits;
  side = side && c->overlap;
  hipStream_t stream = side ? c->side : c->stream;
  a.splitk_ws = side ? c->splitk_ws_side : c->splitk_ws;
  a.splitk_ws_bytes = c->splitk_bytes;
  // algorithmic bytes: each operand read once, the result written once (plus the epilogue's mask/residual reads)
  const double bytes = (double)c->esz * ((double)M * K + (double)K * N + (double)M * N * (1.0 + (mask ? 1.0 : 0.0) + (residual ? 1.0 : 0.0)));
  run(c, TFM_PROF_GEMM, 2.0 * M * N * K, bytes, [&] { launch_gemm(stream, a); }, stream);
}
// Launches the queued weight gradients as one grouped GEMM on the side stream (after everything enqueued on the main
// stream so far, which produced their operands).
void flush_wgrads(tfm_ctx* c) {
  if (c->wq.empty() && c->lnq.empty()) return;
  hipStream_t stream = wstream(c);
  side_begin(c);
  if (!c->lnq.empty()) {
    const int d = c->cfg.d_model;
    run(c, TFM_PROF_NORM, 0.0, 0.0, [&] { launch_ln_reduce_batched(stream, c->dt, c->lnq.data(), (int)c->lnq.size(), d); }, stream);
    c->lnq.clear();
  }
  if (c->wq.empty()) return;
  double flops = 0, bytes = 0;
  for (size_t i = 0; i < c->wq.size(); ++i) {
    const WgradJob& j = c->wq[i];
    flops += 2.0 * j.M * j.N * j.K;
    bytes += (double)c->esz * ((double)j.M * j.K + (double)j.K * j.N + (double)j.M * j.N);
  }
  run(c, TFM_PROF_GEMM, flops, bytes, [&] { launch_wgrad_grouped(stream, c->dt, c->wq.data(), (int)c->wq.size()); }, stream);
  c->wq.clear();
  c->wq_tiles = 0;
}

// Weight gradient dW[M,N] = A^T B over K rows and, if bias_grad is given, the bias gradient [M] = column sums of A.
// A and B must stay untouched until the end of the backward pass: the product is queued, not launched.  Shapes the
// grouped matrix-core kernel does not take (fp32 mode, widths that are not multiples of 8) run at once on the side stream.
void wgrad(tfm_ctx* c, int M, int N, int K, const void* A, int lda, const void* B, int ldb, void* C, int ldc, void* bias_grad = nullptr) {
  if (M <= 0 || N <= 0) return;
  WgradJob j{M, N, K, A, lda, B, ldb, C, ldc, bias_grad};
  if (c->dt != F32 && K > 0 && wgrad_group_supported(c->dt, j)) {
    c->wq.push_back(j);
    c->wq_tiles += (long)((M + 127) / 128) * ((N + 127) / 128);
    if ((int)c->wq.size() == WGRAD_GROUP_MAX || c->wq_tiles >= c->wq_flush_tiles) flush_wgrads(c);
    return;
  }
  side_begin(c);
  gemm(c, 2, M, N, K, A, lda, B, ldb, C, ldc, nullptr, 0, nullptr, nullptr, true);
  if (bias_grad) {
    hipStream_t stream = wstream(c);
    void* scratch = c->overlap ? c->red_scratch_side : c->red_scratch;
    run(c, TFM_PROF_NORM, 0.0, (double)c->esz * K * M, [&] { launch_colsum(stream, c->dt, A, lda, K, M, bias_grad, scratch); }, stream);
  }
}

double attn_flops(const std::vector<int>& lq, const std::vector<int>& lk, int d, bool causal) {
  double f = 0;
  for (size_t b = 0; b < lq.size(); ++b) f += 4.0 * d * lq[b] * (double)lk[b] * (causal ? 0.5 : 1.0);
  return f;
}

}  // namespace

extern "C" {

int tfm_workspace_bytes(const tfm_config* cfg, size_t* bytes) {
  if (!cfg || !bytes) return fail(nullptr, TFM_EINVAL, "null argument");
  char msg[256];
  int rc = validate(*cfg, msg);
  if (rc) return fail(nullptr, rc, "%s", msg);
  tfm_ctx tmp{};
  tmp.cfg = *cfg;
  tmp.dt = cfg->precision;
  tmp.esz = dtype_size(tmp.dt);
  build_params(*cfg, tmp.params, tmp.P, tmp.enc, tmp.dec, &tmp.kv_w0, &tmp.kv_b0);
  *bytes = carve(&tmp, nullptr);
  return TFM_OK;
}

int tfm_create(const tfm_config* cfg, void* ws, size_t bytes, void* hip_stream, tfm_ctx** out) {
  if (!cfg || !ws || !out) return fail(nullptr, TFM_EINVAL, "null argument");
  char msg[256];
  int rc = validate(*cfg, msg);
  if (rc) return fail(nullptr, rc, "%s", msg);
  if (((uintptr_t)ws & 255) != 0) return fail(nullptr, TFM_EINVAL, "workspace must be 256-byte aligned");
  tfm_ctx* c = new tfm_ctx{};
  c->cfg = *cfg;
  c->stream = (hipStream_t)hip_stream;
  c->dt = cfg->precision;
  c->esz = dtype_size(c->dt);
  c->R = cfg->max_tokens;
  build_params(*cfg, c->params, c->P, c->enc, c->dec, &c->kv_w0, &c->kv_b0);
  const size_t need = carve(c, nullptr);
  if (bytes < need) {
    delete c;
    return fail(nullptr, TFM_ENOMEM, "workspace has %zu bytes, %zu needed", bytes, need);
  }
  carve(c, (char*)ws);
  c->count.assign(cfg->vocab, 0);
  c->next_mult = 1.f;
  auto cleanup = [&](int code) { tfm_destroy(c); return code; };
  if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) {
    c->side = nullptr;
    fail(nullptr, TFM_EHIP, "cannot create the side stream");
    return cleanup(TFM_EHIP);
  }
  c->overlap = true;
  c->wq_tiles = 0;
  c->wq_flush_tiles = 4096;
  {
    // chunk boundaries: the embedding, then one chunk per block (its parameters are contiguous; the cross-attention blocks'
    // stacked key/value projections are a chunk of their own between the two streams' blocks), final norms with
    // the block before them
    std::vector<int> first;                         // first parameter of each chunk
    first.push_back(0);
    for (Stream* st : {&c->enc, &c->dec})
      for (Block& b : st->blocks) first.push_back(b.w_a);
    if (c->kv_w0 >= 0) first.push_back(c->kv_w0);    // the stacked key/value projections of the cross-attention blocks
    std::sort(first.begin(), first.end());
    c->chunk_of.assign(c->params.size(), 0);
    for (size_t k = 0; k < first.size(); ++k) {
      const int p0 = first[k], p1 = k + 1 < first.size() ? first[k + 1] : (int)c->params.size();
      const int64_t o0 = c->params[p0].off, o1 = p1 < (int)c->params.size() ? c->params[p1].off : c->P;
      c->chunks.push_back({o0, o1 - o0, p1 - 1});
      for (int i = p0; i < p1; ++i) c->chunk_of[i] = (int)k;
      hipEvent_t e = nullptr;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventReleaseToDevice) != hipSuccess) { fail(nullptr, TFM_EHIP, "cannot create events"); return cleanup(TFM_EHIP); }
      c->adam_ev.push_back(e);
    }
  }
  // zero parameters, moments, gradients and the accumulator (they are contiguous at the start of the workspace)
  hipError_t e = hipMemsetAsync(ws, 0, (char*)c->st - (char*)ws + sizeof(DevState), c->stream);
  if (e != hipSuccess) { fail(nullptr, TFM_EHIP, "hipMemsetAsync: %s", hipGetErrorString(e)); return cleanup(TFM_EHIP); }
  DevState init{};
  init.loss_scale = cfg->init_loss_scale;
  e = hipMemcpyAsync(c->st, &init, sizeof(init), hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess) {
    // sinusoidal position table in double, stored fp32: PE(t,2i) = sin(t / 10000^(2i/d)), PE(t,2i+1) = cos(same)
    std::vector<float> pe((size_t)cfg->max_len * cfg->d_model);
    for (int t = 0; t < cfg->max_len; ++t)
      for (int i = 0; i < cfg->d_model / 2; ++i) {
        const double ang = (double)t / std::pow(10000.0, 2.0 * i / cfg->d_model);
        pe[(size_t)t * cfg->d_model + 2 * i] = (float)std::sin(ang);
        pe[(size_t)t * cfg->d_model + 2 * i + 1] = (float)std::cos(ang);
      }
    e = hipMemcpyAsync(c->pe, pe.data(), pe.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  }
  if (e != hipSuccess) { fail(nullptr, TFM_EHIP, "init copy: %s", hipGetErrorString(e)); return cleanup(TFM_EHIP); }
  for (int i = 0; i < STAGE_SLOTS; ++i) {
    e = hipHostMalloc((void**)&c->stage[i], c->int_block_ints * 4, hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->stage_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) { fail(nullptr, TFM_EHIP, "staging buffers: %s", hipGetErrorString(e)); return cleanup(TFM_EHIP); }
  }
  *out = c;
  return TFM_OK;
}

void tfm_destroy(tfm_ctx* c) {
  if (!c) return;
  hipStreamSynchronize(c->stream);
  if (c->side) { hipStreamSynchronize(c->side); hipStreamDestroy(c->side); }
  for (hipEvent_t e : c->sync_ev) hipEventDestroy(e);
  for (hipEvent_t e : c->adam_ev) hipEventDestroy(e);
  for (int i = 0; i < STAGE_SLOTS; ++i) {
    if (c->stage[i]) hipHostFree(c->stage[i]);
    if (c->stage_ev[i]) hipEventDestroy(c->stage_ev[i]);
  }
  for (ProfRec& r : c->recs) { hipEventDestroy(r.a); hipEventDestroy(r.b); }
  for (hipEvent_t e : c->ev_pool) hipEventDestroy(e);
  delete c;
}

const char* tfm_last_error(const tfm_ctx* c) { return c ? c->err : g_create_error; }

int tfm_num_params(const tfm_ctx* c, int32_t* n) {
  if (!c || !n) return TFM_EINVAL;
  *n = (int32_t)c->params.size();
  return TFM_OK;
}

int tfm_param_info(const tfm_ctx* c, int32_t i, char name[64], int64_t shape[2]) {
  if (!c || i < 0 || i >= (int)c->params.size()) return TFM_EINVAL;
  if (name) { std::strncpy(name, c->params[i].name.c_str(), 63); name[63] = 0; }
  if (shape) { shape[0] = c->params[i].rows; shape[1] = c->params[i].cols; }
  return TFM_OK;
}

static int check_param(tfm_ctx* c, int32_t i, const void* host, int64_t n) {
  if (c) adam_join(c);
  if (!c) return TFM_EINVAL;
  if (i < 0 || i >= (int)c->params.size()) return fail(c, TFM_EINVAL, "parameter index %d out of range", i);
  if (!host || n != c->params[i].numel()) return fail(c, TFM_EINVAL, "parameter %d has %lld elements, got %lld", i, (long long)c->params[i].numel(), (long long)n);
  return TFM_OK;
}

int tfm_set_param(tfm_ctx* c, int32_t i, const float* host, int64_t n) {
  int rc = check_param(c, i, host, n);
  if (rc) return rc;
  const Param& p = c->params[i];
  c->generation += 1;
  HIP_TRY(c, hipMemcpyAsync(c->W + p.off, host, n * 4, hipMemcpyHostToDevice, c->stream));
  if (c->dt != F32) launch_convert(c->stream, F32, c->W + p.off, c->dt, (char*)c->Wh + p.off * c->esz, n);
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return TFM_OK;
}

static int get_flat(tfm_ctx* c, int32_t i, const float* dev, float* host, int64_t n) {
  int rc = check_param(c, i, host, n);
  if (rc) return rc;
  HIP_TRY(c, hipMemcpyAsync(host, dev + c->params[i].off, n * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return TFM_OK;
}

int tfm_get_param(tfm_ctx* c, int32_t i, float* host, int64_t n) { return c ? get_flat(c, i, c->W, host, n) : TFM_EINVAL; }

int tfm_get_grad(tfm_ctx* c, int32_t i, float* host, int64_t n) {
  int rc = check_param(c, i, host, n);
  if (rc) return rc;
  if (c->window_mb == 0) { std::memset(host, 0, n * 4); return TFM_OK; }
  if (c->window_mb >= 2) return get_flat(c, i, c->G, host, n);
  // a single sub-batch so far: its gradient is still in the compute dtype; convert through the accumulator
  const Param& p = c->params[i];
  launch_convert(c->stream, c->dt, (char*)c->g + p.off * c->esz, F32, c->G + p.off, n);
  return get_flat(c, i, c->G, host, n);
}

int tfm_get_adam(tfm_ctx* c, int32_t i, int32_t which, float* host, int64_t n) {
  if (!c || which < 0 || which > 1) return TFM_EINVAL;
  return get_flat(c, i, which ? c->V : c->M, host, n);
}

int tfm_set_adam(tfm_ctx* c, int32_t i, int32_t which, const float* host, int64_t n) {
  if (!c || which < 0 || which > 1) return TFM_EINVAL;
  int rc = check_param(c, i, host, n);
  if (rc) return rc;
  HIP_TRY(c, hipMemcpyAsync((which ? c->V : c->M) + c->params[i].off, host, n * 4, hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return TFM_OK;
}

int tfm_get_scaler(tfm_ctx* c, float* loss_scale, int32_t* clean_steps, int64_t* num_updates) {
  if (!c) return TFM_EINVAL;
  adam_join(c);
  DevState h;
  HIP_TRY(c, hipMemcpyAsync(&h, c->st, sizeof(h), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  if (loss_scale) *loss_scale = h.loss_scale;
  if (clean_steps) *clean_steps = h.clean_steps;
  if (num_updates) *num_updates = h.num_updates;
  if (h.scale_too_small) return fail(c, TFM_ESCALE, "loss scale %g is below the minimum %g", h.loss_scale, c->cfg.min_loss_scale);
  return TFM_OK;
}

int tfm_set_scaler(tfm_ctx* c, float loss_scale, int32_t clean_steps, int64_t num_updates) {
  if (!c) return TFM_EINVAL;
  adam_join(c);
  if (!(loss_scale > 0.f) || clean_steps < 0 || num_updates < 0) return fail(c, TFM_EINVAL, "bad scaler state");
  DevState h;
  HIP_TRY(c, hipMemcpyAsync(&h, c->st, sizeof(h), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  h.loss_scale = loss_scale; h.clean_steps = clean_steps; h.num_updates = num_updates;
  h.scale_too_small = loss_scale < c->cfg.min_loss_scale ? 1 : 0;
  HIP_TRY(c, hipMemcpyAsync(c->st, &h, sizeof(h), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return TFM_OK;
}

int tfm_set_overlap(tfm_ctx* c, int32_t on) {
  if (!c) return TFM_EINVAL;
  adam_join(c);
  c->overlap = on != 0;
  return TFM_OK;
}

int tfm_debug_set_loss_multiplier(tfm_ctx* c, float mult) {
  if (c) adam_join(c);
  if (!c) return TFM_EINVAL;
  c->next_mult = mult;
  return TFM_OK;
}

int tfm_profile_enable(tfm_ctx* c, int32_t on) {
  if (!c) return TFM_EINVAL;
  adam_join(c);
  c->prof = on != 0;
  if (c->prof) {
    // calibrate: the time between two events recorded back to back is bracket overhead, not kernel time
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    std::vector<float> t;
    hipEvent_t a, b;
    HIP_TRY(c, hipEventCreate(&a));
    HIP_TRY(c, hipEventCreate(&b));
    for (int i = 0; i < 33; ++i) {
      HIP_TRY(c, hipEventRecord(a, c->stream));
      HIP_TRY(c, hipEventRecord(b, c->stream));
      HIP_TRY(c, hipEventSynchronize(b));
      float ms = 0.f;
      HIP_TRY(c, hipEventElapsedTime(&ms, a, b));
      t.push_back(ms);
    }
    std::sort(t.begin(), t.end());
    c->prof_overhead_ms = t[t.size() / 2];
    c->ev_pool.push_back(a);
    c->ev_pool.push_back(b);
  }
  return TFM_OK;
}

int tfm_profile_read(tfm_ctx* c, tfm_prof_entry out[TFM_PROF_CLASSES], int32_t reset) {
  if (!c || !out) return TFM_EINVAL;
  adam_join(c);
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  prof_collect(c);
  std::memcpy(out, c->prof_acc, sizeof(c->prof_acc));
  if (reset) std::memset(c->prof_acc, 0, sizeof(c->prof_acc));
  return TFM_OK;
}

}  // extern "C"

// ---- the step ------------------------------------------------------------------------------------------------------------
namespace {

struct StepCtx {
  tfm_ctx* c;
  std::vector<int> slen, tlen;
  int B, Ts, Tt;
  uint64_t step;
  int n_grp[3] = {0, 0, 0};                          // groups of this step per attention kind (0: none, one sentence per block)
};

uint64_t site_key(const StepCtx& s, int stream, int layer, int sub) {
  return dropout_site_key(s.c->cfg.seed, s.step, stream, layer, sub);
}
uint64_t block_key(const StepCtx& s, const Stream& st, int k) {
  const Block& b = st.blocks[k];
  return site_key(s, st.id, b.layer, (int)b.kind);
}

void attention(const StepCtx& s, bool bwd, const Stream& qs, const Stream& ks, const std::vector<int>& lq,
               const std::vector<int>& lk, const void* q, int ldq, const void* k, int ldk, const void* v, int ldv, void* o,
               float* lse, bool causal, uint64_t drop_key, const void* d_o = nullptr, void* dq = nullptr, int lddq = 0,
               void* dk = nullptr, int lddk = 0, void* dv = nullptr, int lddv = 0) {
  tfm_ctx* c = s.c;
  const int d = c->cfg.d_model, H = c->cfg.n_heads;
  AttnArgs a{};
  a.dt = c->dt; a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldk = ldk; a.ldv = ldv; a.o = o; a.ldo = d; a.lse = lse;
  a.q_off = qs.off; a.k_off = ks.off; a.B = s.B; a.H = H; a.dh = d / H; a.max_lq = qs.max_len; a.max_lk = ks.max_len;
  a.total_q = qs.rows; a.total_k = ks.rows; a.causal = causal ? 1 : 0;
  a.d_o = d_o; a.lddo = d; a.dq = dq; a.dk = dk; a.dv = dv; a.lddq = lddq; a.lddk = lddk; a.lddv = lddv;
  a.drop_key = drop_key; a.drop_p = c->cfg.attn_dropout;          // dropout on the attention weights (0: off)
  const int kind = qs.id == 0 ? 0 : (ks.id == 1 ? 1 : 2);
  if (s.n_grp[kind] > 0) { a.groups = c->grp[kind]; a.n_groups = s.n_grp[kind]; }
  const double f = attn_flops(lq, lk, d, causal);
  const double bytes = (double)c->esz * d * (bwd ? (4.0 * qs.rows + 4.0 * ks.rows) : (2.0 * qs.rows + 2.0 * ks.rows));
  if (!bwd) run(c, TFM_PROF_ATTENTION, f, bytes, [&] { launch_attention_fwd(c->stream, a); });
  else run(c, TFM_PROF_ATTENTION, 2.0 * f, bytes, [&] { launch_attention_bwd(c->stream, a); });
}

// y = f_k(fin): the sub-layer without its residual wrapper
void sublayer_fwd(const StepCtx& s, Stream& st, int k, const void* fin, void* y) {
  tfm_ctx* c = s.c;
  Block& b = st.blocks[k];
  const int d = c->cfg.d_model, F = c->cfg.d_ffn, T = st.rows;
  const std::vector<int>& len = st.id ? s.tlen : s.slen;
  need(c, b.ln_b);                                 // the block's parameters are one Adam chunk
  if (b.kind == SELF) {
    gemm(c, 0, T, 3 * d, d, fin, d, wh(c, b.w_a), d, b.inter, 3 * d, wh(c, b.b_a));
    const char* qkv = (const char*)b.inter;
    attention(s, false, st, st, len, len, qkv, 3 * d, qkv + d * c->esz, 3 * d, qkv + 2 * d * c->esz, 3 * d, b.ctx, b.lse, st.id == 1,
              site_key(s, st.id, b.layer, 3));
    gemm(c, 0, T, d, d, b.ctx, d, wh(c, b.w_o), d, y, d, wh(c, b.b_o));
  } else if (b.kind == CROSS) {
    Stream& en = c->enc;
    const void* mem = en.norm[en.blocks.size()];
    gemm(c, 0, T, d, d, fin, d, wh(c, b.w_a), d, b.inter, d, wh(c, b.b_a));
    if (c->kv_ready) { main_wait(c, c->kv_ready); c->kv_ready = nullptr; }   // the keys and values of all layers (see tfm_train_step)
    const char* kv = (const char*)b.kv;
    attention(s, false, st, en, s.tlen, s.slen, b.inter, d, kv, c->ld_kv, kv + d * c->esz, c->ld_kv, b.ctx, b.lse, false,
              site_key(s, st.id, b.layer, 4));
    gemm(c, 0, T, d, d, b.ctx, d, wh(c, b.w_o), d, y, d, wh(c, b.b_o));
  } else {
    // (dropout on the hidden activations, if configured, is applied by the same epilogue after the ReLU)
    gemm(c, 0, T, F, d, fin, d, wh(c, b.w_a), d, b.inter, F, wh(c, b.b_a), 1, nullptr, nullptr, false, site_key(s, st.id, b.layer, 5),
         c->cfg.relu_dropout);
    gemm(c, 0, T, d, F, b.inter, F, wh(c, b.w_o), F, y, d, wh(c, b.b_o));
  }
}

void ln_fwd(tfm_ctx* c, const void* x, const void* y, int g, int b, void* s_out, void* n_out, float* mean, float* rstd,
            int rows, uint64_t key) {
  const int d = c->cfg.d_model;
  need(c, b);
  const double bytes = (double)c->esz * rows * d * (1.0 + (y ? 1.0 : 0.0) + (s_out ? 1.0 : 0.0) + 1.0);
  run(c, TFM_PROF_NORM, 0.0, bytes, [&] {
    launch_residual_layernorm_fwd(c->stream, c->dt, x, y, wh(c, g), wh(c, b), s_out, n_out, mean, rstd, rows, d, key, c->cfg.dropout);
  });
}

void stream_fwd(const StepCtx& s, Stream& st) {
  tfm_ctx* c = s.c;
  const int K = (int)st.blocks.size(), d = c->cfg.d_model, T = st.rows;
  const bool pre = c->cfg.pre_norm != 0;
  void* emb = pre ? st.resid[0] : st.norm[0];
  need(c, 0);
  const Adaptive& ad = c->ad;
  for (int k = 1; k <= ad.n; ++k) {                  // adaptive inputs: narrow rows of tail tokens, projected up to d
    const int n = ad.in_cnt[k], w = ad.width[k];
    if (n == 0) continue;
    need(c, ad.P[k]);
    run(c, TFM_PROF_EMBED, 0.0, (double)c->esz * n * w * 2.0,
        [&] { launch_gather_rows(c->stream, c->dt, wh(c, ad.E[k]), w, ad.in_tok + ad.in_off[k], ad.Xc[k], w, n); });
    gemm(c, 0, n, d, w, ad.Xc[k], w, wh(c, ad.P[k]), w, (char*)ad.Y + (size_t)ad.in_off[k] * d * c->esz, d);
  }
  run(c, TFM_PROF_EMBED, 0.0, (double)c->esz * T * d * 2.0, [&] {
    launch_embed_fwd(c->stream, c->dt, c->Wh, st.ids, st.pos, c->pe, emb, T, d, site_key(s, st.id, -1, 0), c->cfg.dropout,
                     ad.n ? ad.Y : nullptr);
  });
  if (pre) ln_fwd(c, st.resid[0], nullptr, st.blocks[0].ln_g, st.blocks[0].ln_b, nullptr, st.norm[0], st.mean[0], st.rstd[0], T, 0);
  for (int k = 0; k < K; ++k) {
    sublayer_fwd(s, st, k, st.norm[k], c->y);
    int g, b;
    if (pre) { g = k + 1 < K ? st.blocks[k + 1].ln_g : st.lnf_g; b = k + 1 < K ? st.blocks[k + 1].ln_b : st.lnf_b; }
    else { g = st.blocks[k].ln_g; b = st.blocks[k].ln_b; }
    ln_fwd(c, pre ? st.resid[k] : st.norm[k], c->y, g, b, st.resid[k + 1], st.norm[k + 1], st.mean[k + 1], st.rstd[k + 1], T,
           block_key(s, st, k));
  }
}

// backward of sub-layer k given dy (which lives in the block's own b.dy); writes the gradient w.r.t. its input (plus
// `residual` if given) to dout.  Weight and bias gradients are queued (see wgrad).
void sublayer_bwd(const StepCtx& s, Stream& st, int k, const void* dy, const void* fin, const void* residual, void* dout) {
  tfm_ctx* c = s.c;
  Block& b = st.blocks[k];
  const int d = c->cfg.d_model, F = c->cfg.d_ffn, T = st.rows;
  const std::vector<int>& len = st.id ? s.tlen : s.slen;
  if (b.kind == SELF) {
    wgrad(c, d, d, T, dy, d, b.ctx, d, gr(c, b.w_o), d, gr(c, b.b_o));
    gemm(c, 1, T, d, d, dy, d, wh(c, b.w_o), d, c->dctx, d);
    const char* qkv = (const char*)b.inter;
    char* dqkv = (char*)b.dint;
    attention(s, true, st, st, len, len, qkv, 3 * d, qkv + d * c->esz, 3 * d, qkv + 2 * d * c->esz, 3 * d, b.ctx, b.lse, st.id == 1,
              site_key(s, st.id, b.layer, 3), c->dctx, dqkv, 3 * d, dqkv + d * c->esz, 3 * d, dqkv + 2 * d * c->esz, 3 * d);
    gemm(c, 1, T, d, 3 * d, dqkv, 3 * d, wh(c, b.w_a), d, dout, d, nullptr, 0, nullptr, residual);
    wgrad(c, 3 * d, d, T, dqkv, 3 * d, fin, d, gr(c, b.w_a), d, gr(c, b.b_a));
  } else if (b.kind == CROSS) {
    Stream& en = c->enc;
    wgrad(c, d, d, T, dy, d, b.ctx, d, gr(c, b.w_o), d, gr(c, b.b_o));
    gemm(c, 1, T, d, d, dy, d, wh(c, b.w_o), d, c->dctx, d);
    const char* kv = (const char*)b.kv;
    char* dkv = (char*)b.dkv;
    // the gradients w.r.t. this layer's keys and values land in its columns of dkv_all; the encoder output's gradient and the
    // stacked weights' are formed from all layers at once after the decoder's backward pass (see tfm_train_step)
    attention(s, true, st, en, s.tlen, s.slen, b.inter, d, kv, c->ld_kv, kv + d * c->esz, c->ld_kv, b.ctx, b.lse, false,
              site_key(s, st.id, b.layer, 4), c->dctx, b.dint, d, dkv, c->ld_kv, dkv + d * c->esz, c->ld_kv);
    gemm(c, 1, T, d, d, b.dint, d, wh(c, b.w_a), d, dout, d, nullptr, 0, nullptr, residual);
    wgrad(c, d, d, T, b.dint, d, fin, d, gr(c, b.w_a), d, gr(c, b.b_a));
  } else {
    wgrad(c, d, F, T, dy, d, b.inter, F, gr(c, b.w_o), F, gr(c, b.b_o));
    // the saved hidden activations are positive exactly where the ReLU passed AND the unit was kept: the mask, times the
    // dropout scale
    gemm(c, 1, T, F, d, dy, d, wh(c, b.w_o), F, b.dint, F, nullptr, 0, b.inter, nullptr, false, 0, 0.f,
         1.f / (1.f - c->cfg.relu_dropout));
    gemm(c, 1, T, d, F, b.dint, F, wh(c, b.w_a), d, dout, d, nullptr, 0, nullptr, residual);
    wgrad(c, F, d, T, b.dint, F, fin, d, gr(c, b.w_a), d, gr(c, b.b_a));
  }
}

void ln_bwd(tfm_ctx* c, const void* dn, const void* add, const void* sres, const float* mean, const float* rstd, int g, int b,
            void* ds, void* ds_drop, int bias_param, int rows, uint64_t key) {
  const int d = c->cfg.d_model;
  const bool drop = c->cfg.dropout > 0.f && ds_drop;
  const double bytes = (double)c->esz * rows * d * (2.0 + (add ? 1.0 : 0.0) + 1.0 + (drop ? 1.0 : 0.0));
  // the partial sums wait in their own slice of the pool for the batched reduction of the next flush
  LnReduceJob job;
  const bool defer = c->ln_next < c->ln_slices;
  void* scratch = defer ? (void*)(c->ln_pool + (size_t)c->ln_next * c->ln_slice) : c->red_scratch;
  run(c, TFM_PROF_NORM, 0.0, bytes, [&] {
    launch_layernorm_bwd(c->stream, c->dt, dn, add, sres, mean, rstd, wh(c, g), ds, drop ? ds_drop : nullptr, gr(c, g), gr(c, b),
                         bias_param >= 0 ? gr(c, bias_param) : nullptr, rows, d, key, c->cfg.dropout, scratch, defer ? &job : nullptr);
  });
  if (defer) { c->lnq.push_back(job); c->ln_next += 1; }
}

// Backward through a stream.  On entry c->dcur holds the gradient w.r.t. the stream output norm[K]; returns the buffer
// holding the gradient w.r.t. the embedding output.
void* stream_bwd(const StepCtx& s, Stream& st, void* dn_in) {
  tfm_ctx* c = s.c;
  const int K = (int)st.blocks.size(), T = st.rows;
  const bool pre = c->cfg.pre_norm != 0;
  const bool drop = c->cfg.dropout > 0.f;
  // Every gradient w.r.t. a block output is consumed by the LayerNorm-backward kernel before the sub-layer's last
  // GEMM writes the next one, so a single buffer (dcur) carries it down the stack.
  void* dn = dn_in;
  if (!pre) {
    for (int k = K - 1; k >= 0; --k) {
      Block& b = st.blocks[k];
      // with dropout the kernel writes both the residual branch's gradient (dsA) and the sub-layer's (b.dy); without, they
      // are the same tensor
      void* ds = drop ? c->dsA : b.dy;
      ln_bwd(c, dn, nullptr, st.resid[k + 1], st.mean[k + 1], st.rstd[k + 1], b.ln_g, b.ln_b, ds, b.dy, -1, T, block_key(s, st, k));
      void* out = k == 0 ? c->demb[st.id] : c->dcur;
      sublayer_bwd(s, st, k, b.dy, st.norm[k], ds, out);
      dn = out;
    }
    return dn;
  }
  // pre-norm: the residual stream's gradient ping-pongs between dsA and dsB; without dropout it IS the gradient of the
  // sub-layer below and is written straight into that block's own buffer
  void* dR = nullptr;
  void* pp = c->dsA;
  void* pp_alt = c->dsB;
  for (int idx = K; idx >= 0; --idx) {
    const int g = idx < K ? st.blocks[idx].ln_g : st.lnf_g;
    const int b = idx < K ? st.blocks[idx].ln_b : st.lnf_b;
    void* bdy = idx >= 1 ? st.blocks[idx - 1].dy : nullptr;
    void* ds = idx == 0 ? c->demb[st.id] : (drop ? pp : bdy);
    ln_bwd(c, dn, dR, st.resid[idx], st.mean[idx], st.rstd[idx], g, b, ds, bdy, -1, T, idx >= 1 ? block_key(s, st, idx - 1) : 0);
    if (idx == 0) return ds;
    sublayer_bwd(s, st, idx - 1, bdy, st.norm[idx - 1], nullptr, c->dcur);
    dn = c->dcur;
    dR = ds;
    std::swap(pp, pp_alt);
  }
  return nullptr;
}

// Adaptive softmax, tail clusters (the head went through the ordinary vocabulary path with the cluster entries as
// extra classes): for the positions whose target lies in cluster k, project the state down with the cluster's input
// projection transposed, score the cluster's tokens with its input table, take the loss in place, and send the
// gradients back: into the table, the projection, and (scattered) into dcur.
void adaptive_tails(const StepCtx& s, const void* top, float mult) {
  tfm_ctx* c = s.c;
  const Adaptive& ad = c->ad;
  const int d = c->cfg.d_model;
  const size_t esz = c->esz;
  char* Zt = (char*)c->logits + (((size_t)c->cfg.max_tokens * ad.v0 * esz + 255) & ~(size_t)255);
  for (int k = 1; k <= ad.n; ++k) {
    const int n = ad.out_cnt[k], w = ad.width[k], Vk = ad.hi[k] - ad.lo[k], off = ad.out_off[k];
    void* gE = gr(c, ad.E[k]);
    if (n == 0) {                                   // no target in this cluster: its table gets no output-side gradient
      hipMemsetAsync(gE, 0, (size_t)Vk * w * esz, c->stream);
      continue;
    }
    const void* Pk = wh(c, ad.P[k]);
    const void* Ek = wh(c, ad.E[k]);
    run(c, TFM_PROF_EMBED, 0.0, (double)esz * n * d * 2.0, [&] { launch_gather_rows(c->stream, c->dt, top, d, ad.out_idx + off, ad.Hc, d, n); });
    gemm(c, 1, n, w, d, ad.Hc, d, Pk, w, ad.U[k], w);                       // u = P^T h
    gemm(c, 0, n, Vk, w, ad.U[k], w, Ek, w, Zt, Vk);                         // z = E u
    run(c, TFM_PROF_LOSS, 0.0, 2.0 * esz * (double)n * Vk, [&] {
      launch_loss(c->stream, c->dt, Zt, ad.out_lab + off, ad.tail_loss + off, ad.tail_nll + off, n, Vk, 0.f, &c->st->loss_scale, mult, nullptr);
    });
    gemm(c, 1, n, w, Vk, Zt, Vk, Ek, w, ad.dU[k], w);                        // du = E^T dz
    gemm(c, 2, Vk, w, n, Zt, Vk, ad.U[k], w, gE, w);                         // dE = dz^T u
    gemm(c, 0, n, d, w, ad.dU[k], w, Pk, w, ad.dHc, d);                      // dh = P du
    // dP (output side) = h^T du; the input side adds its own share if the cluster also occurs among the inputs
    gemm(c, 2, d, w, n, ad.Hc, d, ad.dU[k], w, ad.in_cnt[k] ? ad.tmpP[k] : gr(c, ad.P[k]), w);
    run(c, TFM_PROF_EMBED, 0.0, (double)esz * n * d * 3.0, [&] {
      launch_scatter_add_rows(c->stream, c->dt, c->dcur, d, ad.out_idx + off, ad.dHc, d, n);
      launch_scatter_add_f32(c->stream, c->loss_rows, c->nll_rows, ad.out_idx + off, ad.tail_loss + off, ad.tail_nll + off, n);
    });
  }
}

// Adaptive inputs, backward: ddec is the gradient w.r.t. the embedding output.  For the positions fed with a token of
// tail cluster k: gather sqrt(d) * dropout-backward(ddec), pull it through the projection, add the rows of equal
// tokens into the table's gradient (segments in a fixed order) and form the projection's gradient.
void adaptive_embed_bwd(const StepCtx& s, const void* ddec) {
  tfm_ctx* c = s.c;
  const Adaptive& ad = c->ad;
  const int d = c->cfg.d_model;
  const size_t esz = c->esz;
  for (int k = 1; k <= ad.n; ++k) {
    const int n = ad.in_cnt[k], w = ad.width[k], off = ad.in_off[k];
    if (n == 0) {
      if (ad.out_cnt[k] == 0) hipMemsetAsync(gr(c, ad.P[k]), 0, (size_t)d * w * esz, c->stream);
      continue;
    }
    run(c, TFM_PROF_EMBED, 0.0, (double)esz * n * d * 2.0, [&] {
      launch_gather_dx(c->stream, c->dt, ddec, ad.in_idx + off, ad.dY, d, n, sqrtf((float)d), site_key(s, 1, -1, 0), c->cfg.dropout);
    });
    gemm(c, 1, n, w, d, ad.dY, d, wh(c, ad.P[k]), w, ad.dXc[k], w);           // dx_narrow = P^T dy
    gemm(c, 2, d, w, n, ad.dY, d, ad.Xc[k], w, gr(c, ad.P[k]), w, nullptr, 0, nullptr, ad.out_cnt[k] ? ad.tmpP[k] : nullptr);
    run(c, TFM_PROF_EMBED, 0.0, (double)esz * n * w * 3.0, [&] {
      launch_segsum_add_rows(c->stream, c->dt, gr(c, ad.E[k]), ad.dXc[k], w, ad.sg_tok + ad.sg_off[k], ad.sg_beg + ad.sg_off[k],
                             ad.sg_end + ad.sg_off[k], ad.sg_ent, ad.sg_cnt[k]);
    });
  }
}

}  // namespace

extern "C" {

int tfm_train_step(tfm_ctx* c, const int32_t* src, const int32_t* tgt, const int32_t* src_lens, const int32_t* tgt_lens,
                   int32_t B, int32_t Ls, int32_t Lt, tfm_step_out* out) {
  if (!c) return TFM_EINVAL;
  const tfm_config& cf = c->cfg;
  const bool has_enc = cf.enc_layers > 0;
  // ---- validation: nothing is enqueued before every check has passed
  if (!tgt || !tgt_lens) return fail(c, TFM_EINVAL, "tgt and tgt_lens are required");
  if (has_enc && (!src || !src_lens)) return fail(c, TFM_EINVAL, "src and src_lens are required for an encoder-decoder model");
  if (!has_enc && (src || src_lens)) return fail(c, TFM_EINVAL, "src must be NULL for a decoder-only model");
  if (B < 1 || B > cf.max_sentences) return fail(c, TFM_EINVAL, "B = %d outside [1, %d]", B, cf.max_sentences);
  if (Lt < 1 || Lt > cf.max_len || (has_enc && (Ls < 1 || Ls > cf.max_len))) return fail(c, TFM_EINVAL, "padded length outside [1, %d]", cf.max_len);
  long long Ts = 0, Tt = 0;
  for (int b = 0; b < B; ++b) {
    if (tgt_lens[b] < 1 || tgt_lens[b] > Lt) return fail(c, TFM_EINVAL, "tgt_lens[%d] = %d outside [1, %d]", b, tgt_lens[b], Lt);
    Tt += tgt_lens[b];
    if (has_enc) {
      if (src_lens[b] < 1 || src_lens[b] > Ls) return fail(c, TFM_EINVAL, "src_lens[%d] = %d outside [1, %d]", b, src_lens[b], Ls);
      Ts += src_lens[b];
    }
  }
  if (Tt > cf.max_tokens || Ts > cf.max_tokens) return fail(c, TFM_EINVAL, "%lld source / %lld target tokens exceed max_tokens = %d", Ts, Tt, cf.max_tokens);
  for (int b = 0; b < B; ++b) {
    for (int t = 0; t < tgt_lens[b]; ++t) {
      const int id = tgt[(size_t)b * Lt + t];
      if (id < 0 || id >= cf.vocab) return fail(c, TFM_EINVAL, "tgt[%d,%d] = %d outside the vocabulary", b, t, id);
    }
    if (has_enc) for (int t = 0; t < src_lens[b]; ++t) {
      const int id = src[(size_t)b * Ls + t];
      if (id < 0 || id >= cf.vocab) return fail(c, TFM_EINVAL, "src[%d,%d] = %d outside the vocabulary", b, t, id);
    }
  }

  c->generation += 1;
  // ---- ingest: pack into the staging slot
  const int slot = c->stage_next;
  c->stage_next = (slot + 1) % STAGE_SLOTS;
  if (c->stage_used[slot]) HIP_TRY(c, hipEventSynchronize(c->stage_ev[slot]));
  int* hb = c->stage[slot];
  const size_t R = (size_t)cf.max_tokens, Bc = (size_t)cf.max_sentences + 1;
  int* e_ids = hb; int* e_pos = e_ids + R; int* e_off = e_pos + R;
  int* d_ids = e_off + Bc; int* d_pos = d_ids + R; int* d_off = d_pos + R;
  int* labels = d_off + Bc;
  const size_t NS = 2 * R + 2 * R / EMB_SEG + 2, NM = 2 * R / EMB_SEG + 2;
  int* uent = labels + R;
  int* seg_tok = uent + 2 * R; int* seg_beg = seg_tok + NS; int* seg_end = seg_beg + NS; int* seg_dst = seg_end + NS;
  int* mt_tok = seg_dst + NS; int* mt_row0 = mt_tok + NM; int* mt_n = mt_row0 + NM;
  Adaptive& ad = c->ad;
  int* a_in_idx = mt_n + NM; int* a_in_tok = a_in_idx + R; int* a_out_idx = a_in_tok + R; int* a_out_lab = a_out_idx + R;
  int* a_sg_tok = a_out_lab + R; int* a_sg_beg = a_sg_tok + R; int* a_sg_end = a_sg_beg + R; int* a_sg_ent = a_sg_end + R;
  StepCtx s{c};
  s.B = B; s.Ts = (int)Ts; s.Tt = (int)Tt; s.step = c->train_steps;
  s.tlen.assign(tgt_lens, tgt_lens + B);
  if (has_enc) s.slen.assign(src_lens, src_lens + B);
  int r = 0, maxs = 0, maxt = 0;
  if (has_enc) {
    for (int b = 0; b < B; ++b) {
      e_off[b] = r;
      for (int t = 0; t < src_lens[b]; ++t, ++r) { e_ids[r] = src[(size_t)b * Ls + t]; e_pos[r] = t; }
      maxs = std::max(maxs, src_lens[b]);
    }
    e_off[B] = r;
  }
  r = 0;
  for (int b = 0; b < B; ++b) {
    d_off[b] = r;
    for (int t = 0; t < tgt_lens[b]; ++t, ++r) {
      labels[r] = tgt[(size_t)b * Lt + t];
      d_ids[r] = t == 0 ? cf.eos_id : tgt[(size_t)b * Lt + t - 1];   // teacher forcing: eos, then the target shifted right
      d_pos[r] = t;
    }
    maxt = std::max(maxt, tgt_lens[b]);
  }
  d_off[B] = r;
  // token -> occurrences (counting sort over the vocabulary; order: encoder rows, then decoder rows, ascending)
  int nu = 0, n_seg = 0, n_multi = 0;
  {
    std::vector<int>& cnt = c->count;
    c->uniq.resize(2 * R + 1);
    c->ustart.resize(2 * R + 2);
    int* uniq = c->uniq.data();
    int* ustart = c->ustart.data();
    // (adaptive inputs: only head tokens live in "embed"; tail tokens are grouped per cluster below)
    const int head_end = ad.n ? ad.hi[0] : cf.vocab;
    for (int i = 0; i < (int)Ts; ++i) if (cnt[e_ids[i]]++ == 0) uniq[nu++] = e_ids[i];
    for (int i = 0; i < (int)Tt; ++i) if (d_ids[i] < head_end && cnt[d_ids[i]]++ == 0) uniq[nu++] = d_ids[i];
    std::sort(uniq, uniq + nu);
    int acc = 0;
    for (int u = 0; u < nu; ++u) { ustart[u] = acc; const int n = cnt[uniq[u]]; cnt[uniq[u]] = acc; acc += n; }
    ustart[nu] = acc;
    for (int i = 0; i < (int)Ts; ++i) uent[cnt[e_ids[i]]++] = i;
    for (int i = 0; i < (int)Tt; ++i) if (d_ids[i] < head_end) uent[cnt[d_ids[i]]++] = (1 << 30) | i;
    for (int u = 0; u < nu; ++u) cnt[uniq[u]] = 0;
    // cut every token's occurrence list into segments of at most EMB_SEG entries
    int prow = 0;
    for (int u = 0; u < nu; ++u) {
      const int b0 = ustart[u], e0 = ustart[u + 1], ns = (e0 - b0 + EMB_SEG - 1) / EMB_SEG;
      if (ns > 1) { mt_tok[n_multi] = uniq[u]; mt_row0[n_multi] = prow; mt_n[n_multi] = ns; ++n_multi; }
      for (int k = 0; k < ns; ++k) {
        seg_tok[n_seg] = uniq[u];
        seg_beg[n_seg] = b0 + k * EMB_SEG;
        seg_end[n_seg] = std::min(e0, b0 + (k + 1) * EMB_SEG);
        seg_dst[n_seg] = ns > 1 ? prow++ : -1;
        ++n_seg;
      }
    }
  }
  if (ad.n) {
    // Input side: the positions whose token lies in tail cluster k, in order; their ids become -1 - (compact row) so
    // that the embedding kernel reads the projected vector.  Rows of equal token form a segment of the table's gradient.
    for (int k = 0; k <= ad.n; ++k) ad.in_cnt[k] = ad.out_cnt[k] = ad.sg_cnt[k] = 0;
    for (int i = 0; i < (int)Tt; ++i) { ad.in_cnt[ad.cluster_of(d_ids[i])]++; ad.out_cnt[ad.cluster_of(labels[i])]++; }
    int acc_in = 0, acc_out = 0;
    for (int k = 1; k <= ad.n; ++k) { ad.in_off[k] = acc_in; acc_in += ad.in_cnt[k]; ad.out_off[k] = acc_out; acc_out += ad.out_cnt[k]; }
    int fill_in[4] = {0, 0, 0, 0}, fill_out[4] = {0, 0, 0, 0};
    for (int i = 0; i < (int)Tt; ++i) {
      const int ki = ad.cluster_of(d_ids[i]);
      if (ki) {
        const int row = ad.in_off[ki] + fill_in[ki]++;
        a_in_idx[row] = i;
        a_in_tok[row] = d_ids[i] - ad.lo[ki];
        d_ids[i] = -1 - row;
      }
      const int ko = ad.cluster_of(labels[i]);
      if (ko) {
        const int row = ad.out_off[ko] + fill_out[ko]++;
        a_out_idx[row] = i;
        a_out_lab[row] = labels[i] - ad.lo[ko];
        labels[i] = ad.hi[0] + ko - 1;                     // the head predicts the cluster
      }
    }
    int nseg = 0;
    std::vector<std::pair<int, int>>& pairs = c->ad_pairs;
    for (int k = 1; k <= ad.n; ++k) {
      pairs.clear();
      for (int j = 0; j < ad.in_cnt[k]; ++j) pairs.emplace_back(a_in_tok[ad.in_off[k] + j], j);
      std::sort(pairs.begin(), pairs.end());
      ad.sg_off[k] = nseg;
      for (size_t j = 0; j < pairs.size(); ++j) {
        a_sg_ent[ad.in_off[k] + j] = pairs[j].second;      // row of this cluster's compact matrices
        if (j == 0 || pairs[j].first != pairs[j - 1].first) {
          a_sg_tok[nseg] = pairs[j].first;
          a_sg_beg[nseg] = ad.in_off[k] + (int)j;
          if (j) a_sg_end[nseg - 1] = ad.in_off[k] + (int)j;
          ++nseg;
        }
      }
      if (!pairs.empty()) a_sg_end[nseg - 1] = ad.in_off[k] + (int)pairs.size();
      ad.sg_cnt[k] = nseg - ad.sg_off[k];
    }
  }
  // Short sentences share attention blocks: runs of at most 16 consecutive sentences whose query rows and key rows each fill
  // at most one 64-row tile (the one-chunk attention kernels take the table; not used with longer sentences in the batch, nor
  // when no two sentences fit together).
  {
    int* grp = hb + (c->grp[0] - c->ibase);
    auto build = [&](const int32_t* lq, const int32_t* lk, int maxq, int maxk, int* out) {
      if (maxq > 64 || maxk > 64) return 0;
      int n = 0, first = 0, sq = 0, sk = 0, rq = 0, rk = 0;            // rq, rk: rows before sentence b
      out[0] = 0; out[1] = 0; out[2] = 0; out[3] = 0;
      for (int b = 0; b < B; ++b) {
        if (b > first && (sq + lq[b] > 64 || sk + lk[b] > 64 || b - first >= 16)) {
          ++n;
          out[4 * n] = b; out[4 * n + 1] = rq; out[4 * n + 2] = rk; out[4 * n + 3] = 0;
          first = b; sq = sk = 0;
        }
        sq += lq[b]; sk += lk[b]; rq += lq[b]; rk += lk[b];
      }
      ++n;
      out[4 * n] = B; out[4 * n + 1] = rq; out[4 * n + 2] = rk; out[4 * n + 3] = 0;
      return n < B ? n : 0;                                            // one sentence per group everywhere: nothing to pack
    };
    if (has_enc) {
      s.n_grp[0] = build(src_lens, src_lens, maxs, maxs, grp);
      s.n_grp[2] = build(tgt_lens, src_lens, maxt, maxs, grp + 8 * Bc);
    }
    s.n_grp[1] = build(tgt_lens, tgt_lens, maxt, maxt, grp + 4 * Bc);
  }
  HIP_TRY(c, hipMemcpyAsync(c->ibase, hb, c->int_block_ints * 4, hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipEventRecord(c->stage_ev[slot], c->stream));
  c->stage_used[slot] = true;
  c->enc.rows = (int)Ts; c->enc.max_len = maxs;
  c->dec.rows = (int)Tt; c->dec.max_len = maxt;

  const int d = cf.d_model, V = cf.vocab;
  // a second sub-batch in the window: move the first one's gradient into the fp32 accumulator before g is reused
  if (c->window_mb == 1)
    run(c, TFM_PROF_OPTIM, 0.0, (double)c->P * (c->esz + 4.0), [&] { launch_convert(c->stream, c->dt, c->g, F32, c->G, c->P); });

  // ---- forward
  c->sync_used = 0;
  c->wq.clear();
  c->wq_tiles = 0;
  c->lnq.clear();
  c->ln_next = 0;
  c->kv_ready = nullptr;
  if (has_enc) {
    stream_fwd(s, c->enc);
    // Every decoder layer's cross-attention keys and values depend on the encoder output alone: one product with the
    // stacked weights projects them all.  With the side stream on it runs there beside the decoder's first block, and
    // the first cross-attention block waits for it.
    const void* mem = c->enc.norm[c->enc.blocks.size()];
    need(c, c->kv_b0 + cf.dec_layers - 1);
    if (c->overlap) side_begin(c);
    gemm(c, 0, c->enc.rows, c->ld_kv, d, mem, d, wh(c, c->kv_w0), d, c->kv_all, c->ld_kv, wh(c, c->kv_b0), 0, nullptr, nullptr, true);
    if (c->overlap) c->kv_ready = mark(c, c->side);
  }
  stream_fwd(s, c->dec);
  Stream& de = c->dec;
  const int Kd = (int)de.blocks.size();
  const void* top = de.norm[Kd];
  adam_join(c);                                    // every parameter has been touched by now; nothing is left pending
  // flat vocabulary: all V logits; adaptive softmax: the head's tokens plus one entry per tail cluster
  const int V0 = ad.n ? ad.v0 : V;
  gemm(c, 0, (int)Tt, V0, d, top, d, c->Wh, d, c->logits, V0);
  const float mult = c->next_mult;
  c->next_mult = 1.f;
  run(c, TFM_PROF_LOSS, 0.0, 2.0 * c->esz * (double)Tt * V0, [&] {
    launch_loss(c->stream, c->dt, c->logits, c->labels, c->loss_rows, c->nll_rows, (int)Tt, V0, cf.label_smoothing, &c->st->loss_scale,
                mult, &c->st->step_scale);
  });

  // ---- backward
  wgrad(c, V0, d, (int)Tt, c->logits, V0, top, d, c->g, d);                // embedding gradient, output side
  gemm(c, 1, (int)Tt, d, V0, c->logits, V0, c->Wh, d, c->dcur, d);
  if (ad.n) adaptive_tails(s, top, mult);          // tail clusters: their losses, gradients, and their share of dcur
  run(c, TFM_PROF_LOSS, 0.0, 8.0 * (double)Tt, [&] { launch_sum_rows(c->stream, c->loss_rows, c->nll_rows, (int)Tt, &c->st->loss_sum); });
  void* ddec = stream_bwd(s, de, c->dcur);
  void* denc = nullptr;
  if (has_enc) {
    // all layers' key/value gradients at once: the encoder output's gradient (one product over the layers * 2d columns) and
    // the stacked projection weights' and biases'
    const void* mem = c->enc.norm[c->enc.blocks.size()];
    gemm(c, 1, c->enc.rows, d, c->ld_kv, c->dkv_all, c->ld_kv, wh(c, c->kv_w0), d, c->dmem, d);
    wgrad(c, c->ld_kv, d, c->enc.rows, c->dkv_all, c->ld_kv, mem, d, gr(c, c->kv_w0), d, gr(c, c->kv_b0));
  }
  flush_wgrads(c);                                 // the decoder's weight gradients run beside the encoder's backward pass
  if (has_enc) denc = stream_bwd(s, c->enc, c->dmem);
  flush_wgrads(c);
  if (c->overlap) order(c, c->side, c->stream);                            // join: every weight gradient is in g
  if (ad.n) adaptive_embed_bwd(s, ddec);
  run(c, TFM_PROF_EMBED, 0.0, (double)c->esz * d * ((double)Ts + Tt + 2.0 * nu), [&] {
    EmbedBwdArgs ea{};
    ea.dt = c->dt; ea.gE = c->g; ea.partial = c->emb_partial;
    ea.seg_tok = c->seg_tok; ea.seg_beg = c->seg_beg; ea.seg_end = c->seg_end; ea.seg_dst = c->seg_dst;
    ea.entries = c->uentries; ea.n_seg = n_seg;
    ea.mt_tok = c->mt_tok; ea.mt_row0 = c->mt_row0; ea.mt_n = c->mt_n; ea.n_multi = n_multi;
    ea.dx0 = denc; ea.dx1 = ddec; ea.d = d; ea.key0 = site_key(s, 0, -1, 0); ea.key1 = site_key(s, 1, -1, 0); ea.p = cf.dropout;
    launch_embed_bwd(c->stream, ea);
  });

  // ---- inf/nan scan of this sub-batch's gradient (+ accumulation from the second sub-batch on)
  const int acc_mode = c->window_mb >= 1 ? 2 : 0;
  run(c, TFM_PROF_OPTIM, 0.0, (double)c->P * (c->esz + (acc_mode ? 8.0 : 0.0)), [&] {
    launch_scan(c->stream, c->dt, c->g, c->P, nullptr, c->st, acc_mode ? c->G : nullptr, acc_mode, c->scan_scratch);
  });
  c->window_mb += 1;
  c->window_tokens += Tt;
  c->train_steps += 1;
  HIP_TRY(c, hipGetLastError());
  if (out) {
    DevState h;
    HIP_TRY(c, hipMemcpyAsync(&h, c->st, sizeof(h), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    out->loss_sum = h.loss_sum; out->nll_sum = h.nll_sum; out->ntokens = Tt; out->overflow = h.step_overflow;
    out->loss_scale = h.loss_scale;
    // an update enqueued without synchronisation may have taken the scale below the minimum: this is where it shows
    if (h.scale_too_small) return fail(c, TFM_ESCALE, "loss scale %g is below the minimum %g", h.loss_scale, cf.min_loss_scale);
  }
  return TFM_OK;
}

int tfm_apply_update(tfm_ctx* c, float lr, tfm_update_out* out) {
  if (!c) return TFM_EINVAL;
  if (c->window_mb == 0) return fail(c, TFM_ESTATE, "no sub-batch has been accumulated");
  if (!std::isfinite(lr)) return fail(c, TFM_EINVAL, "learning rate is not finite");
  adam_join(c);
  c->generation += 1;
  const tfm_config& cf = c->cfg;
  const bool single = c->window_mb == 1;
  // the scan of a single sub-batch already produced the sum of squares; an accumulated window is scanned again
  if (!single)
    run(c, TFM_PROF_OPTIM, 0.0, (double)c->P * 4.0, [&] {
      // window_overflow is sticky (|=) so this scan cannot clear an earlier sub-batch's flag
      launch_scan(c->stream, F32, c->G, c->P, nullptr, c->st, nullptr, 0, c->scan_scratch);
    });
  launch_scaler_update(c->stream, c->st, c->window_tokens, cf.clip_norm, cf.adam_beta1, cf.adam_beta2, cf.scale_window,
                       cf.min_loss_scale, cf.precision == TFM_FP16 ? 1 : 0);
  AdamArgs a{};
  a.w = c->W; a.m = c->M; a.v = c->V; a.n = c->P;
  a.g = single ? c->g : (const void*)c->G; a.gdt = single ? c->dt : (int)F32;
  a.half_copy = c->dt == F32 ? nullptr : c->Wh; a.hdt = c->dt;
  a.lr = lr; a.beta1 = cf.adam_beta1; a.beta2 = cf.adam_beta2; a.eps = cf.adam_eps; a.weight_decay = cf.weight_decay; a.st = c->st;
  const double bpp = 24.0 + (single ? c->esz : 4.0) + (c->dt == F32 ? 0.0 : 2.0);
  if (!c->overlap) {
    run(c, TFM_PROF_OPTIM, 0.0, (double)c->P * bpp, [&] { launch_adam(c->stream, a); });
  } else {
    c->sync_used = 0;
    order(c, c->stream, c->side);                  // the step scalars are in the device state
    const size_t gsz = single ? c->esz : 4;
    for (size_t k = 0; k < c->chunks.size(); ++k) {
      const tfm_ctx::Chunk& ch = c->chunks[k];
      AdamArgs b = a;
      b.w = c->W + ch.off; b.m = c->M + ch.off; b.v = c->V + ch.off; b.n = ch.n;
      b.g = (const char*)a.g + ch.off * gsz;
      b.half_copy = a.half_copy ? (char*)a.half_copy + ch.off * c->esz : nullptr;
      run(c, TFM_PROF_OPTIM, 0.0, (double)ch.n * bpp, [&] { launch_adam(c->side, b); }, c->side);
      hipEventRecord(c->adam_ev[k], c->side);
    }
    c->adam_pending = true;
    c->adam_waited = 0;
  }
  const long long ntok = c->window_tokens;
  c->window_mb = 0;
  c->window_tokens = 0;
  HIP_TRY(c, hipGetLastError());
  if (out) {
    adam_join(c);
    DevState h;
    HIP_TRY(c, hipMemcpyAsync(&h, c->st, sizeof(h), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    out->skipped = h.skipped; out->loss_scale_after = h.loss_scale; out->clean_steps = h.clean_steps;
    out->num_updates = h.num_updates; out->grad_norm = h.grad_norm; out->ntokens_total = ntok;
    if (h.scale_too_small) return fail(c, TFM_ESCALE, "loss scale %g fell below the minimum %g", h.loss_scale, cf.min_loss_scale);
  }
  return TFM_OK;
}

// ---- incremental decoding -----------------------------------------------------------------------------------------------------
struct tfm_decoder {
  tfm_ctx* c;
  int max_rows, max_steps, max_src, topk;
  // device buffers (caller's workspace)
  void *resid[2], *norm[2], *y, *qkv, *att, *q, *inter, *logits;
  float *mean, *rstd, *lse, *top_logp, *lp_stage;
  int *top_id, *anc[2], *ibuf;
  int* src_off;                                    // [max_sentences + 1]: this batch's source offsets (the context's are re-used by training)
  // adaptive inputs / adaptive softmax (null without clusters)
  void *a_head, *a_tail, *a_u, *a_xc, *a_y;        // head scores [R, v0]; one tail cluster's scores [R, vmax]; projected state [R, wmax];
                                                   // gathered narrow input rows [R, wmax]; projected input vectors [R, d]
  float *a_lse, *a_lp1;                            // [R]: a cluster's log-sum-exp; throw-away best value of that pass
  int* a_id1;                                      // [R]: throw-away best id
  std::vector<void*> Kc, Vc, xkv;                  // per decoder layer
  // pinned host staging
  int* h_in;                                       // prev, parent, pos [3 * max_rows]; also source ids / pos / offsets
  size_t h_in_ints;
  float* h_out;                                    // top_logp [max_rows * topk] followed by top_id
  // state of the batch being decoded
  int B, beam, rows, t, cur, n_src_max, src_rows;
  uint64_t generation;                             // the context's when the batch began
  bool begun;
};

namespace {

size_t decoder_carve(tfm_decoder* D, char* base) {
  tfm_ctx* c = D->c;
  const tfm_config& cf = c->cfg;
  const size_t R = (size_t)D->max_rows, d = cf.d_model, F = cf.d_ffn, esz = c->esz;
  Arena a{base};
  for (int i = 0; i < 2; ++i) { D->resid[i] = a.take(R * d * esz); D->norm[i] = a.take(R * d * esz); }
  D->y = a.take(R * d * esz);
  D->qkv = a.take(R * 3 * d * esz);
  D->att = a.take(R * d * esz);
  D->q = a.take(R * d * esz);
  D->inter = a.take(R * F * esz);
  D->logits = a.take(R * (size_t)cf.vocab * esz);
  D->mean = (float*)a.take(R * 4);
  D->rstd = (float*)a.take(R * 4);
  D->lse = (float*)a.take(R * 4);
  D->top_logp = (float*)a.take(R * D->topk * 8);   // values, then ids: one device-to-host copy per step
  D->top_id = base ? (int*)(D->top_logp + R * D->topk) : nullptr;
  D->lp_stage = (float*)a.take((size_t)16 * cf.vocab * 4);
  D->anc[0] = (int*)a.take(R * D->max_steps * 4);
  D->anc[1] = (int*)a.take(R * D->max_steps * 4);
  D->ibuf = (int*)a.take(4 * R * 4);              // token, parent, position, index into a tail cluster's table
  D->src_off = (int*)a.take(((size_t)cf.max_sentences + 1) * 4);
  if (c->ad.n) {
    const Adaptive& ad = c->ad;
    size_t wmax = 0;
    for (int k = 1; k <= ad.n; ++k) wmax = std::max(wmax, (size_t)ad.width[k]);
    D->a_head = a.take(R * (size_t)ad.v0 * esz);
    D->a_tail = a.take(R * (size_t)ad.vmax * esz);
    D->a_u = a.take(R * wmax * esz);
    D->a_xc = a.take(R * wmax * esz);
    D->a_y = a.take(R * d * esz);
    D->a_lse = (float*)a.take(R * 4);
    D->a_lp1 = (float*)a.take(R * 4);
    D->a_id1 = (int*)a.take(R * 4);
  }
  D->Kc.assign(cf.dec_layers, nullptr); D->Vc.assign(cf.dec_layers, nullptr); D->xkv.assign(cf.dec_layers, nullptr);
  for (int l = 0; l < cf.dec_layers; ++l) {
    D->Kc[l] = a.take(R * D->max_steps * d * esz);
    D->Vc[l] = a.take(R * D->max_steps * d * esz);
    if (cf.enc_layers) D->xkv[l] = a.take((size_t)D->max_src * 2 * d * esz);
  }
  return (a.off + 255) & ~(size_t)255;
}

int decoder_check(const tfm_ctx* c, int max_rows, int max_steps, int max_src, int topk) {
  if (!c) return TFM_EINVAL;
  const tfm_config& cf = c->cfg;
  if (max_rows < 1 || max_steps < 1 || max_steps > cf.max_len || topk < 1 || topk > 16 || topk > cf.vocab) return TFM_EINVAL;
  if (cf.enc_layers && (max_src < 1 || max_src > cf.max_tokens)) return TFM_EINVAL;
  // the attention kernel keeps element offsets into one cache in 32 bits
  if ((double)max_rows * max_steps * cf.d_model >= 2147483648.0 || (double)std::max(max_src, 1) * 2 * cf.d_model >= 2147483648.0) return TFM_EINVAL;
  return TFM_OK;
}

// bias_param: the bias the deferred slices still lack (used only with splits > 0)
void decode_ln(tfm_decoder* D, const void* x, const void* y, int g, int b, void* s_out, void* n_out, int splits = 0, int bias_param = -1) {
  tfm_ctx* c = D->c;
  const int d = c->cfg.d_model;
  if (splits > 0) {
    run(c, TFM_PROF_NORM, 0.0, (double)D->rows * d * (4.0 * splits + c->esz * (2.0 + (s_out ? 1.0 : 0.0))), [&] {
      launch_splitk_layernorm_fwd(c->stream, c->dt, x, (const float*)c->splitk_ws, splits, bias_param >= 0 ? wh(c, bias_param) : nullptr,
                                  wh(c, g), wh(c, b), s_out, n_out, D->rows, d);
    });
    return;
  }
  run(c, TFM_PROF_NORM, 0.0, (double)c->esz * D->rows * d * (2.0 + (y ? 1.0 : 0.0) + (s_out ? 1.0 : 0.0)), [&] {
    launch_residual_layernorm_fwd(c->stream, c->dt, x, y, wh(c, g), wh(c, b), s_out, n_out, D->mean, D->rstd, D->rows, d, 0, 0.f);
  });
}

// qkv_new (self-attention): the step's fused [rows, 3d] projection, whose keys and values are to be appended to the caches k
// and v at position t: by the attention kernel itself where it can, else by a copy kernel first
void decode_attention(tfm_decoder* D, const void* q, int ldq, const void* k, const void* v, int row_stride, const int* anc, int n_max,
                      double positions, const void* qkv_new = nullptr, int q_splits = 0, const void* q_bias = nullptr) {
  tfm_ctx* c = D->c;
  const int d = c->cfg.d_model, H = c->cfg.n_heads;
  DecodeAttnArgs a{};
  a.dt = c->dt; a.q = q; a.ldq = ldq; a.k = k; a.v = v; a.row_stride = row_stride; a.o = D->att; a.ldo = d;
  a.anc = anc; a.src_off = D->src_off; a.rows = D->rows; a.H = H; a.dh = d / H; a.beam = D->beam; a.t = D->t;
  a.max_steps = D->max_steps; a.n_max = n_max;
  if (q_splits > 0) { a.q_partial = (const float*)c->splitk_ws; a.q_splits = q_splits; a.q_bias = q_bias; }
  if (qkv_new) {
    a.k_new = (const char*)qkv_new + (size_t)d * c->esz; a.v_new = (const char*)qkv_new + (size_t)2 * d * c->esz; a.ld_new = 3 * d;
    if (!decode_attention_appends(a)) {
      run(c, TFM_PROF_EMBED, 0.0, (double)c->esz * D->rows * d * 4.0, [&] {
        launch_cache_append(c->stream, c->dt, qkv_new, const_cast<void*>(k), const_cast<void*>(v), D->rows, d, D->max_steps, D->t);
      });
      a.k_new = a.v_new = nullptr;
    }
  }
  // positions = sum over rows of the positions attended to: K and V rows read once each, q read, output written
  run(c, TFM_PROF_ATTENTION, 4.0 * d * positions, (double)c->esz * d * (2.0 * positions + 2.0 * D->rows),
      [&] { launch_decode_attention(c->stream, a); });
}

// y = f_k(fin) for the single new position of every row
// y = f_k(fin) for the step's rows.  The sub-layer's last product has few tiles and usually runs split along K: its fp32
// slices are then left in the split-K workspace, without the bias, and their count is returned for the kernel that fuses
// their sum with the residual connection and LayerNorm (0: D->y is complete).
int decode_sublayer(tfm_decoder* D, const Block& b, int layer, const void* fin, double src_positions) {
  tfm_ctx* c = D->c;
  const int d = c->cfg.d_model, F = c->cfg.d_ffn, R = D->rows;
  int deferred = 0;
  if (b.kind == SELF) {
    gemm(c, 0, R, 3 * d, d, fin, d, wh(c, b.w_a), d, D->qkv, 3 * d, wh(c, b.b_a));
    decode_attention(D, D->qkv, 3 * d, D->Kc[layer], D->Vc[layer], d, D->anc[D->cur], D->t + 1, (double)R * (D->t + 1), D->qkv);
    gemm(c, 0, R, d, d, D->att, d, wh(c, b.w_o), d, D->y, d, wh(c, b.b_o), 0, nullptr, nullptr, false, 0, 0.f, 1.f, &deferred);
  } else if (b.kind == CROSS) {
    // (the query projection has as few tiles as the output projection: its slices are summed by the attention kernel)
    int q_splits = 0;
    gemm(c, 0, R, d, d, fin, d, wh(c, b.w_a), d, D->q, d, wh(c, b.b_a), 0, nullptr, nullptr, false, 0, 0.f, 1.f, &q_splits);
    const char* kv = (const char*)D->xkv[layer];
    decode_attention(D, D->q, d, kv, kv + d * c->esz, 2 * d, nullptr, D->n_src_max, src_positions, nullptr, q_splits, wh(c, b.b_a));
    gemm(c, 0, R, d, d, D->att, d, wh(c, b.w_o), d, D->y, d, wh(c, b.b_o), 0, nullptr, nullptr, false, 0, 0.f, 1.f, &deferred);
  } else {
    gemm(c, 0, R, F, d, fin, d, wh(c, b.w_a), d, D->inter, F, wh(c, b.b_a), 1);
    gemm(c, 0, R, d, F, D->inter, F, wh(c, b.w_o), F, D->y, d, wh(c, b.b_o), 0, nullptr, nullptr, false, 0, 0.f, 1.f, &deferred);
  }
  return deferred;
}

}  // namespace

int tfm_decoder_workspace_bytes(const tfm_ctx* c, int32_t max_rows, int32_t max_steps, int32_t max_src_tokens, int32_t topk,
                                size_t* bytes) {
  if (!bytes || decoder_check(c, max_rows, max_steps, max_src_tokens, topk)) return TFM_EINVAL;
  tfm_decoder D{};
  D.c = const_cast<tfm_ctx*>(c); D.max_rows = max_rows; D.max_steps = max_steps; D.max_src = max_src_tokens; D.topk = topk;
  *bytes = decoder_carve(&D, nullptr);
  return TFM_OK;
}

int tfm_decoder_create(tfm_ctx* c, void* ws, size_t bytes, int32_t max_rows, int32_t max_steps, int32_t max_src_tokens,
                       int32_t topk, tfm_decoder** out) {
  if (!ws || !out || decoder_check(c, max_rows, max_steps, max_src_tokens, topk)) return c ? fail(c, TFM_EINVAL, "bad decoder sizes") : TFM_EINVAL;
  if (((uintptr_t)ws & 255) != 0) return fail(c, TFM_EINVAL, "workspace must be 256-byte aligned");
  tfm_decoder* D = new tfm_decoder{};
  D->c = c; D->max_rows = max_rows; D->max_steps = max_steps; D->max_src = max_src_tokens; D->topk = topk;
  const size_t need = decoder_carve(D, nullptr);
  if (bytes < need) { delete D; return fail(c, TFM_ENOMEM, "decoder workspace has %zu bytes, %zu needed", bytes, need); }
  decoder_carve(D, (char*)ws);
  D->h_in_ints = std::max<size_t>(4 * (size_t)max_rows, 2 * (size_t)c->cfg.max_tokens + c->cfg.max_sentences + 1);
  hipError_t e = hipHostMalloc((void**)&D->h_in, D->h_in_ints * 4, hipHostMallocDefault);
  if (e == hipSuccess) e = hipHostMalloc((void**)&D->h_out, (size_t)max_rows * topk * 8, hipHostMallocDefault);
  if (e != hipSuccess) {
    if (D->h_in) hipHostFree(D->h_in);
    delete D;
    return fail(c, TFM_EHIP, "decoder staging buffers: %s", hipGetErrorString(e));
  }
  *out = D;
  return TFM_OK;
}

void tfm_decoder_destroy(tfm_decoder* D) {
  if (!D) return;
  hipStreamSynchronize(D->c->stream);
  if (D->h_in) hipHostFree(D->h_in);
  if (D->h_out) hipHostFree(D->h_out);
  delete D;
}

int tfm_decoder_begin(tfm_decoder* D, const int32_t* src, const int32_t* src_lens, int32_t B, int32_t Ls, int32_t beam) {
  if (!D) return TFM_EINVAL;
  tfm_ctx* c = D->c;
  const tfm_config& cf = c->cfg;
  const bool has_enc = cf.enc_layers > 0;
  D->begun = false;
  if (B < 1 || beam < 1 || (long long)B * beam > D->max_rows || B > cf.max_sentences)
    return fail(c, TFM_EINVAL, "B = %d sentences x beam = %d exceeds the decoder's %d rows", B, beam, D->max_rows);
  if (has_enc != (src != nullptr) || has_enc != (src_lens != nullptr)) return fail(c, TFM_EINVAL, "src is required exactly when the model has an encoder");
  long long Ts = 0;
  int maxs = 0;
  if (has_enc) {
    if (Ls < 1 || Ls > cf.max_len) return fail(c, TFM_EINVAL, "padded source length outside [1, %d]", cf.max_len);
    for (int b = 0; b < B; ++b) {
      if (src_lens[b] < 1 || src_lens[b] > Ls) return fail(c, TFM_EINVAL, "src_lens[%d] = %d outside [1, %d]", b, src_lens[b], Ls);
      for (int t = 0; t < src_lens[b]; ++t)
        if (src[(size_t)b * Ls + t] < 0 || src[(size_t)b * Ls + t] >= cf.vocab) return fail(c, TFM_EINVAL, "src[%d,%d] outside the vocabulary", b, t);
      Ts += src_lens[b];
      maxs = std::max(maxs, src_lens[b]);
    }
    if (Ts > D->max_src || Ts > cf.max_tokens) return fail(c, TFM_EINVAL, "%lld source tokens exceed the capacity", Ts);
  }
  adam_join(c);
  D->B = B; D->beam = beam; D->rows = B * beam; D->t = 0; D->cur = 0; D->n_src_max = maxs;
  if (has_enc) {
    // the encoder runs once over the packed source sentences, without dropout, in the context's own buffers
    HIP_TRY(c, hipStreamSynchronize(c->stream));             // the staging buffer may still feed an earlier copy
    const size_t R = (size_t)cf.max_tokens;
    int* ids = D->h_in; int* pos = ids + R; int* off = pos + R;
    int r = 0;
    StepCtx s{c};
    s.B = B; s.Ts = (int)Ts; s.Tt = 0; s.step = 0;
    s.slen.assign(src_lens, src_lens + B);
    for (int b = 0; b < B; ++b) {
      off[b] = r;
      for (int t = 0; t < src_lens[b]; ++t, ++r) { ids[r] = src[(size_t)b * Ls + t]; pos[r] = t; }
    }
    off[B] = r;
    HIP_TRY(c, hipMemcpyAsync(c->enc.ids, D->h_in, (2 * R + B + 1) * 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(D->src_off, off, (size_t)(B + 1) * 4, hipMemcpyHostToDevice, c->stream));
    c->enc.rows = (int)Ts; c->enc.max_len = maxs;
    const float p_train = c->cfg.dropout, pa_train = c->cfg.attn_dropout, pr_train = c->cfg.relu_dropout;
    c->cfg.dropout = c->cfg.attn_dropout = c->cfg.relu_dropout = 0.f;
    stream_fwd(s, c->enc);
    c->cfg.dropout = p_train; c->cfg.attn_dropout = pa_train; c->cfg.relu_dropout = pr_train;
    const void* mem = c->enc.norm[c->enc.blocks.size()];
    const int d = cf.d_model;
    int layer = 0;
    for (const Block& b : c->dec.blocks) {
      if (b.kind != CROSS) continue;
      gemm(c, 0, (int)Ts, 2 * d, d, mem, d, wh(c, b.w_kv), d, D->xkv[layer], 2 * d, wh(c, b.b_kv));
      ++layer;
    }
  }
  HIP_TRY(c, hipGetLastError());
  D->src_rows = (int)Ts;
  D->generation = c->generation;
  D->begun = true;
  return TFM_OK;
}

int tfm_decoder_step(tfm_decoder* D, const int32_t* prev, const int32_t* parent, float* top_logp, int32_t* top_id) {
  if (!D || !prev || !top_logp || !top_id) return TFM_EINVAL;
  tfm_ctx* c = D->c;
  const tfm_config& cf = c->cfg;
  if (!D->begun) return fail(c, TFM_ESTATE, "tfm_decoder_begin has not been called");
  if (D->generation != c->generation) {
    D->begun = false;
    return fail(c, TFM_ESTATE, "the context trained or changed parameters since tfm_decoder_begin: begin the batch again");
  }
  if (D->t >= D->max_steps) return fail(c, TFM_ESTATE, "the decoder was created for %d steps", D->max_steps);
  const int R = D->rows, d = cf.d_model, V = cf.vocab;
  for (int r = 0; r < R; ++r) {
    if (prev[r] < 0 || prev[r] >= V) return fail(c, TFM_EINVAL, "prev[%d] = %d outside the vocabulary", r, prev[r]);
    if (parent && (parent[r] < 0 || parent[r] >= R || parent[r] / D->beam != r / D->beam))
      return fail(c, TFM_EINVAL, "parent[%d] = %d is not a row of the same sentence", r, parent[r]);
  }
  // the previous step's call synchronised, so the staging buffer is free
  for (int r = 0; r < R; ++r) { D->h_in[r] = prev[r]; D->h_in[R + r] = parent ? parent[r] : r; D->h_in[2 * R + r] = D->t; }
  // Adaptive inputs: a row fed with a token of tail cluster k gets the id -1 - (its row in the compact list of projected vectors);
  // the lists are ordered by cluster, rows ascending
  const Adaptive& ad = c->ad;
  int in_cnt[4] = {0, 0, 0, 0}, in_off[4] = {0, 0, 0, 0};
  if (ad.n) {
    for (int r = 0; r < R; ++r) in_cnt[ad.cluster_of(prev[r])]++;
    for (int k = 2; k <= ad.n; ++k) in_off[k] = in_off[k - 1] + in_cnt[k - 1];
    int fill[4] = {0, 0, 0, 0};
    for (int r = 0; r < R; ++r) {
      const int k = ad.cluster_of(prev[r]);
      if (!k) continue;
      const int row = in_off[k] + fill[k]++;
      D->h_in[3 * R + row] = prev[r] - ad.lo[k];
      D->h_in[r] = -1 - row;
    }
  }
  HIP_TRY(c, hipMemcpyAsync(D->ibuf, D->h_in, (size_t)4 * R * 4, hipMemcpyHostToDevice, c->stream));
  const int* d_prev = D->ibuf; const int* d_parent = D->ibuf + R; const int* d_pos = D->ibuf + 2 * R; const int* d_in_tok = D->ibuf + 3 * R;
  run(c, TFM_PROF_EMBED, 0.0, 4.0 * R * (D->t + 1) * 2.0,
      [&] { launch_ancestry(c->stream, D->anc[D->cur], D->anc[D->cur ^ 1], d_parent, R, D->max_steps, D->t); });
  D->cur ^= 1;
  const bool pre = cf.pre_norm != 0;
  const std::vector<Block>& blocks = c->dec.blocks;
  const int K = (int)blocks.size();
  void* emb = pre ? D->resid[0] : D->norm[0];
  for (int k = 1; k <= ad.n; ++k) {                  // tail tokens: narrow table rows, projected up to the model width
    const int n = in_cnt[k], w = ad.width[k];
    if (n == 0) continue;
    run(c, TFM_PROF_EMBED, 0.0, (double)c->esz * n * w * 2.0,
        [&] { launch_gather_rows(c->stream, c->dt, wh(c, ad.E[k]), w, d_in_tok + in_off[k], D->a_xc, w, n); });
    gemm(c, 0, n, d, w, D->a_xc, w, wh(c, ad.P[k]), w, (char*)D->a_y + (size_t)in_off[k] * d * c->esz, d);
  }
  run(c, TFM_PROF_EMBED, 0.0, (double)c->esz * R * d * 2.0,
      [&] { launch_embed_fwd(c->stream, c->dt, c->Wh, d_prev, d_pos, c->pe, emb, R, d, 0, 0.f, ad.n ? D->a_y : nullptr); });
  if (pre) decode_ln(D, D->resid[0], nullptr, blocks[0].ln_g, blocks[0].ln_b, nullptr, D->norm[0]);
  double src_positions = 0;
  if (cf.enc_layers) src_positions = (double)D->src_rows * D->beam;
  for (int k = 0; k < K; ++k) {
    const int i = k & 1, j = i ^ 1;
    const int splits = decode_sublayer(D, blocks[k], blocks[k].layer, D->norm[i], src_positions);
    if (pre) {
      const int g = k + 1 < K ? blocks[k + 1].ln_g : c->dec.lnf_g, b = k + 1 < K ? blocks[k + 1].ln_b : c->dec.lnf_b;
      decode_ln(D, D->resid[i], D->y, g, b, D->resid[j], D->norm[j], splits, blocks[k].b_o);
    } else {
      decode_ln(D, D->norm[i], D->y, blocks[k].ln_g, blocks[k].ln_b, nullptr, D->norm[j], splits, blocks[k].b_o);
    }
  }
  const void* top = D->norm[K & 1];
  if (!ad.n) {
    gemm(c, 0, R, V, d, top, d, c->Wh, d, D->logits, V);
  } else {
    // Adaptive softmax: the head scores its tokens and one entry per tail cluster; a tail cluster projects the state down
    // and scores its own tokens.  All scores are assembled into one row of virtual logits over the vocabulary (see
    // launch_adaptive_virtual), which the ordinary top-k / log-softmax pass then reads.
    const int v0 = ad.v0, c0 = ad.hi[0];
    gemm(c, 0, R, v0, d, top, d, c->Wh, d, D->a_head, v0);
    run(c, TFM_PROF_LOSS, 0.0, (double)c->esz * R * c0 * 2.0,
        [&] { launch_adaptive_virtual(c->stream, c->dt, D->a_head, v0, c0, D->logits, V, 0, nullptr, 0, -1, nullptr, R); });
    for (int k = 1; k <= ad.n; ++k) {
      const int w = ad.width[k], Vk = ad.hi[k] - ad.lo[k];
      gemm(c, 1, R, w, d, top, d, wh(c, ad.P[k]), w, D->a_u, w);                      // u = P^T h
      gemm(c, 0, R, Vk, w, D->a_u, w, wh(c, ad.E[k]), w, D->a_tail, Vk);              // z = E u
      run(c, TFM_PROF_LOSS, 0.0, (double)c->esz * R * Vk * 3.0, [&] {
        launch_row_topk(c->stream, c->dt, D->a_tail, Vk, R, Vk, 1, D->a_lp1, D->a_id1, D->a_lse);   // (for its log-sum-exp)
        launch_adaptive_virtual(c->stream, c->dt, D->a_tail, Vk, Vk, D->logits, V, ad.lo[k], D->a_head, v0, c0 + k - 1, D->a_lse, R);
      });
    }
  }
  run(c, TFM_PROF_LOSS, 0.0, (double)c->esz * R * V,
      [&] { launch_row_topk(c->stream, c->dt, D->logits, V, R, V, D->topk, D->top_logp, D->top_id, D->lse); });
  const size_t n = (size_t)R * D->topk;
  HIP_TRY(c, hipMemcpyAsync(D->h_out, D->top_logp, n * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipMemcpyAsync(D->h_out + n, D->top_id, n * 4, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  HIP_TRY(c, hipGetLastError());
  std::memcpy(top_logp, D->h_out, n * 4);
  std::memcpy(top_id, D->h_out + n, n * 4);
  D->t += 1;
  return TFM_OK;
}

int tfm_decoder_get_logprobs(tfm_decoder* D, float* host, int64_t n) {
  if (!D || !host) return TFM_EINVAL;
  tfm_ctx* c = D->c;
  const int V = c->cfg.vocab;
  if (!D->begun || D->t == 0) return fail(c, TFM_ESTATE, "no step has been taken");
  if (n != (int64_t)D->rows * V) return fail(c, TFM_EINVAL, "expected rows * vocab = %lld values", (long long)D->rows * V);
  for (int r0 = 0; r0 < D->rows; r0 += 16) {
    const int nr = std::min(16, D->rows - r0);
    launch_logprob_rows(c->stream, c->dt, (const char*)D->logits + (size_t)r0 * V * c->esz, V, D->lse + r0, D->lp_stage, nr, V);
    HIP_TRY(c, hipMemcpyAsync(host + (size_t)r0 * V, D->lp_stage, (size_t)nr * V * 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
  }
  return TFM_OK;
}

// ---- single operations ---------------------------------------------------------------------------------------------------------
static int op_done() { return hipGetLastError() == hipSuccess ? TFM_OK : TFM_EHIP; }

int tfm_op_gemm(int32_t dtype, int32_t form, int32_t M, int32_t N, int32_t K, const void* A, int32_t lda, const void* B,
                int32_t ldb, void* C, int32_t ldc, const void* bias, int32_t relu, const void* mask, const void* residual,
                void* stream) {
  if (dtype < 0 || dtype > 2 || form < 0 || form > 2 || M < 0 || N < 0 || K < 0 || !A || !B || !C) return TFM_EINVAL;
  if (lda < (form == 2 ? M : K) || ldb < (form == 0 ? K : N) || ldc < N) return TFM_EINVAL;
  GemmArgs a{dtype, form, M, N, K, A, lda, B, ldb, C, ldc, bias, relu, mask, residual};
  launch_gemm((hipStream_t)stream, a);
  return op_done();
}

int tfm_op_gemm_ws(int32_t dtype, int32_t form, int32_t M, int32_t N, int32_t K, const void* A, int32_t lda, const void* B,
                   int32_t ldb, void* C, int32_t ldc, const void* bias, int32_t relu, const void* mask, const void* residual,
                   void* workspace, size_t workspace_bytes, uint64_t drop_key, float drop_p, float mask_scale, void* stream) {
  if (dtype < 0 || dtype > 2 || form < 0 || form > 2 || M < 0 || N < 0 || K < 0 || !A || !B || !C) return TFM_EINVAL;
  if (lda < (form == 2 ? M : K) || ldb < (form == 0 ? K : N) || ldc < N) return TFM_EINVAL;
  if (!(drop_p >= 0.f && drop_p < 1.f)) return TFM_EINVAL;
  GemmArgs a{dtype, form, M, N, K, A, lda, B, ldb, C, ldc, bias, relu, mask, residual};
  a.drop_key = drop_key; a.drop_p = drop_p; a.mask_scale = mask_scale;
  a.splitk_ws = workspace;
  a.splitk_ws_bytes = workspace ? workspace_bytes : 0;
  launch_gemm((hipStream_t)stream, a);
  return op_done();
}

int tfm_op_wgrad_grouped(int32_t dtype, int32_t n, const int32_t* dims, const void* const* A, const void* const* B, void* const* C,
                         void* const* colsum, void* stream) {
  if ((dtype != TFM_FP16 && dtype != TFM_BF16) || n < 0 || n > WGRAD_GROUP_MAX || (n && (!dims || !A || !B || !C))) return TFM_EINVAL;
  WgradJob jobs[WGRAD_GROUP_MAX];
  for (int i = 0; i < n; ++i) {
    const int32_t* q = dims + 6 * i;
    WgradJob& j = jobs[i];
    j.M = q[0]; j.N = q[1]; j.K = q[2]; j.lda = q[3]; j.ldb = q[4]; j.ldc = q[5];
    j.A = A[i]; j.B = B[i]; j.C = C[i]; j.colsum = colsum ? colsum[i] : nullptr;
    if (j.M <= 0 || j.N <= 0 || j.K <= 0 || !j.A || !j.B || !j.C || j.lda < j.M || j.ldb < j.N || j.ldc < j.N) return TFM_EINVAL;
    if (!wgrad_group_supported(dtype, j)) return TFM_EINVAL;
  }
  launch_wgrad_grouped((hipStream_t)stream, dtype, jobs, n);
  return op_done();
}

int tfm_op_attention_fwd(int32_t dtype, const void* q, int32_t ldq, const void* k, int32_t ldk, const void* v, int32_t ldv,
                         void* o, int32_t ldo, float* lse, const int32_t* q_off, const int32_t* k_off, int32_t B, int32_t H,
                         int32_t dh, int32_t max_lq, int32_t max_lk, int32_t total_q, int32_t causal, uint64_t drop_key, float drop_p,
                         const int32_t* groups, int32_t n_groups, void* stream) {
  if (dtype < 0 || dtype > 2 || !q || !k || !v || !o || !lse || !q_off || !k_off || B < 1 || H < 1 || dh < 1 || dh > 128) return TFM_EINVAL;
  if (max_lq < 1 || max_lk < 1 || max_lq > 4096 || max_lk > 4096 || !(drop_p >= 0.f && drop_p < 1.f)) return TFM_EINVAL;
  if (n_groups < 0 || n_groups > B || (groups == nullptr) != (n_groups == 0)) return TFM_EINVAL;
  AttnArgs a{};
  a.dt = dtype; a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldk = ldk; a.ldv = ldv; a.o = o; a.ldo = ldo; a.lse = lse;
  a.q_off = q_off; a.k_off = k_off; a.B = B; a.H = H; a.dh = dh; a.max_lq = max_lq; a.max_lk = max_lk; a.total_q = total_q;
  a.causal = causal; a.drop_key = drop_key; a.drop_p = drop_p; a.groups = groups; a.n_groups = n_groups;
  launch_attention_fwd((hipStream_t)stream, a);
  return op_done();
}

int tfm_op_attention_bwd(int32_t dtype, const void* q, int32_t ldq, const void* k, int32_t ldk, const void* v, int32_t ldv,
                         const void* o, int32_t ldo, const void* d_o, int32_t lddo, const float* lse, void* dq, int32_t lddq,
                         void* dk, int32_t lddk, void* dv, int32_t lddv, const int32_t* q_off, const int32_t* k_off, int32_t B,
                         int32_t H, int32_t dh, int32_t max_lq, int32_t max_lk, int32_t total_q, int32_t total_k, int32_t causal,
                         uint64_t drop_key, float drop_p, const int32_t* groups, int32_t n_groups, void* stream) {
  if (dtype < 0 || dtype > 2 || !q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !q_off || !k_off) return TFM_EINVAL;
  if (B < 1 || H < 1 || dh < 1 || dh > 128 || max_lq < 1 || max_lk < 1 || max_lq > 4096 || max_lk > 4096) return TFM_EINVAL;
  if (!(drop_p >= 0.f && drop_p < 1.f)) return TFM_EINVAL;
  if (n_groups < 0 || n_groups > B || (groups == nullptr) != (n_groups == 0)) return TFM_EINVAL;
  AttnArgs a{};
  a.dt = dtype; a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldk = ldk; a.ldv = ldv; a.o = const_cast<void*>(o); a.ldo = ldo;
  a.lse = const_cast<float*>(lse); a.q_off = q_off; a.k_off = k_off; a.B = B; a.H = H; a.dh = dh; a.max_lq = max_lq;
  a.max_lk = max_lk; a.total_q = total_q; a.total_k = total_k; a.causal = causal; a.d_o = d_o; a.lddo = lddo; a.dq = dq;
  a.dk = dk; a.dv = dv; a.lddq = lddq; a.lddk = lddk; a.lddv = lddv; a.drop_key = drop_key; a.drop_p = drop_p;
  a.groups = groups; a.n_groups = n_groups;
  launch_attention_bwd((hipStream_t)stream, a);
  return op_done();
}

int tfm_op_residual_layernorm_fwd(int32_t dtype, const void* x, const void* y, const void* gamma, const void* beta, void* s_out,
                                  void* n_out, float* mean, float* rstd, int32_t rows, int32_t d, uint64_t drop_key, float p,
                                  void* stream) {
  if (dtype < 0 || dtype > 2 || !x || !gamma || !beta || !n_out || !mean || !rstd || rows < 0 || d < 8 || d % 8 || d > 2048) return TFM_EINVAL;
  launch_residual_layernorm_fwd((hipStream_t)stream, dtype, x, y, gamma, beta, s_out, n_out, mean, rstd, rows, d, drop_key, p);
  return op_done();
}

size_t tfm_op_layernorm_bwd_scratch(int32_t rows, int32_t d) { return layernorm_bwd_scratch_bytes(rows, d); }

int tfm_op_layernorm_bwd(int32_t dtype, const void* dn, const void* add, const void* s, const float* mean, const float* rstd,
                         const void* gamma, void* ds, void* ds_drop, void* dgamma, void* dbeta, void* dbias, int32_t rows,
                         int32_t d, uint64_t drop_key, float p, void* scratch, void* stream) {
  if (dtype < 0 || dtype > 2 || !dn || !s || !mean || !rstd || !gamma || !ds || !dgamma || !dbeta || !scratch) return TFM_EINVAL;
  if (rows < 1 || d < 8 || d % 8 || d > 2048) return TFM_EINVAL;
  launch_layernorm_bwd((hipStream_t)stream, dtype, dn, add, s, mean, rstd, gamma, ds, ds_drop, dgamma, dbeta, dbias, rows, d,
                       drop_key, p, scratch);
  return op_done();
}

int tfm_op_loss(int32_t dtype, void* z, const int32_t* labels, float* loss_rows, float* nll_rows, int32_t rows, int32_t V,
                float eps, float scale, void* stream) {
  if (dtype < 0 || dtype > 2 || !z || !labels || !loss_rows || !nll_rows || rows < 0 || V < 1) return TFM_EINVAL;
  launch_loss((hipStream_t)stream, dtype, z, labels, loss_rows, nll_rows, rows, V, eps, nullptr, scale, nullptr);
  return op_done();
}

int tfm_op_adam(float* w, float* m, float* v, const void* g, int32_t gdtype, void* half_copy, int32_t hdtype, int64_t n,
                float lr, float beta1, float beta2, float eps, float weight_decay, float grad_mult, float bc1, float bc2,
                void* stream) {
  if (!w || !m || !v || !g || gdtype < 0 || gdtype > 2 || hdtype < 0 || hdtype > 2 || n < 0 || n % 8) return TFM_EINVAL;
  AdamArgs a{w, m, v, g, gdtype, half_copy, hdtype, n, lr, beta1, beta2, eps, weight_decay, nullptr, grad_mult, bc1, bc2};
  launch_adam((hipStream_t)stream, a);
  return op_done();
}

size_t tfm_op_scan_scratch(int64_t n) { return scan_scratch_bytes(n); }

int tfm_op_scan(int32_t dtype, const void* x, int64_t n, float* result, void* scratch, void* stream) {
  if (dtype < 0 || dtype > 2 || !x || !result || !scratch || n < 0 || n % 8) return TFM_EINVAL;
  launch_scan((hipStream_t)stream, dtype, x, n, result, nullptr, nullptr, 0, scratch);
  return op_done();
}

int tfm_op_dropout_mask(uint64_t key, float p, uint8_t* out, int64_t n, void* stream) {
  if (!out || n < 0 || !(p >= 0.f && p < 1.f)) return TFM_EINVAL;
  launch_dropout_mask((hipStream_t)stream, key, p, out, n);
  return op_done();
}

uint64_t tfm_dropout_key(uint64_t seed, uint64_t step, int32_t stream, int32_t layer, int32_t sub) {
  return dropout_site_key(seed, step, stream, layer, sub);
}

}  // extern "C"
