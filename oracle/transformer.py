"""CPU oracle for the mixed-precision Transformer training step.  TEST INFRASTRUCTURE ONLY.

This file is the plain, slow, obviously-correct definition that the HIP path is checked against.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import it; the product never does.  It
shares no code with the HIP path.

What it computes (numpy, float64, one sentence at a time, no padding, explicit backward formulas):

* the Transformer encoder-decoder / decoder-only forward pass of the model family the paper trains
  (Applications: machine translation, language modeling), with the sizes given by a synth.ModelShape;
* criterion: loss = criterion(model, batch) (Design, Criterions) as label-smoothed cross-entropy summed
  over the non-pad target tokens, in nats;
* mixed-precision data flow (Implementation, Mixed precision): the loss is multiplied by the loss scale
  right after the forward pass, the backward pass is unchanged, gradients are unscaled before the update and
  the update is carried out in full precision; dynamic loss scaling halves the scale and skips the update on
  overflow and doubles it after `scale_window` clean updates;
* delayed updates (Implementation, Multi-GPU training): gradients of several sub-batches are summed before
  one optimiser step;
* optimiser: Adam with bias correction.

Readings where the paper is silent are listed in the repository's design notes; each one is a named
argument or a commented line below.

Pins (tests, CPU only): central finite differences of the whole model; an independent autograd model built
from torch.nn.functional primitives; closed forms of the loss; softmax/LayerNorm invariants; torch.optim.Adam;
a hand-computed loss-scale schedule; brute-force attention.  No function here is "parity unpinned".
"""
from dataclasses import dataclass, field

import numpy as np

LN_EPS = 1e-5
FP16_MAX = 65504.0
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


# ----------------------------------------------------------------------------------------------------------------
# dropout: counter-based keep bits (the HIP path implements the same generator on its own)
# ----------------------------------------------------------------------------------------------------------------
def _mix64(z):
    """Finaliser of the splitmix64 generator on uint64 arrays (wrapping arithmetic)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def dropout_key(seed, step, site):
    """64-bit key of one dropout site at one training step."""
    with np.errstate(over="ignore"):
        k = _mix64(np.uint64(seed) + np.uint64(0x9E3779B97F4A7C15))
        k = _mix64(k ^ (np.uint64(step) * np.uint64(0xD1B54A32D192ED03)))
        k = _mix64(k ^ (np.uint64(site) * np.uint64(0x8CB92BA72F3D8DD7)))
    return np.uint64(k)


def dropout_threshold(p):
    return int(np.floor(p * 65536.0))


def dropout_keep(key, row0, nrows, width, p):
    """Boolean keep mask [nrows, width] for rows row0.. of a [*, width] activation.

    Element e = row * width + col.  One 64-bit word serves four consecutive elements: word
    w = mix64(key + (e >> 2) * 0x9E3779B97F4A7C15); the 16-bit field (e & 3) of w is compared with
    floor(p * 65536): keep iff field >= threshold.
    """
    rows = np.arange(row0, row0 + nrows, dtype=np.uint64)[:, None]
    cols = np.arange(width, dtype=np.uint64)[None, :]
    e = rows * np.uint64(width) + cols
    with np.errstate(over="ignore"):
        w = _mix64(np.uint64(key) + (e >> np.uint64(2)) * np.uint64(0x9E3779B97F4A7C15))
    f = (w >> ((e & np.uint64(3)) * np.uint64(16))) & np.uint64(0xFFFF)
    return f >= np.uint64(dropout_threshold(p))


def site_id(stream, layer, sub):
    """Dropout site number.  stream: 0 encoder, 1 decoder.  layer: -1 for the embedding, else the layer index.
    sub: 0 self-attention output, 1 cross-attention output, 2 feed-forward output, 3 self-attention weights,
    4 cross-attention weights, 5 feed-forward hidden activations (after the ReLU)."""
    return 1000 * stream + 10 * (layer + 1) + sub


def attention_keep(key, qrow0, n, n_heads, h, m, p):
    """Boolean keep mask [n, m] for the attention weights of head h: queries are the packed rows qrow0.. of their
    stream, keys j = 0..m-1 of the same sentence (m < 65536).

    Element e = ((query row * n_heads + h) << 16) + j, then as in dropout_keep: one 64-bit word serves four
    consecutive keys of one (query, head).
    """
    rows = np.arange(qrow0, qrow0 + n, dtype=np.uint64)[:, None]
    cols = np.arange(m, dtype=np.uint64)[None, :]
    e = ((rows * np.uint64(n_heads) + np.uint64(h)) << np.uint64(16)) + cols
    with np.errstate(over="ignore"):
        w = _mix64(np.uint64(key) + (e >> np.uint64(2)) * np.uint64(0x9E3779B97F4A7C15))
    f = (w >> ((e & np.uint64(3)) * np.uint64(16))) & np.uint64(0xFFFF)
    return f >= np.uint64(dropout_threshold(p))


# ----------------------------------------------------------------------------------------------------------------
# building blocks: forward returns (output, cache); backward takes the cache
# ----------------------------------------------------------------------------------------------------------------
def positional_encoding(n, d):
    """PE(t, 2i) = sin(t / 10000^(2i/d)), PE(t, 2i+1) = cos(t / 10000^(2i/d)), t = 0..n-1."""
    t = np.arange(n, dtype=np.float64)[:, None]
    i = np.arange(d // 2, dtype=np.float64)[None, :]
    ang = t / np.power(10000.0, 2.0 * i / d)
    pe = np.zeros((n, d))
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)
    return pe


def layer_norm_fwd(x, g, b):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)          # biased variance over the features
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = (x - mu) * rstd
    return g * xhat + b, (xhat, rstd, g)


def layer_norm_bwd(dy, cache):
    xhat, rstd, g = cache
    dxhat = dy * g
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention_fwd(q, k, v, n_heads, causal, keep=None, p_drop=0.0):
    """softmax(q k^T / sqrt(d_h) [+ causal mask]) v per head; q [n,d], k,v [m,d].

    keep (optional): per head a boolean [n, m]; the attention weights are then multiplied by keep / (1 - p_drop)
    (inverted dropout on the weights) before they average the values.
    """
    n, d = q.shape
    dh = d // n_heads
    ctx = np.zeros((n, d))
    probs = []
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = q[:, sl] @ k[:, sl].T / np.sqrt(dh)
        if causal:
            s = np.where(np.arange(k.shape[0])[None, :] <= np.arange(n)[:, None], s, -np.inf)
        p = softmax_rows(s)
        probs.append(p)
        pd = p if keep is None else np.where(keep[h], p / (1.0 - p_drop), 0.0)
        ctx[:, sl] = pd @ v[:, sl]
    return ctx, (q, k, v, probs, n_heads, keep, p_drop)


def attention_bwd(dctx, cache):
    q, k, v, probs, n_heads, keep, p_drop = cache
    d = q.shape[1]
    dh = d // n_heads
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        p = probs[h]
        pd = p if keep is None else np.where(keep[h], p / (1.0 - p_drop), 0.0)
        dv[:, sl] = pd.T @ dctx[:, sl]
        dp = dctx[:, sl] @ v[:, sl].T                            # gradient w.r.t. the dropped weights ...
        if keep is not None:
            dp = np.where(keep[h], dp / (1.0 - p_drop), 0.0)     # ... and w.r.t. the softmax output
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
        dq[:, sl] = ds @ k[:, sl] / np.sqrt(dh)
        dk[:, sl] = ds.T @ q[:, sl] / np.sqrt(dh)
    return dq, dk, dv


def label_smoothed_nll(z, y, eps):
    """Per-row loss and d(loss)/dz for logits z [n, V] and targets y [n].

    nll_t = lse - z[y_t]; smooth_t = lse - mean_i z_i; loss_t = (1-eps) nll_t + eps smooth_t, i.e. the
    cross-entropy against q = (1-eps) onehot(y) + eps/V.  dz = softmax(z) - q.
    """
    n, V = z.shape
    m = z.max(axis=-1, keepdims=True)
    lse = (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))[:, 0]
    nll = lse - z[np.arange(n), y]
    smooth = lse - z.mean(axis=-1)
    loss = (1.0 - eps) * nll + eps * smooth
    dz = np.exp(z - lse[:, None])
    dz -= eps / V
    dz[np.arange(n), y] -= (1.0 - eps)
    return loss, nll, dz


# ----------------------------------------------------------------------------------------------------------------
# the model
# ----------------------------------------------------------------------------------------------------------------
@dataclass
class TrainConfig:
    dropout: float = 0.0            # on the embedding sums and on each sub-layer output before the residual sum
    attn_dropout: float = 0.0       # on the attention weights (after the softmax)
    relu_dropout: float = 0.0       # on the feed-forward hidden activations (after the ReLU)
    label_smoothing: float = 0.1
    adam_beta1: float = 0.9
    adam_beta2: float = 0.98
    adam_eps: float = 1e-8
    weight_decay: float = 0.0       # L2 form: weight_decay * w joins the (unscaled, clipped) gradient inside the Adam step
    clip_norm: float = 0.0
    init_loss_scale: float = 128.0
    scale_window: int = 2000
    min_loss_scale: float = 2.0 ** -14
    fp16_overflow: bool = False     # True: a scaled gradient value beyond the fp16 range counts as overflow
    dynamic_scale: bool = True      # False (bf16 reading): the scale stays fixed, overflow still skips
    seed: int = 0


class _Grads(dict):
    def add(self, name, value):
        if name in self:
            self[name] += value
        else:
            self[name] = np.array(value, dtype=np.float64)

    def add_rows(self, name, rows, value, nrows):
        if name not in self:
            self[name] = np.zeros((nrows, value.shape[1]))
        np.add.at(self[name], rows, value)              # repeated rows accumulate


class OracleTransformer:
    """State = parameters (float64), Adam moments, accumulated scaled gradients, scaler state."""

    def __init__(self, shape, params, cfg: TrainConfig):
        self.shape, self.cfg = shape, cfg
        self.p = {k: np.array(v, dtype=np.float64) for k, v in params.items()}
        self.m = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.v = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.G = {k: np.zeros_like(v) for k, v in self.p.items()}
        self.loss_scale = float(cfg.init_loss_scale)
        self.clean_steps = 0
        self.num_updates = 0
        self.train_steps = 0           # dropout step counter: number of train_step calls so far
        self.window_overflow = False
        self.window_ntokens = 0
        self.window_microbatches = 0

    # -- sub-layers -------------------------------------------------------------------------------------------
    def _drop(self, x, stream, layer, sub, row0):
        p = self.cfg.dropout
        if p <= 0.0:
            return x, None
        key = dropout_key(self.cfg.seed, self._step, site_id(stream, layer, sub))
        keep = dropout_keep(key, row0, x.shape[0], x.shape[1], p)
        return np.where(keep, x / (1.0 - p), 0.0), keep

    def _drop_bwd(self, dy, keep):
        if keep is None:
            return dy
        return np.where(keep, dy / (1.0 - self.cfg.dropout), 0.0)

    def _attn_keep(self, site, sub, n, m):
        """Keep masks of the attention weights, one per head, or None.  site = (stream, layer, first packed query row)."""
        p = self.cfg.attn_dropout
        if p <= 0.0:
            return None
        stream, layer, row0 = site
        key = dropout_key(self.cfg.seed, self._step, site_id(stream, layer, sub))
        H = self.shape.n_heads
        return [attention_keep(key, row0, n, H, h, m, p) for h in range(H)]

    def _self_attn_fwd(self, pre, x, causal, site=None):
        P, d = self.p, self.shape.d_model
        qkv = x @ P[pre + ".wqkv"].T + P[pre + ".bqkv"]
        keep = self._attn_keep(site, 3, x.shape[0], x.shape[0])
        ctx, ac = attention_fwd(qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:], self.shape.n_heads, causal, keep,
                                self.cfg.attn_dropout)
        y = ctx @ P[pre + ".wo"].T + P[pre + ".bo"]
        return y, (x, ctx, ac)

    def _self_attn_bwd(self, pre, dy, cache, g):
        P = self.p
        x, ctx, ac = cache
        g.add(pre + ".wo", dy.T @ ctx)
        g.add(pre + ".bo", dy.sum(axis=0))
        dq, dk, dv = attention_bwd(dy @ P[pre + ".wo"], ac)
        dqkv = np.concatenate([dq, dk, dv], axis=1)
        g.add(pre + ".wqkv", dqkv.T @ x)
        g.add(pre + ".bqkv", dqkv.sum(axis=0))
        return dqkv @ P[pre + ".wqkv"]

    def _cross_attn_fwd(self, pre, x, mem, site=None):
        P, d = self.p, self.shape.d_model
        q = x @ P[pre + ".wq"].T + P[pre + ".bq"]
        kv = mem @ P[pre + ".wkv"].T + P[pre + ".bkv"]
        keep = self._attn_keep(site, 4, x.shape[0], mem.shape[0])
        ctx, ac = attention_fwd(q, kv[:, :d], kv[:, d:], self.shape.n_heads, False, keep, self.cfg.attn_dropout)
        y = ctx @ P[pre + ".wo"].T + P[pre + ".bo"]
        return y, (x, mem, ctx, ac)

    def _cross_attn_bwd(self, pre, dy, cache, g):
        P = self.p
        x, mem, ctx, ac = cache
        g.add(pre + ".wo", dy.T @ ctx)
        g.add(pre + ".bo", dy.sum(axis=0))
        dq, dk, dv = attention_bwd(dy @ P[pre + ".wo"], ac)
        g.add(pre + ".wq", dq.T @ x)
        g.add(pre + ".bq", dq.sum(axis=0))
        dkv = np.concatenate([dk, dv], axis=1)
        g.add(pre + ".wkv", dkv.T @ mem)
        g.add(pre + ".bkv", dkv.sum(axis=0))
        return dq @ P[pre + ".wq"], dkv @ P[pre + ".wkv"]

    def _ffn_fwd(self, pre, x, site=None):
        P = self.p
        a = x @ P[pre + ".w1"].T + P[pre + ".b1"]
        h = np.maximum(a, 0.0)
        keep, pr = None, self.cfg.relu_dropout
        if pr > 0.0:                                             # inverted dropout on the hidden activations
            stream, layer, row0 = site
            key = dropout_key(self.cfg.seed, self._step, site_id(stream, layer, 5))
            keep = dropout_keep(key, row0, h.shape[0], h.shape[1], pr)
            h = np.where(keep, h / (1.0 - pr), 0.0)
        return h @ P[pre + ".w2"].T + P[pre + ".b2"], (x, a, h, keep)

    def _ffn_bwd(self, pre, dy, cache, g):
        P = self.p
        x, a, h, keep = cache
        g.add(pre + ".w2", dy.T @ h)
        g.add(pre + ".b2", dy.sum(axis=0))
        dh = dy @ P[pre + ".w2"]
        if keep is not None:
            dh = np.where(keep, dh / (1.0 - self.cfg.relu_dropout), 0.0)
        da = dh * (a > 0.0)
        g.add(pre + ".w1", da.T @ x)
        g.add(pre + ".b1", da.sum(axis=0))
        return da @ P[pre + ".w1"]

    # residual wrapper: post-norm  x <- LN(x + drop(f(x)));  pre-norm  x <- x + drop(f(LN(x)))
    def _block_fwd(self, ln, x, f, drop_args):
        P = self.p
        if self.shape.pre_norm:
            nx, lc = layer_norm_fwd(x, P[ln + ".g"], P[ln + ".b"])
            y, fc = f(nx)
            y, keep = self._drop(y, *drop_args)
            return x + y, (lc, fc, keep)
        y, fc = f(x)
        y, keep = self._drop(y, *drop_args)
        out, lc = layer_norm_fwd(x + y, P[ln + ".g"], P[ln + ".b"])
        return out, (lc, fc, keep)

    def _block_bwd(self, ln, dout, cache, fb, g):
        """fb(dy, fcache) -> gradient w.r.t. the sub-layer input (extra returns are passed through)."""
        lc, fc, keep = cache
        if self.shape.pre_norm:
            r = fb(self._drop_bwd(dout, keep), fc)
            dnx, extra = (r if isinstance(r, tuple) else (r, None))
            dx, dg, db = layer_norm_bwd(dnx, lc)
            g.add(ln + ".g", dg)
            g.add(ln + ".b", db)
            return dout + dx, extra
        ds, dg, db = layer_norm_bwd(dout, lc)
        g.add(ln + ".g", dg)
        g.add(ln + ".b", db)
        r = fb(self._drop_bwd(ds, keep), fc)
        dx, extra = (r if isinstance(r, tuple) else (r, None))
        return ds + dx, extra

    # -- one sentence ------------------------------------------------------------------------------------------
    def _embed_fwd(self, ids, stream, row0):
        d = self.shape.d_model
        x = np.sqrt(d) * self._lookup(ids) + positional_encoding(len(ids), d)
        return self._drop(x, stream, -1, 0, row0)

    def _embed_bwd(self, ids, dx, keep, g):
        dx = np.sqrt(self.shape.d_model) * self._drop_bwd(dx, keep)
        if not self.shape.cutoffs:
            g.add_rows("embed", ids, dx, self.shape.vocab)
            return
        P = self.p
        for c, (lo, hi) in enumerate(self.shape.cluster_bounds()):
            sel = (ids >= lo) & (ids < hi)
            if not sel.any():
                continue
            if c == 0:
                g.add_rows("embed", ids[sel], dx[sel], P["embed"].shape[0])
            else:
                rows = P[f"embed.{c}"][ids[sel] - lo]
                g.add(f"embed.{c}.proj", dx[sel].T @ rows)
                g.add_rows(f"embed.{c}", ids[sel] - lo, dx[sel] @ P[f"embed.{c}.proj"], hi - lo)

    # -- adaptive input embeddings / adaptive softmax (Applications, language modeling) ------------------------
    def _lookup(self, ids):
        """Token vectors before scaling: the head's rows as they are, a tail cluster's narrow rows through
        the cluster's projection up to the model width."""
        P = self.p
        if not self.shape.cutoffs:
            return P["embed"][ids]
        out = np.zeros((len(ids), self.shape.d_model))
        for c, (lo, hi) in enumerate(self.shape.cluster_bounds()):
            sel = (ids >= lo) & (ids < hi)
            if c == 0:
                out[sel] = P["embed"][ids[sel]]
            else:
                out[sel] = P[f"embed.{c}"][ids[sel] - lo] @ P[f"embed.{c}.proj"].T
        return out

    def _adaptive_nll(self, y, tgt, scale, g):
        """log p(w) = log p_head(w) for a head token, log p_head(cluster of w) + log p_cluster(w) otherwise; the
        head is a softmax over its tokens plus one entry per tail cluster, a tail cluster projects the state down
        to its width (transposed input projection) and scores its own tokens (its input table).  Returns
        (nll per token, d nll * scale / d y, max |d logits|) and adds the parameter gradients to g."""
        P = self.p
        bounds = self.shape.cluster_bounds()
        c0 = bounds[0][1]
        cluster = np.zeros(len(tgt), dtype=np.int64)
        for c, (lo, hi) in enumerate(bounds):
            cluster[(tgt >= lo) & (tgt < hi)] = c
        z = y @ P["embed"].T
        head_label = np.where(cluster == 0, tgt, c0 + cluster - 1)
        _, nll, dz = label_smoothed_nll(z, head_label, 0.0)
        dz *= scale
        dz_max = float(np.max(np.abs(dz))) if dz.size else 0.0
        g.add("embed", dz.T @ y)
        dy = dz @ P["embed"]
        for c in range(1, len(bounds)):
            sel = np.nonzero(cluster == c)[0]
            if len(sel) == 0:
                continue
            lo = bounds[c][0]
            E, Pc = P[f"embed.{c}"], P[f"embed.{c}.proj"]
            u = y[sel] @ Pc
            _, nll_c, dzc = label_smoothed_nll(u @ E.T, tgt[sel] - lo, 0.0)
            dzc *= scale
            dz_max = max(dz_max, float(np.max(np.abs(dzc))))
            nll[sel] += nll_c
            du = dzc @ E
            g.add(f"embed.{c}", dzc.T @ u)
            g.add(f"embed.{c}.proj", y[sel].T @ du)
            dy[sel] += du @ Pc.T
        return nll, dy, dz_max

    def _sentence(self, src, tgt, srow0, trow0, scale, g):
        """Forward + backward of scale * sum_t loss_t for one sentence.  Returns (loss_sum, nll_sum, max|dz|)."""
        sh, P = self.shape, self.p
        # teacher forcing: decoder input = eos followed by the target without its last token
        dec_in = np.concatenate([[sh.eos_id], tgt[:-1]]).astype(np.int64)
        caches = []
        mem = None
        if sh.enc_layers:
            x, ekeep = self._embed_fwd(src, 0, srow0)
            for i in range(sh.enc_layers):
                pre = f"enc.{i}"
                x, c1 = self._block_fwd(pre + ".ln_self", x,
                                        lambda u, pre=pre, i=i: self._self_attn_fwd(pre + ".self", u, False, (0, i, srow0)),
                                        (0, i, 0, srow0))
                x, c2 = self._block_fwd(pre + ".ln_ffn", x,
                                        lambda u, pre=pre, i=i: self._ffn_fwd(pre + ".ffn", u, (0, i, srow0)), (0, i, 2, srow0))
                caches.append((c1, c2))
            if sh.pre_norm:
                x, enc_lnf = layer_norm_fwd(x, P["enc.ln_final.g"], P["enc.ln_final.b"])
            mem = x
        y, dkeep = self._embed_fwd(dec_in, 1, trow0)
        dcaches = []
        for i in range(sh.dec_layers):
            pre = f"dec.{i}"
            y, c1 = self._block_fwd(pre + ".ln_self", y,
                                    lambda u, pre=pre, i=i: self._self_attn_fwd(pre + ".self", u, True, (1, i, trow0)),
                                    (1, i, 0, trow0))
            c2 = None
            if sh.enc_layers:
                y, c2 = self._block_fwd(pre + ".ln_cross", y,
                                        lambda u, pre=pre, i=i: self._cross_attn_fwd(pre + ".cross", u, mem, (1, i, trow0)),
                                        (1, i, 1, trow0))
            y, c3 = self._block_fwd(pre + ".ln_ffn", y,
                                    lambda u, pre=pre, i=i: self._ffn_fwd(pre + ".ffn", u, (1, i, trow0)), (1, i, 2, trow0))
            dcaches.append((c1, c2, c3))
        if sh.pre_norm:
            y, dec_lnf = layer_norm_fwd(y, P["dec.ln_final.g"], P["dec.ln_final.b"])
        if sh.cutoffs:
            assert self.cfg.label_smoothing == 0.0, "the adaptive softmax is trained on the plain likelihood"
            nll, dy, dz_max = self._adaptive_nll(y, np.asarray(tgt, dtype=np.int64), scale, g)
            loss = nll
        else:
            z = y @ P["embed"].T                                # tied output projection, no bias
            loss, nll, dz = label_smoothed_nll(z, tgt, self.cfg.label_smoothing)
            dz *= scale                                         # the loss is scaled right after the forward pass
            dz_max = float(np.max(np.abs(dz))) if dz.size else 0.0
            # ---- backward
            g.add("embed", dz.T @ y)
            dy = dz @ P["embed"]
        if sh.pre_norm:
            dy, dg, db = layer_norm_bwd(dy, dec_lnf)
            g.add("dec.ln_final.g", dg)
            g.add("dec.ln_final.b", db)
        dmem = np.zeros_like(mem) if mem is not None else None
        for i in reversed(range(sh.dec_layers)):
            pre = f"dec.{i}"
            c1, c2, c3 = dcaches[i]
            dy, _ = self._block_bwd(pre + ".ln_ffn", dy, c3,
                                    lambda d_, fc, pre=pre: self._ffn_bwd(pre + ".ffn", d_, fc, g), g)
            if sh.enc_layers:
                dy, dm = self._block_bwd(pre + ".ln_cross", dy, c2,
                                         lambda d_, fc, pre=pre: self._cross_attn_bwd(pre + ".cross", d_, fc, g), g)
                dmem += dm
            dy, _ = self._block_bwd(pre + ".ln_self", dy, c1,
                                    lambda d_, fc, pre=pre: self._self_attn_bwd(pre + ".self", d_, fc, g), g)
        self._embed_bwd(dec_in, dy, dkeep, g)
        if sh.enc_layers:
            dx = dmem
            if sh.pre_norm:
                dx, dg, db = layer_norm_bwd(dx, enc_lnf)
                g.add("enc.ln_final.g", dg)
                g.add("enc.ln_final.b", db)
            for i in reversed(range(sh.enc_layers)):
                pre = f"enc.{i}"
                c1, c2 = caches[i]
                dx, _ = self._block_bwd(pre + ".ln_ffn", dx, c2,
                                        lambda d_, fc, pre=pre: self._ffn_bwd(pre + ".ffn", d_, fc, g), g)
                dx, _ = self._block_bwd(pre + ".ln_self", dx, c1,
                                        lambda d_, fc, pre=pre: self._self_attn_bwd(pre + ".self", d_, fc, g), g)
            self._embed_bwd(np.asarray(src, dtype=np.int64), dx, ekeep, g)
        return float(loss.sum()), float(nll.sum()), dz_max

    # -- public API (mirrors the C boundary) -------------------------------------------------------------------
    def forward_loss(self, src, tgt, src_lens, tgt_lens, step=None):
        """Loss only (used by the finite-difference pin) at dropout step `step`; leaves the state unchanged."""
        saveG, savew = self.G, (self.window_overflow, self.window_ntokens, self.window_microbatches)
        self.G = {k: np.zeros_like(v) for k, v in self.p.items()}
        keep_step = self.train_steps
        if step is not None:
            self.train_steps = step
        out = self.train_step(src, tgt, src_lens, tgt_lens)
        self.G = saveG
        self.window_overflow, self.window_ntokens, self.window_microbatches = savew
        self.train_steps = keep_step
        return out["loss_sum"]

    def train_step(self, src, tgt, src_lens, tgt_lens, loss_mult=1.0):
        """One sub-batch: G += d(S * mult * sum loss)/d(params).  Padded [B, L] arrays plus lengths, as at the
        C boundary; padding is stripped here because a pad position does not exist semantically."""
        sh = self.shape
        self._step = self.train_steps
        scale = self.loss_scale * loss_mult
        g = _Grads()
        loss_sum = nll_sum = 0.0
        dz_max = 0.0
        srow = trow = 0
        B = len(tgt_lens)
        for b in range(B):
            n = int(tgt_lens[b])
            t = np.asarray(tgt[b, :n], dtype=np.int64)
            if sh.enc_layers:
                m = int(src_lens[b])
                s = np.asarray(src[b, :m], dtype=np.int64)
            else:
                m, s = 0, None
            ls, ns, zm = self._sentence(s, t, srow, trow, scale, g)
            loss_sum += ls
            nll_sum += ns
            dz_max = max(dz_max, zm) if np.isfinite(zm) else np.inf
            srow += m
            trow += n
        overflow = not np.isfinite(dz_max)
        gmax = 0.0
        for k, v in g.items():
            if not np.all(np.isfinite(v)):
                overflow = True
            else:
                gmax = max(gmax, float(np.max(np.abs(v))) if v.size else 0.0)
        if self.cfg.fp16_overflow and (dz_max > FP16_MAX or gmax > FP16_MAX):
            overflow = True
        with np.errstate(invalid="ignore", over="ignore"):
            for k, v in g.items():
                self.G[k] += v
        self.train_steps += 1
        self.window_overflow |= overflow
        self.window_ntokens += int(np.sum(tgt_lens))
        self.window_microbatches += 1
        return dict(loss_sum=loss_sum, nll_sum=nll_sum, ntokens=int(np.sum(tgt_lens)), overflow=int(overflow),
                    loss_scale=self.loss_scale)

    def unscaled_grads(self):
        """G / (S * N): the per-token gradient the optimiser sees."""
        c = 1.0 / (self.loss_scale * max(self.window_ntokens, 1))
        return {k: v * c for k, v in self.G.items()}

    def apply_update(self, lr):
        cfg = self.cfg
        assert self.window_microbatches > 0
        skipped = bool(self.window_overflow)
        grad_norm = float("nan")
        if skipped:
            # overflow: drop the accumulated gradients, halve the scale, leave parameters and moments alone
            if cfg.dynamic_scale:
                self.loss_scale /= 2.0
            self.clean_steps = 0
        else:
            gr = self.unscaled_grads()
            grad_norm = float(np.sqrt(sum(float((v * v).sum()) for v in gr.values())))
            coef = 1.0
            if cfg.clip_norm > 0.0 and grad_norm > cfg.clip_norm:
                coef = cfg.clip_norm / grad_norm
            self.num_updates += 1
            t = self.num_updates
            b1, b2 = cfg.adam_beta1, cfg.adam_beta2
            for k in self.p:
                gk = gr[k] * coef + cfg.weight_decay * self.p[k]
                self.m[k] = b1 * self.m[k] + (1.0 - b1) * gk
                self.v[k] = b2 * self.v[k] + (1.0 - b2) * gk * gk
                mhat = self.m[k] / (1.0 - b1 ** t)
                vhat = self.v[k] / (1.0 - b2 ** t)
                self.p[k] = self.p[k] - lr * mhat / (np.sqrt(vhat) + cfg.adam_eps)
            self.clean_steps += 1
            if cfg.dynamic_scale and self.clean_steps == cfg.scale_window:
                self.loss_scale *= 2.0
                self.clean_steps = 0
        ntok = self.window_ntokens
        for v in self.G.values():
            v[...] = 0.0
        self.window_overflow = False
        self.window_ntokens = 0
        self.window_microbatches = 0
        return dict(skipped=int(skipped), loss_scale_after=self.loss_scale, clean_steps=self.clean_steps,
                    num_updates=self.num_updates, grad_norm=grad_norm, ntokens_total=ntok,
                    scale_too_small=bool(self.loss_scale < cfg.min_loss_scale))
