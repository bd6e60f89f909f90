"""Model shapes and the canonical parameter list (names and shapes only).

The model family is the Transformer encoder-decoder and the decoder-only Transformer language model the
paper evaluates (Applications: machine translation; language modeling).  Sizes follow the benchmark
configurations: "tiny", "base", "big" and the 16-block language model with inner dimension 4K and
embedding dimension 1K.

Every linear layer is stored as W[out, in] and computes y = x W^T + b.  The query/key/value projections
of self-attention are one fused matrix `wqkv` whose row blocks are (Wq; Wk; Wv); cross-attention keeps
`wq` for the decoder side and a fused `wkv` = (Wk; Wv) for the encoder side.  There is one shared
embedding table `embed` [V, d]; the output projection is tied to it and has no bias.

With `cutoffs` (language model only) the vocabulary, sorted by frequency, is cut into a head [0, c_0) and tail
clusters [c_{i-1}, c_i), the last one ending at V (adaptive input embeddings and adaptive softmax, Applications:
language modeling).  Tail cluster i = 1, 2, ... has its own table `embed.i` [V_i, d / factor^i] and a projection
`embed.i.proj` [d, d / factor^i]; both are shared between the input and the output side.  `embed` then has
c_0 + (number of tail clusters) rows: the head's tokens followed by one output row per tail cluster.
"""
from dataclasses import dataclass, asdict


@dataclass(frozen=True)
class ModelShape:
    enc_layers: int
    dec_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    vocab: int
    pad_id: int = 1
    eos_id: int = 2
    pre_norm: int = 0      # 0: LayerNorm after each residual sum; 1: before each sub-layer plus a final one
    cutoffs: tuple = ()    # adaptive input/softmax: ascending ends of the head and of every tail cluster but the last
    factor: int = 4        # width of tail cluster i is d_model / factor^i

    def cluster_bounds(self):
        """[(lo, hi)] of the head and the tail clusters; a single (0, vocab) without cutoffs."""
        edges = [0, *self.cutoffs, self.vocab]
        return [(edges[i], edges[i + 1]) for i in range(len(edges) - 1)]

    def cluster_width(self, i):
        return self.d_model // self.factor ** i

    def asdict(self):
        return asdict(self)


PRESETS = {
    "tiny": ModelShape(1, 1, 64, 4, 256, 1000),
    "base": ModelShape(6, 6, 512, 8, 2048, 32768),
    "big": ModelShape(6, 6, 1024, 16, 4096, 32768),
    "lm16": ModelShape(0, 16, 1024, 16, 4096, 32768, pre_norm=1),
    # the larger language model: 24 blocks, inner dimension 8K, embedding dimension 1.5K (24 heads of width 64)
    "lm24": ModelShape(0, 24, 1536, 24, 8192, 32768, pre_norm=1),
    # The same network with adaptive inputs / adaptive softmax over a WikiText-103-sized vocabulary (267.7 K types, cut
    # near 20 K and 60 K).  The cuts are placed so that every table has a multiple of 8 rows (19998 head tokens + 2
    # cluster entries, 40000, 207744): the matrix-core GEMMs then serve all of them.
    "lm16a": ModelShape(0, 16, 1024, 16, 4096, 267742, pre_norm=1, cutoffs=(19998, 59998)),
}


def _attn_self(prefix, d):
    return [(prefix + ".wqkv", (3 * d, d)), (prefix + ".bqkv", (3 * d,)),
            (prefix + ".wo", (d, d)), (prefix + ".bo", (d,))]


def _attn_cross(prefix, d):
    return [(prefix + ".wq", (d, d)), (prefix + ".bq", (d,)),
            (prefix + ".wkv", (2 * d, d)), (prefix + ".bkv", (2 * d,)),
            (prefix + ".wo", (d, d)), (prefix + ".bo", (d,))]


def _ln(prefix, d):
    return [(prefix + ".g", (d,)), (prefix + ".b", (d,))]


def _ffn(prefix, d, f):
    return [(prefix + ".w1", (f, d)), (prefix + ".b1", (f,)),
            (prefix + ".w2", (d, f)), (prefix + ".b2", (d,))]


def param_specs(shape: ModelShape):
    """Canonical ordered list of (name, shape) for every learnable tensor."""
    d, f = shape.d_model, shape.d_ffn
    if shape.cutoffs:
        bounds = shape.cluster_bounds()
        out = [("embed", (bounds[0][1] + len(bounds) - 1, d))]
        for i in range(1, len(bounds)):
            di = shape.cluster_width(i)
            out += [(f"embed.{i}", (bounds[i][1] - bounds[i][0], di)), (f"embed.{i}.proj", (d, di))]
    else:
        out = [("embed", (shape.vocab, d))]
    for i in range(shape.enc_layers):
        p = f"enc.{i}"
        out += _attn_self(p + ".self", d) + _ln(p + ".ln_self", d)
        out += _ffn(p + ".ffn", d, f) + _ln(p + ".ln_ffn", d)
    if shape.enc_layers and shape.pre_norm:
        out += _ln("enc.ln_final", d)
    for i in range(shape.dec_layers):
        p = f"dec.{i}"
        out += _attn_self(p + ".self", d) + _ln(p + ".ln_self", d)
        if shape.enc_layers:
            out += _attn_cross(p + ".cross", d) + _ln(p + ".ln_cross", d)
        out += _ffn(p + ".ffn", d, f) + _ln(p + ".ln_ffn", d)
    if shape.pre_norm:
        out += _ln("dec.ln_final", d)
    return out


def count_params(shape: ModelShape) -> int:
    n = 0
    for _, s in param_specs(shape):
        k = 1
        for v in s:
            k *= v
        n += k
    return n
