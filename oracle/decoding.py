"""Oracle for step-wise prediction during inference.  TEST INFRASTRUCTURE ONLY (numpy float64).

Implementation, Inference describes a cache: what earlier positions contributed is kept per hypothesis, and a step
only computes the newest position.  Caching changes the cost, not the result: the
distribution over the next token given a source sentence and the tokens generated so far is, by definition, what
the full decoder computes at its last position when it is run over the whole prefix.  The oracle is that definition:
it recomputes the whole prefix at every step, without dropout, and keeps no cache.  It shares no code with the HIP
path; the parameters and sub-layers are those of oracle/transformer.py.

  DecodingOracle.encode(src)                    encoder output for one source sentence (None for a decoder-only model)
  DecodingOracle.logprobs(mem, dec_in)          log-softmax over the vocabulary at every position of dec_in
  DecodingOracle.next_logprobs(mem, history)    the last row of the above: the step's prediction
  DecodingOracle.vocabulary_logprobs(y)         final states -> log-probabilities of every token; for a model with an
                                                adaptive softmax (Applications, language modeling) a head token has
                                                log p_head(w), a token of tail cluster c has log p_head(entry of c) +
                                                log p_c(w), the definition the training criterion uses per target
  top_k(logp, k)                                the k best (log-probability, id) pairs, best first; equal values in
                                                ascending id order (the rule the library documents)
"""
import dataclasses

import numpy as np

from .transformer import OracleTransformer, TrainConfig, layer_norm_fwd


class DecodingOracle:
    def __init__(self, shape, params):
        self.shape = shape
        self.model = OracleTransformer(shape, params, dataclasses.replace(TrainConfig(), dropout=0.0))

    def encode(self, src):
        m, sh, P = self.model, self.shape, self.model.p
        if not sh.enc_layers:
            return None
        m._step = 0
        x, _ = m._embed_fwd(np.asarray(src, dtype=np.int64), 0, 0)
        for i in range(sh.enc_layers):
            pre = f"enc.{i}"
            x, _ = m._block_fwd(pre + ".ln_self", x, lambda u, pre=pre: m._self_attn_fwd(pre + ".self", u, False), (0, i, 0, 0))
            x, _ = m._block_fwd(pre + ".ln_ffn", x, lambda u, pre=pre: m._ffn_fwd(pre + ".ffn", u), (0, i, 2, 0))
        if sh.pre_norm:
            x, _ = layer_norm_fwd(x, P["enc.ln_final.g"], P["enc.ln_final.b"])
        return x

    def logprobs(self, mem, dec_in):
        m, sh, P = self.model, self.shape, self.model.p
        m._step = 0
        y, _ = m._embed_fwd(np.asarray(dec_in, dtype=np.int64), 1, 0)
        for i in range(sh.dec_layers):
            pre = f"dec.{i}"
            y, _ = m._block_fwd(pre + ".ln_self", y, lambda u, pre=pre: m._self_attn_fwd(pre + ".self", u, True), (1, i, 0, 0))
            if sh.enc_layers:
                y, _ = m._block_fwd(pre + ".ln_cross", y, lambda u, pre=pre: m._cross_attn_fwd(pre + ".cross", u, mem), (1, i, 1, 0))
            y, _ = m._block_fwd(pre + ".ln_ffn", y, lambda u, pre=pre: m._ffn_fwd(pre + ".ffn", u), (1, i, 2, 0))
        if sh.pre_norm:
            y, _ = layer_norm_fwd(y, P["dec.ln_final.g"], P["dec.ln_final.b"])
        return self.vocabulary_logprobs(y)

    def vocabulary_logprobs(self, y):
        sh, P = self.shape, self.model.p
        head = _log_softmax(y @ P["embed"].T)
        if not sh.cutoffs:
            return head
        bounds = sh.cluster_bounds()
        c0 = bounds[0][1]
        out = np.empty((y.shape[0], sh.vocab))
        out[:, :c0] = head[:, :c0]                                # the head's own tokens
        for c in range(1, len(bounds)):
            lo, hi = bounds[c]
            u = y @ P[f"embed.{c}.proj"]                          # state projected down to the cluster's width
            out[:, lo:hi] = head[:, c0 + c - 1:c0 + c] + _log_softmax(u @ P[f"embed.{c}"].T)
        return out

    def next_logprobs(self, mem, history):
        """history: the tokens fed to the decoder so far (the first one is eos)."""
        return self.logprobs(mem, history)[-1]


def _log_softmax(z):
    z = z - z.max(axis=1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=1, keepdims=True))


def top_k(logp, k):
    order = sorted(range(len(logp)), key=lambda i: (-logp[i], i))[:k]
    return [(float(logp[i]), int(i)) for i in order]
