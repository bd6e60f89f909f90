"""Seeded synthetic batches with the shapes of the paper's workloads.

The paper trains on WMT'16 En-De / WMT'14 En-Fr with a joint 32K/40K BPE vocabulary (Applications, machine
translation) and on WikiText-103 blocks (language modeling), and builds token-capped batches of sentences
of similar length (Implementation, batching).  None of those corpora is used here: only their shapes are.
Token ids follow a bounded Zipf law, sentence lengths are uniform in a range, sentences are sorted by
length and packed greedily under a cap on the padded token count.
"""
from dataclasses import dataclass

import numpy as np

from .shapes import ModelShape, PRESETS

N_SPECIAL = 4      # ids 0..3: bos, pad(1), eos(2), unk


@dataclass
class Batch:
    src: np.ndarray        # int32 [B, Ls], right padded with pad_id; None for the language model
    tgt: np.ndarray        # int32 [B, Lt], right padded with pad_id; every row ends with eos (translation)
    src_lens: np.ndarray   # int32 [B]; None for the language model
    tgt_lens: np.ndarray   # int32 [B]

    @property
    def ntokens(self):
        return int(self.tgt_lens.sum())


def zipf_ids(rng, n, vocab, exponent=1.1):
    """n content ids in [N_SPECIAL, vocab): id = N_SPECIAL - 1 + rank, P(rank) ~ rank^-exponent."""
    ranks = np.arange(1, vocab - N_SPECIAL + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** -exponent)
    cdf /= cdf[-1]
    r = np.searchsorted(cdf, rng.random(n), side="left")
    return (N_SPECIAL + np.minimum(r, vocab - N_SPECIAL - 1)).astype(np.int32)


def _pad(rows, pad_id):
    L = max(len(r) for r in rows)
    out = np.full((len(rows), L), pad_id, dtype=np.int32)
    for i, r in enumerate(rows):
        out[i, :len(r)] = r
    return out


def _translation_pool(rng, shape, n_sent, lo, hi, uniform_ids):
    src_len = rng.integers(lo, hi + 1, size=n_sent)
    tgt_len = np.clip(src_len + rng.integers(-3, 4, size=n_sent), lo, hi)
    draw = (lambda n: rng.integers(N_SPECIAL, shape.vocab, size=n).astype(np.int32)) if uniform_ids \
        else (lambda n: zipf_ids(rng, n, shape.vocab))
    sents = []
    for m, n in zip(src_len, tgt_len):
        s = np.concatenate([draw(m - 1), [shape.eos_id]]).astype(np.int32)
        t = np.concatenate([draw(n - 1), [shape.eos_id]]).astype(np.int32)
        sents.append((s, t))
    return sents


def _pack(sents, max_tokens, max_sentences):
    """Greedy fill of length-sorted sentences while B * max(len) <= max_tokens (padded count)."""
    order = sorted(range(len(sents)), key=lambda i: (max(len(sents[i][0]), len(sents[i][1])), i))
    batches, cur, cur_max = [], [], 0
    for i in order:
        L = max(len(sents[i][0]), len(sents[i][1]))
        if cur and ((len(cur) + 1) * max(cur_max, L) > max_tokens or len(cur) >= max_sentences):
            batches.append(cur)
            cur, cur_max = [], 0
        cur.append(i)
        cur_max = max(cur_max, L)
    if cur:
        batches.append(cur)
    out = []
    for b in batches:
        if len(b) >= 8:
            b = b[: len(b) // 8 * 8]
        out.append(b)
    return out


# name -> (model preset, recipe)
WORKLOADS = {
    "tiny": dict(model="tiny", kind="fixed", B=8, L=16, seed=0),
    "base": dict(model="base", kind="translation", lo=10, hi=50, max_tokens=4096, seed=1),
    "big": dict(model="big", kind="translation", lo=10, hi=80, max_tokens=3584, seed=2),
    "big_accum": dict(model="big", kind="translation", lo=10, hi=120, max_tokens=3584, seed=3),
    "lm16": dict(model="lm16", kind="lm", blocks=8, block_len=512, seed=4),
    "lm16a": dict(model="lm16a", kind="lm", blocks=8, block_len=512, seed=5),
    "lm24": dict(model="lm24", kind="lm", blocks=8, block_len=512, seed=6),
}


def make_batches(workload, n_batches, *, shape: ModelShape = None, seed=None, max_tokens=None,
                 lo=None, hi=None, max_sentences=1024):
    """Return a list of n_batches Batch objects for a named workload (optionally on another model shape,
    token cap or length range, so that the parity tests can run the same recipe at small sizes)."""
    w = dict(WORKLOADS[workload])
    shape = shape or PRESETS[w["model"]]
    seed = w["seed"] if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    if w["kind"] == "fixed":
        for _ in range(n_batches):
            rows_s, rows_t = [], []
            for _ in range(w["B"]):
                rows_s.append(np.concatenate([rng.integers(N_SPECIAL, shape.vocab, w["L"] - 1), [shape.eos_id]]))
                rows_t.append(np.concatenate([rng.integers(N_SPECIAL, shape.vocab, w["L"] - 1), [shape.eos_id]]))
            lens = np.full(w["B"], w["L"], dtype=np.int32)
            out.append(Batch(_pad(rows_s, shape.pad_id), _pad(rows_t, shape.pad_id), lens.copy(), lens.copy()))
        return out
    if w["kind"] == "lm":
        nb = w["blocks"] if max_sentences >= w["blocks"] else max_sentences
        bl = w["block_len"] if hi is None else hi
        for _ in range(n_batches):
            ids = zipf_ids(rng, nb * bl, shape.vocab).reshape(nb, bl)
            out.append(Batch(None, ids, None, np.full(nb, bl, dtype=np.int32)))
        return out
    lo = w["lo"] if lo is None else lo
    hi = w["hi"] if hi is None else hi
    cap = w["max_tokens"] if max_tokens is None else max_tokens
    per_batch = max(1, cap // ((lo + hi) // 2))
    pool = _translation_pool(rng, shape, max(64, 4 * per_batch * n_batches), lo, hi, False)
    packed = _pack(pool, cap, max_sentences)
    if len(packed) > n_batches:
        packed = packed[:-1]           # the last batch holds the leftovers and is far below the cap
    pick = rng.permutation(len(packed))[:n_batches]
    assert len(pick) == n_batches, "pool too small"
    for j in pick:
        idx = packed[j]
        s = _pad([pool[i][0] for i in idx], shape.pad_id)
        t = _pad([pool[i][1] for i in idx], shape.pad_id)
        out.append(Batch(s, t, np.array([len(pool[i][0]) for i in idx], dtype=np.int32),
                         np.array([len(pool[i][1]) for i in idx], dtype=np.int32)))
    return out
