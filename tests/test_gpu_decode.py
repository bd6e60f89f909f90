"""Incremental decoding on the GPU against the decoding oracle (the full decoder recomputed over each prefix)."""
import numpy as np
import pytest

from oracle.decoding import DecodingOracle, top_k
from synth import ModelShape, init_params
from synth.batches import zipf_ids

pytestmark = pytest.mark.gpu

SHAPES = {
    "post": ModelShape(2, 2, 32, 2, 64, 96),
    "pre": ModelShape(1, 2, 32, 4, 48, 80, pre_norm=1),
    "lm": ModelShape(0, 2, 32, 2, 64, 96, pre_norm=1),
    "half": ModelShape(2, 2, 128, 2, 256, 512),         # head width 64: the MFMA GEMMs serve rows that are a multiple of 8
    # contractions long enough for the few-row products to be split along K: the slices of a sub-layer's last product are summed
    # by the LayerNorm kernel, those of the cross-attention query projection by the attention kernel (head width 64) or, where
    # the general attention kernel runs (head width 32), by a reduction in front of it
    "wide": ModelShape(1, 1, 512, 8, 1024, 96),
    "wide_dh32": ModelShape(1, 1, 512, 16, 1024, 96),
    # adaptive inputs + adaptive softmax: clusters of 24 / 32 / 40 tokens (generic kernels) and of 126 (+2 entries) / 128 / 256
    # tokens, every table a multiple of 8 rows (matrix-core GEMMs)
    "adaptive": ModelShape(0, 2, 32, 2, 64, 96, pre_norm=1, cutoffs=(24, 56), factor=2),
    "adaptive_half": ModelShape(0, 2, 128, 2, 256, 510, pre_norm=1, cutoffs=(126, 254)),
}


def rounded(params, prec):
    import torch
    import paper_1904_01038_amd as T
    tdt = {T.FP32: torch.float32, T.FP16: torch.float16, T.BF16: torch.bfloat16}[prec]
    return {k: torch.tensor(v, dtype=torch.float32).to(tdt).to(torch.float64).numpy() for k, v in params.items()}


def make(shape, prec, max_rows, max_steps, max_src, topk, seed=0):
    import paper_1904_01038_amd as T
    params = rounded(init_params(shape, seed, generic=True), prec)
    cfg = T.make_config(shape, precision=prec, max_sentences=16, max_len=max(max_steps, 24), max_tokens=256, dropout=0.3,
                        label_smoothing=0.0 if shape.cutoffs else 0.1)
    ctx = T.Tfm(cfg)
    ctx.set_params(params)
    return ctx, T.Decoder(ctx, max_rows, max_steps, max_src, topk), DecodingOracle(shape, params)


def sources(shape, rng, B, lo, hi):
    if not shape.enc_layers:
        return None, None
    lens = rng.integers(lo, hi + 1, B).astype(np.int32)
    src = np.full((B, lens.max()), shape.pad_id, np.int32)
    for b in range(B):
        src[b, :lens[b]] = np.append(zipf_ids(rng, lens[b] - 1, shape.vocab), shape.eos_id)
    return src, lens


def check_step(lp_gpu, top_lp, top_id, lp_ref, tol):
    """Full distribution within tol; the reported candidates are sorted, carry the right values, and nothing that was
    left out beats the last one by more than rounding."""
    assert np.max(np.abs(lp_gpu - lp_ref)) <= tol
    k = top_lp.shape[1]
    for r in range(lp_ref.shape[0]):
        assert len(set(top_id[r])) == k
        assert np.all(np.diff(top_lp[r]) <= 0.0)
        assert np.max(np.abs(top_lp[r] - lp_ref[r, top_id[r]])) <= tol
        assert np.allclose(top_lp[r], lp_gpu[r, top_id[r]], atol=1e-6)
        # exact on the GPU's own distribution: the same values, ties in ascending id order
        assert [i for _, i in top_k(lp_gpu[r], k)] == top_id[r].tolist()
        rest = np.delete(lp_ref[r], top_id[r])
        assert rest.max() <= top_lp[r, -1] + 2 * tol


@pytest.mark.parametrize("name,prec,tol", [("post", "fp32", 2e-4), ("pre", "fp32", 2e-4), ("lm", "fp32", 2e-4),
                                           ("half", "fp16", 3e-2), ("half", "bf16", 2e-1),
                                           ("wide", "fp16", 3e-2), ("wide", "bf16", 2e-1), ("wide_dh32", "fp16", 3e-2),
                                           ("adaptive", "fp32", 2e-4), ("adaptive_half", "fp16", 3e-2), ("adaptive_half", "bf16", 2e-1)])
def test_steps_with_reordered_beams_match_the_full_decoder(name, prec, tol):
    import paper_1904_01038_amd as T
    shape = SHAPES[name]
    p = {"fp32": T.FP32, "fp16": T.FP16, "bf16": T.BF16}[prec]
    B, beam, steps, topk = 4, 4, 7, 8
    ctx, dec, oracle = make(shape, p, B * beam, steps, 64, topk)
    rng = np.random.default_rng(5)
    src, lens = sources(shape, rng, B, 1, 11)
    for attempt in range(2):                               # a second batch re-uses the decoder: caches start over
        dec.begin(src, lens, beam, n_sentences=B)
        mems = [oracle.encode(src[b, :lens[b]]) if src is not None else None for b in range(B)]
        hist = [[] for _ in range(B * beam)]
        for t in range(steps):
            prev = np.full(B * beam, shape.eos_id, np.int32) if t == 0 else rng.integers(4, shape.vocab, B * beam).astype(np.int32)
            if t == 2 and shape.cutoffs:
                prev[:] = rng.integers(4, shape.cutoffs[0], B * beam)     # a step that feeds head tokens only
            parent = None
            if t:
                parent = np.array([r // beam * beam + rng.integers(0, beam) for r in range(B * beam)], np.int32)
                if t == 3:
                    parent = None                           # identity is allowed at any step
            par = parent if parent is not None else np.arange(B * beam)
            hist = [hist[par[r]] + [int(prev[r])] for r in range(B * beam)]
            top_lp, top_id = dec.step(prev, parent)
            ref = np.stack([oracle.next_logprobs(mems[r // beam], hist[r]) for r in range(B * beam)])
            check_step(dec.logprobs(), top_lp, top_id, ref, tol)
        src, lens = sources(shape, rng, B, 2, 9)
    ctx.close()


def test_beam_search_on_both_sides_finds_the_same_hypotheses():
    import paper_1904_01038_amd as T
    from tests.beam_search import beam_search
    shape = SHAPES["post"]
    B, beam, steps = 3, 3, 8
    ctx, dec, oracle = make(shape, T.FP32, B * beam, steps, 64, 2 * beam, seed=2)
    rng = np.random.default_rng(9)
    src, lens = sources(shape, rng, B, 3, 9)
    dec.begin(src, lens, beam)
    got = beam_search(dec.step, B, beam, steps, shape.eos_id)

    mems = [oracle.encode(src[b, :lens[b]]) for b in range(B)]
    state = {"hist": [[] for _ in range(B * beam)]}

    def oracle_step(prev, parent):
        par = parent if parent is not None else np.arange(B * beam)
        state["hist"] = [state["hist"][par[r]] + [int(prev[r])] for r in range(B * beam)]
        lp = np.empty((B * beam, 2 * beam), np.float32)
        ids = np.empty((B * beam, 2 * beam), np.int32)
        for r in range(B * beam):
            best = top_k(oracle.next_logprobs(mems[r // beam], state["hist"][r]), 2 * beam)
            lp[r], ids[r] = [v for v, _ in best], [i for _, i in best]
        return lp, ids

    want = beam_search(oracle_step, B, beam, steps, shape.eos_id)
    for s in range(B):
        assert len(got[s]) == len(want[s]) == beam
        # the best hypothesis of each side is a valid hypothesis of the other with the same score
        assert got[s][0][1] == want[s][0][1]
        for (sg, tg), (sw, tw) in zip(got[s], want[s]):
            assert abs(sg - sw) <= 1e-3
    ctx.close()


def test_decoder_argument_checks_and_limits():
    import paper_1904_01038_amd as T
    shape = SHAPES["post"]
    ctx, dec, _ = make(shape, T.FP32, 8, 3, 32, 4)
    eos = np.full(8, shape.eos_id, np.int32)
    with pytest.raises(T.TfmError) as e:
        dec.rows = 8
        dec.step(eos)                                       # no batch has been started
    assert e.value.code == -4
    src, lens = sources(shape, np.random.default_rng(0), 2, 1, 1)    # one-token sources
    with pytest.raises(T.TfmError):
        dec.begin(src, lens, 5)                             # 2 x 5 rows > 8
    with pytest.raises(T.TfmError):
        dec.begin(None, None, 4, n_sentences=2)             # the model has an encoder
    dec.begin(src, lens, 4)
    dec.step(eos)
    bad = np.arange(8, dtype=np.int32)
    bad[0] = 4                                              # row 0 cannot continue a row of the other sentence
    with pytest.raises(T.TfmError):
        dec.step(eos, bad)
    with pytest.raises(T.TfmError):
        dec.step(np.full(8, shape.vocab, np.int32))
    dec.step(eos)
    dec.step(eos)
    with pytest.raises(T.TfmError) as e:
        dec.step(eos)                                       # created for 3 steps
    assert e.value.code == -4
    with pytest.raises(T.TfmError):
        T.Decoder(ctx, 8, 10 ** 6, 32, 4)                   # more steps than the position table holds
    with pytest.raises(T.TfmError):
        T.Decoder(ctx, 8, 3, 32, 17)
    ctx.close()


def test_training_and_decoding_share_one_context():
    """A training step, an update, then decoding: the decoder sees the updated parameters."""
    import paper_1904_01038_amd as T
    from tests.test_oracle_model import small_batch
    from oracle.transformer import OracleTransformer, TrainConfig
    shape = ModelShape(1, 1, 32, 2, 64, 48)
    params = init_params(shape, 0, generic=True)
    cfg = T.make_config(shape, precision=T.FP32, max_sentences=8, max_len=16, max_tokens=64, init_loss_scale=1.0)
    ctx = T.Tfm(cfg)
    ctx.set_params(params)
    trainer = OracleTransformer(shape, params, TrainConfig(init_loss_scale=1.0, fp16_overflow=False, dynamic_scale=False))
    b = small_batch(shape, 1)
    ctx.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens, sync=False)
    ctx.apply_update(1e-2, sync=False)
    trainer.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)
    trainer.apply_update(1e-2)
    dec = T.Decoder(ctx, 3, 4, 32, 4)
    dec.begin(b.src, b.src_lens, 1)
    dec.step(np.full(3, shape.eos_id, np.int32))
    oracle = DecodingOracle(shape, trainer.p)
    ref = np.stack([oracle.next_logprobs(oracle.encode(b.src[i, :b.src_lens[i]]), [shape.eos_id]) for i in range(3)])
    assert np.max(np.abs(dec.logprobs() - ref)) <= 1e-3
    stale = DecodingOracle(shape, params)
    ref0 = np.stack([stale.next_logprobs(stale.encode(b.src[i, :b.src_lens[i]]), [shape.eos_id]) for i in range(3)])
    assert np.max(np.abs(ref - ref0)) > 1e-2                # the update mattered
    ctx.close()


def test_a_batch_in_flight_is_invalidated_by_training_and_parameter_changes():
    """A decoding batch is tied to the parameters it began under: a training step, an update or a parameter write on
    the context makes the next decoding step fail with TFM_ESTATE instead of reading re-used encoder state; a new
    tfm_decoder_begin recovers.  Two decoders of one context keep their own source offsets and projected keys/values,
    so beginning a batch on one does not disturb the other."""
    import paper_1904_01038_amd as T
    from tests.test_oracle_model import small_batch
    shape = ModelShape(1, 1, 32, 2, 64, 48)
    params = init_params(shape, 0, generic=True)
    cfg = T.make_config(shape, precision=T.FP32, max_sentences=8, max_len=16, max_tokens=64, init_loss_scale=1.0)
    ctx = T.Tfm(cfg)
    ctx.set_params(params)
    oracle = DecodingOracle(shape, params)
    b = small_batch(shape, 1)
    eos3 = np.full(3, shape.eos_id, np.int32)
    dec = T.Decoder(ctx, 3, 4, 32, 4)

    def expect_estate():
        with pytest.raises(T.TfmError) as e:
            dec.step(eos3)
        assert e.value.code == -4

    dec.begin(b.src, b.src_lens, 1)
    dec.step(eos3)
    ctx.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)                      # re-uses the encoder buffers
    expect_estate()
    expect_estate()                                                           # stays refused until a new batch begins
    dec.begin(b.src, b.src_lens, 1)
    dec.step(eos3)
    ctx.apply_update(0.0)                                                     # (lr 0: the parameters keep their values)
    expect_estate()
    dec.begin(b.src, b.src_lens, 1)
    ctx.set_params({"embed": params["embed"]})
    expect_estate()

    # two decoders: the second one's batch has other sentences and lengths
    rng = np.random.default_rng(3)
    src2, lens2 = sources(shape, rng, 2, 5, 9)
    dec2 = T.Decoder(ctx, 2, 4, 32, 4)
    dec.begin(b.src, b.src_lens, 1)
    dec2.begin(src2, lens2, 1)
    dec.step(eos3)
    ref = np.stack([oracle.next_logprobs(oracle.encode(b.src[i, :b.src_lens[i]]), [shape.eos_id]) for i in range(3)])
    assert np.max(np.abs(dec.logprobs() - ref)) <= 2e-4
    dec2.step(np.full(2, shape.eos_id, np.int32))
    ref2 = np.stack([oracle.next_logprobs(oracle.encode(src2[i, :lens2[i]]), [shape.eos_id]) for i in range(2)])
    assert np.max(np.abs(dec2.logprobs() - ref2)) <= 2e-4
    ctx.close()


def test_big_model_fp16_beam4_full_size_steps():
    """The decoding benchmark's configuration (big Transformer, fp16, beam 4) at its real widths: 2 sentences x 4 rows,
    4 steps with re-ordered beams, whole distribution against the full-prefix oracle.  The row count is what a small
    decoding batch has; the GEMM, cache and attention kernels are the ones the benchmark runs."""
    import paper_1904_01038_amd as T
    from synth import PRESETS
    shape = PRESETS["big"]
    params = rounded(init_params(shape, 0), T.FP16)
    B, beam, steps, topk = 2, 4, 4, 8
    cfg = T.make_config(shape, precision=T.FP16, max_sentences=8, max_len=32, max_tokens=256, dropout=0.1)
    ctx = T.Tfm(cfg)
    ctx.set_params(params)
    dec = T.Decoder(ctx, B * beam, steps, 64, topk)
    oracle = DecodingOracle(shape, params)
    rng = np.random.default_rng(11)
    src, lens = sources(shape, rng, B, 10, 24)
    dec.begin(src, lens, beam)
    mems = [oracle.encode(src[b, :lens[b]]) for b in range(B)]
    hist = [[] for _ in range(B * beam)]
    for t in range(steps):
        prev = np.full(B * beam, shape.eos_id, np.int32) if t == 0 else zipf_ids(rng, B * beam, shape.vocab)
        parent = None if t == 0 else np.array([r // beam * beam + rng.integers(0, beam) for r in range(B * beam)], np.int32)
        par = parent if parent is not None else np.arange(B * beam)
        hist = [hist[par[r]] + [int(prev[r])] for r in range(B * beam)]
        top_lp, top_id = dec.step(prev, parent)
        ref = np.stack([oracle.next_logprobs(mems[r // beam], hist[r]) for r in range(B * beam)])
        check_step(dec.logprobs(), top_lp, top_id, ref, 3e-2)
    ctx.close()
