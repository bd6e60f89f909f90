"""Pins of the decoding oracle: an independently assembled network, the training criterion, and the property that
makes caching valid (a position's prediction does not depend on later tokens)."""
import numpy as np
import pytest

from oracle.decoding import DecodingOracle, top_k
from oracle.transformer import OracleTransformer, TrainConfig
from synth import ModelShape, init_params
from tests.torch_autograd_model import next_token_logprobs

SHAPES = [ModelShape(2, 2, 32, 4, 64, 50), ModelShape(1, 2, 32, 2, 48, 40, pre_norm=1), ModelShape(0, 2, 32, 4, 64, 50, pre_norm=1)]


@pytest.mark.parametrize("shape", SHAPES, ids=["post", "pre", "lm"])
def test_logprobs_match_an_independent_network(shape):
    params = init_params(shape, 3, generic=True)
    o = DecodingOracle(shape, params)
    rng = np.random.default_rng(0)
    src = rng.integers(4, shape.vocab, 7) if shape.enc_layers else None
    dec_in = np.concatenate([[shape.eos_id], rng.integers(4, shape.vocab, 8)])
    got = o.logprobs(o.encode(src), dec_in)
    want = next_token_logprobs(shape, params, src, dec_in)
    assert got.shape == (9, shape.vocab)
    assert np.max(np.abs(got - want)) < 1e-10
    assert np.allclose(np.exp(got).sum(axis=1), 1.0, atol=1e-12)


@pytest.mark.parametrize("shape", SHAPES, ids=["post", "pre", "lm"])
def test_prefix_invariance(shape):
    """The prediction at position t is the same whether or not later tokens are present: recomputing the prefix and
    re-using cached states must agree."""
    o = DecodingOracle(shape, init_params(shape, 4, generic=True))
    rng = np.random.default_rng(1)
    mem = o.encode(rng.integers(4, shape.vocab, 5)) if shape.enc_layers else None
    dec_in = np.concatenate([[shape.eos_id], rng.integers(4, shape.vocab, 6)])
    full = o.logprobs(mem, dec_in)
    for t in range(len(dec_in)):
        assert np.max(np.abs(o.next_logprobs(mem, dec_in[:t + 1]) - full[t])) < 1e-11
    other = dec_in.copy()
    other[4:] = (other[4:] + 1 - 4) % (shape.vocab - 4) + 4
    assert np.max(np.abs(o.logprobs(mem, other)[:4] - full[:4])) < 1e-11
    assert np.max(np.abs(o.logprobs(mem, other)[4] - full[4])) > 1e-6


def test_sum_of_step_predictions_is_the_training_nll():
    shape = SHAPES[0]
    params = init_params(shape, 5, generic=True)
    o = DecodingOracle(shape, params)
    rng = np.random.default_rng(2)
    src = rng.integers(4, shape.vocab, (1, 6)).astype(np.int32)
    tgt = np.concatenate([rng.integers(4, shape.vocab, 5), [shape.eos_id]])[None].astype(np.int32)
    lp = o.logprobs(o.encode(src[0]), np.concatenate([[shape.eos_id], tgt[0, :-1]]))
    nll = -sum(lp[t, tgt[0, t]] for t in range(6))
    trainer = OracleTransformer(shape, params, TrainConfig(dropout=0.0, label_smoothing=0.0))
    r = trainer.train_step(src, tgt, np.array([6]), np.array([6]))
    assert abs(r["nll_sum"] - nll) < 1e-9 * abs(nll)


ADAPTIVE = ModelShape(0, 2, 16, 2, 24, 37, pre_norm=1, cutoffs=(9, 20), factor=2)        # clusters of 9, 11, 17 tokens; widths 16, 8, 4


def test_adaptive_softmax_distribution_against_the_library_module_and_the_training_criterion():
    """The full-vocabulary distribution of a model with an adaptive softmax: PyTorch's own module (log_prob over all
    tokens) loaded with the same weights, probabilities that sum to one, and, token by token, minus the per-target
    negative log-likelihood of the training oracle."""
    import torch
    from oracle.transformer import _Grads
    shape = ADAPTIVE
    params = init_params(shape, 6, generic=True)
    o = DecodingOracle(shape, params)
    bounds = shape.cluster_bounds()
    mod = torch.nn.AdaptiveLogSoftmaxWithLoss(shape.d_model, shape.vocab, cutoffs=list(shape.cutoffs), div_value=float(shape.factor),
                                              head_bias=False).double()
    with torch.no_grad():
        mod.head.weight.copy_(torch.tensor(params["embed"]))
        for c in range(1, len(bounds)):
            mod.tail[c - 1][0].weight.copy_(torch.tensor(params[f"embed.{c}.proj"].T))
            mod.tail[c - 1][1].weight.copy_(torch.tensor(params[f"embed.{c}"]))
    y = np.random.default_rng(0).normal(size=(5, shape.d_model))
    got = o.vocabulary_logprobs(y)
    assert got.shape == (5, shape.vocab)
    with torch.no_grad():
        want = mod.log_prob(torch.tensor(y)).numpy()
    assert np.max(np.abs(got - want)) < 1e-12
    assert np.allclose(np.exp(got).sum(axis=1), 1.0, atol=1e-12)
    for w in (0, 8, 9, 19, 20, 36):                          # first and last token of every cluster
        nll, _, _ = o.model._adaptive_nll(y, np.full(5, w), 1.0, _Grads())
        assert np.max(np.abs(got[:, w] + nll)) < 1e-12


def test_adaptive_language_model_steps():
    """Adaptive inputs and adaptive softmax in step-wise prediction: prefix invariance, and the step predictions of a
    target sequence add up to the trainer's negative log-likelihood."""
    shape = ADAPTIVE
    params = init_params(shape, 7, generic=True)
    o = DecodingOracle(shape, params)
    rng = np.random.default_rng(3)
    tgt = rng.integers(0, shape.vocab, 9)                    # every cluster occurs as input and as target
    dec_in = np.concatenate([[shape.eos_id], tgt[:-1]])
    full = o.logprobs(None, dec_in)
    for t in (0, 3, 8):
        assert np.max(np.abs(o.next_logprobs(None, dec_in[:t + 1]) - full[t])) < 1e-11
    trainer = OracleTransformer(shape, params, TrainConfig(dropout=0.0, label_smoothing=0.0))
    r = trainer.train_step(None, tgt[None].astype(np.int32), None, np.array([9]))
    nll = -sum(full[t, tgt[t]] for t in range(9))
    assert abs(r["nll_sum"] - nll) < 1e-9 * abs(nll)


def test_top_k_order():
    assert top_k(np.array([-1.0, -0.5, -3.0, -0.5, -2.0]), 3) == [(-0.5, 1), (-0.5, 3), (-1.0, 0)]
