"""Pins of the oracle's adaptive input embeddings and adaptive softmax (Applications, language modeling): PyTorch's own
adaptive-softmax module and embedding/linear routines, a distribution that sums to one over the whole vocabulary, the
flat softmax as the special case of one cluster, and finite differences through the whole language model."""
import numpy as np
import pytest
import torch

from oracle.transformer import OracleTransformer, TrainConfig, _Grads
from synth import ModelShape, Batch, init_params, param_specs

SHAPE = ModelShape(0, 2, 16, 2, 24, 37, pre_norm=1, cutoffs=(9, 20), factor=2)       # clusters of 9, 11, 17 tokens; widths 16, 8, 4
SHAPE4 = ModelShape(0, 1, 32, 2, 16, 50, pre_norm=0, cutoffs=(16,), factor=4)         # one tail cluster of width 8


def lm_batch(shape, seed, lens=(7, 5, 9)):
    rng = np.random.default_rng(seed)
    lens = np.array(lens, dtype=np.int32)
    tgt = np.full((len(lens), lens.max()), shape.pad_id, dtype=np.int32)
    for i, n in enumerate(lens):
        tgt[i, :n] = rng.integers(0, shape.vocab, n)          # every cluster occurs, as input and as target
    return Batch(None, tgt, None, lens)


def make(shape, seed=1, dropout=0.0):
    params = init_params(shape, seed, generic=True)
    return OracleTransformer(shape, params, TrainConfig(dropout=dropout, label_smoothing=0.0, init_loss_scale=1.0, seed=5)), params


@pytest.mark.parametrize("shape", [SHAPE, SHAPE4], ids=["three", "two"])
def test_output_side_against_the_library_module(shape):
    o, params = make(shape)
    bounds = shape.cluster_bounds()
    mod = torch.nn.AdaptiveLogSoftmaxWithLoss(shape.d_model, shape.vocab, cutoffs=list(shape.cutoffs), div_value=float(shape.factor),
                                              head_bias=False).double()
    with torch.no_grad():
        mod.head.weight.copy_(torch.tensor(params["embed"]))
        for c in range(1, len(bounds)):
            mod.tail[c - 1][0].weight.copy_(torch.tensor(params[f"embed.{c}.proj"].T))     # d -> d_c
            mod.tail[c - 1][1].weight.copy_(torch.tensor(params[f"embed.{c}"]))            # d_c -> V_c
    rng = np.random.default_rng(0)
    n = 40
    y = rng.normal(size=(n, shape.d_model))
    tgt = rng.integers(0, shape.vocab, n)
    tgt[:3] = [0, shape.cutoffs[0], shape.vocab - 1]                                       # boundaries
    g = _Grads()
    nll, dy, _ = o._adaptive_nll(y, tgt, 1.0, g)
    yt = torch.tensor(y, requires_grad=True)
    out = mod(yt, torch.tensor(tgt))
    assert np.max(np.abs(-out.output.detach().numpy() - nll)) < 1e-10
    (-out.output.sum()).backward()
    assert np.max(np.abs(yt.grad.numpy() - dy)) < 1e-10
    assert np.max(np.abs(mod.head.weight.grad.numpy() - g["embed"])) < 1e-10
    for c in range(1, len(bounds)):
        assert np.max(np.abs(mod.tail[c - 1][1].weight.grad.numpy() - g[f"embed.{c}"])) < 1e-10
        assert np.max(np.abs(mod.tail[c - 1][0].weight.grad.numpy().T - g[f"embed.{c}.proj"])) < 1e-10


def test_distribution_sums_to_one_over_the_vocabulary():
    o, _ = make(SHAPE)
    y = np.random.default_rng(1).normal(size=(1, SHAPE.d_model))
    total = 0.0
    for w in range(SHAPE.vocab):
        nll, _, _ = o._adaptive_nll(y, np.array([w]), 1.0, _Grads())
        total += np.exp(-nll[0])
    assert abs(total - 1.0) < 1e-12


def test_input_side_against_library_routines():
    o, params = make(SHAPE)
    ids = np.arange(SHAPE.vocab)
    got = o._lookup(ids)
    for c, (lo, hi) in enumerate(SHAPE.cluster_bounds()):
        idx = torch.arange(hi - lo)
        if c == 0:
            want = torch.nn.functional.embedding(idx, torch.tensor(params["embed"]))
        else:
            want = torch.nn.functional.linear(torch.nn.functional.embedding(idx, torch.tensor(params[f"embed.{c}"])),
                                              torch.tensor(params[f"embed.{c}.proj"]))
        assert np.max(np.abs(got[lo:hi] - want.numpy())) < 1e-13
    assert got.shape == (SHAPE.vocab, SHAPE.d_model)


def test_without_tail_tokens_it_is_the_flat_model_on_the_head():
    """Targets and inputs inside the head only: the loss equals that of a flat model whose vocabulary is the head
    plus the (never chosen) cluster entries."""
    o, params = make(SHAPE4)
    flat_shape = ModelShape(0, 1, 32, 2, 16, 16 + 1, pre_norm=0)
    flat = OracleTransformer(flat_shape, {k: v for k, v in params.items() if not k.startswith("embed.")},
                             TrainConfig(dropout=0.0, label_smoothing=0.0, init_loss_scale=1.0))
    rng = np.random.default_rng(3)
    lens = np.array([6, 4], np.int32)
    tgt = rng.integers(0, 16, (2, 6)).astype(np.int32)
    a = o.train_step(None, tgt, None, lens)
    b = flat.train_step(None, tgt, None, lens)
    assert abs(a["loss_sum"] - b["loss_sum"]) < 1e-10
    for k in flat.G:
        assert np.max(np.abs(o.G[k] - flat.G[k])) < 1e-10, k
    assert not o.G["embed.1"].any() and not o.G["embed.1.proj"].any()


@pytest.mark.parametrize("dropout", [0.0, 0.25])
def test_finite_differences_through_the_language_model(dropout):
    o, _ = make(SHAPE, dropout=dropout)
    batch = lm_batch(SHAPE, 2)
    r = o.train_step(None, batch.tgt, None, batch.tgt_lens)
    assert r["loss_sum"] == r["nll_sum"]
    rng = np.random.default_rng(0)
    h = 1e-5
    for pname, _ in param_specs(SHAPE):
        flat = o.p[pname].reshape(-1)
        nz = np.nonzero(o.G[pname].reshape(-1))[0]
        pick = rng.choice(nz, size=min(5, len(nz)), replace=False) if len(nz) else []
        for i in list(pick) + [int(rng.integers(flat.size))]:
            keep = flat[i]
            flat[i] = keep + h
            lp = o.forward_loss(None, batch.tgt, None, batch.tgt_lens, step=0)
            flat[i] = keep - h
            lm = o.forward_loss(None, batch.tgt, None, batch.tgt_lens, step=0)
            flat[i] = keep
            fd, an = (lp - lm) / (2 * h), o.G[pname].reshape(-1)[i]
            assert abs(fd - an) / max(1e-3, abs(fd), abs(an)) < 2e-6, (pname, i, fd, an)
