"""Pins for the oracle's whole forward/backward: finite differences and an independent autograd model."""
import numpy as np
import pytest

from oracle.transformer import OracleTransformer, TrainConfig
from synth import ModelShape, Batch, init_params, param_specs
from tests.torch_autograd_model import loss_and_grads


def small_batch(shape, seed, lm=False):
    rng = np.random.default_rng(seed)
    tl = np.array([5, 3, 4], dtype=np.int32)
    sl = np.array([4, 6, 2], dtype=np.int32)
    def rows(lens):
        L = lens.max()
        a = np.full((len(lens), L), shape.pad_id, dtype=np.int32)
        for i, n in enumerate(lens):
            a[i, :n - 1] = rng.integers(4, shape.vocab, n - 1)
            a[i, n - 1] = shape.eos_id
        return a
    if lm:
        return Batch(None, rows(tl), None, tl)
    return Batch(rows(sl), rows(tl), sl, tl)


SHAPES = {
    "postnorm": ModelShape(1, 1, 8, 2, 16, 13),
    "prenorm": ModelShape(2, 1, 8, 2, 12, 11, pre_norm=1),
    "lm": ModelShape(0, 2, 8, 4, 16, 17, pre_norm=1),
    "lm_post": ModelShape(0, 1, 12, 2, 8, 11, pre_norm=0),
}


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("dropout", [(0.0, 0.0, 0.0), (0.3, 0.0, 0.0), (0.2, 0.25, 0.3), (0.0, 0.4, 0.0), (0.0, 0.0, 0.3)])
def test_finite_differences(name, dropout):
    """dropout = (sub-layer outputs and embeddings, attention weights, feed-forward hidden activations); the masks are
    functions of (seed, step, site, index) only, so they stay frozen while a parameter is perturbed."""
    shape = SHAPES[name]
    params = init_params(shape, 11, generic=True)
    batch = small_batch(shape, 5, lm=shape.enc_layers == 0)
    cfg = TrainConfig(dropout=dropout[0], attn_dropout=dropout[1], relu_dropout=dropout[2], label_smoothing=0.1,
                      init_loss_scale=1.0, seed=3)
    o = OracleTransformer(shape, params, cfg)
    o.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    rng = np.random.default_rng(0)
    h = 1e-5
    worst = 0.0
    for pname, shp in param_specs(shape):
        flat = o.p[pname].reshape(-1)
        idx = rng.choice(flat.size, size=min(6, flat.size), replace=False)
        for i in idx:
            keep = flat[i]
            flat[i] = keep + h
            lp = o.forward_loss(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens, step=0)
            flat[i] = keep - h
            lm = o.forward_loss(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens, step=0)
            flat[i] = keep
            fd = (lp - lm) / (2 * h)
            an = o.G[pname].reshape(-1)[i]
            err = abs(fd - an) / max(1e-3, abs(fd), abs(an))
            worst = max(worst, err)
            assert err < 2e-6, (pname, i, fd, an)
    assert worst < 2e-6


@pytest.mark.parametrize("name", list(SHAPES))
def test_against_autograd_library_model(name):
    shape = SHAPES[name]
    params = init_params(shape, 7, generic=True)
    batch = small_batch(shape, 9, lm=shape.enc_layers == 0)
    o = OracleTransformer(shape, params, TrainConfig(label_smoothing=0.1, init_loss_scale=1.0))
    r = o.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    loss, grads = loss_and_grads(shape, params, batch, 0.1)
    assert abs(loss - r["loss_sum"]) < 1e-9 * abs(loss)
    for k in params:
        np.testing.assert_allclose(o.G[k], grads[k], rtol=1e-8, atol=1e-10, err_msg=k)


def test_whole_model_with_zero_embedding_gives_n_log_v():
    shape = SHAPES["postnorm"]
    params = init_params(shape, 1, generic=True)
    params["embed"][...] = 0.0
    batch = small_batch(shape, 2)
    for eps in (0.0, 0.1, 0.4):
        o = OracleTransformer(shape, params, TrainConfig(label_smoothing=eps, init_loss_scale=1.0))
        r = o.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
        n = int(batch.tgt_lens.sum())
        assert r["ntokens"] == n
        assert abs(r["loss_sum"] - n * np.log(shape.vocab)) < 1e-10
        assert abs(r["nll_sum"] - n * np.log(shape.vocab)) < 1e-10


def test_padding_and_batch_composition_do_not_matter():
    shape = SHAPES["postnorm"]
    params = init_params(shape, 1, generic=True)
    batch = small_batch(shape, 2)
    cfg = TrainConfig(init_loss_scale=1.0)
    whole = OracleTransformer(shape, params, cfg)
    whole.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    parts = OracleTransformer(shape, params, cfg)
    tot = 0.0
    for b in range(3):
        sl, tl = batch.src_lens[b:b + 1], batch.tgt_lens[b:b + 1]
        r = parts.train_step(batch.src[b:b + 1, :sl[0]], batch.tgt[b:b + 1, :tl[0]], sl, tl)
        tot += r["loss_sum"]
    for k in params:
        np.testing.assert_allclose(whole.G[k], parts.G[k], rtol=1e-12, atol=1e-13)
    # accumulation == one concatenated batch also through the update (token normalisation)
    whole.apply_update(1e-2)
    parts.apply_update(1e-2)
    for k in params:
        np.testing.assert_allclose(whole.p[k], parts.p[k], rtol=1e-12, atol=1e-14)


def test_causality_of_decoder():
    shape = SHAPES["lm"]
    params = init_params(shape, 4, generic=True)
    o = OracleTransformer(shape, params, TrainConfig(init_loss_scale=1.0, label_smoothing=0.0))
    # per-token nll of a prefix must not change when later tokens change
    t1 = np.array([[5, 6, 7, 8, 9, 10]], dtype=np.int32)
    t2 = np.array([[5, 6, 7, 12, 4, 10]], dtype=np.int32)
    lens = np.array([6], dtype=np.int32)
    from oracle import transformer as T
    rec = []
    orig = T.label_smoothed_nll
    def spy(z, y, eps):
        out = orig(z, y, eps)
        rec.append(out[1].copy())
        return out
    T.label_smoothed_nll = spy
    try:
        o.train_step(None, t1, None, lens)
        o.train_step(None, t2, None, lens)
    finally:
        T.label_smoothed_nll = orig
    assert np.array_equal(rec[0][:3], rec[1][:3])
    assert not np.allclose(rec[0][4:], rec[1][4:])
