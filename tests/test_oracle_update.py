"""Pins for the oracle's update path: Adam, loss scaling, overflow skip, accumulation."""
import os

import numpy as np
import pytest
import torch

from oracle.transformer import OracleTransformer, TrainConfig
from synth import ModelShape, init_params
from tests.test_oracle_model import small_batch

SHAPE = ModelShape(1, 1, 8, 2, 16, 13)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "loss_scale_schedule.txt")


def run_steps(scale, n_updates=3, k=1, lr=1e-2, **kw):
    params = init_params(SHAPE, 3, generic=True)
    o = OracleTransformer(SHAPE, params, TrainConfig(init_loss_scale=scale, **kw))
    for u in range(n_updates):
        for j in range(k):
            b = small_batch(SHAPE, 100 + u * k + j)
            o.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)
        o.apply_update(lr)
    return o


def test_power_of_two_scale_is_exactly_transparent():
    a, b = run_steps(1.0), run_steps(128.0)
    for k in a.p:
        assert np.array_equal(a.p[k], b.p[k]), k
        assert np.array_equal(a.m[k], b.m[k]) and np.array_equal(a.v[k], b.v[k])


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_adam_matches_library_and_closed_forms(wd):
    """wd > 0: weight decay in the L2 form of the library routine (wd * w joins the gradient inside the step)."""
    params = init_params(SHAPE, 3, generic=True)
    o = OracleTransformer(SHAPE, params, TrainConfig(init_loss_scale=4.0, weight_decay=wd))
    tp = {k: torch.tensor(v.copy(), requires_grad=True) for k, v in params.items()}
    opt = torch.optim.Adam(list(tp.values()), lr=3e-3, betas=(0.9, 0.98), eps=1e-8, weight_decay=wd)
    for u in range(4):
        b = small_batch(SHAPE, 50 + u)
        o.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)
        g = o.unscaled_grads()
        if u == 0:
            w0 = {k: v.copy() for k, v in o.p.items()}
            g0 = {k: v.copy() for k, v in g.items()}
        for k in tp:
            tp[k].grad = torch.tensor(g[k])
        opt.step()
        r = o.apply_update(3e-3)
        if u == 0:                                   # step 1: delta = -lr * g / (|g| + eps), g including the decay term
            for k in w0:
                ge = g0[k] + wd * w0[k]
                np.testing.assert_allclose(o.p[k] - w0[k], -3e-3 * ge / (np.abs(ge) + 1e-8), rtol=1e-9, atol=1e-15)
        assert r["skipped"] == 0 and r["num_updates"] == u + 1
        for k in tp:
            np.testing.assert_allclose(o.p[k], tp[k].detach().numpy(), rtol=1e-12, atol=1e-15, err_msg=k)


def test_zero_gradient_changes_nothing_and_constant_gradient_closed_form():
    params = {k: v for k, v in init_params(SHAPE, 3).items()}
    o = OracleTransformer(SHAPE, params, TrainConfig(init_loss_scale=2.0))
    o.window_microbatches, o.window_ntokens = 1, 10
    o.apply_update(0.1)
    for k in params:
        assert np.array_equal(o.p[k], params[k])
    # constant gradient c: mhat = c, vhat = c^2 at every step -> every step moves by -lr*c/(|c|+eps)
    c = 0.25
    o = OracleTransformer(SHAPE, params, TrainConfig(init_loss_scale=2.0))
    for t in range(1, 5):
        for k in o.G:
            o.G[k][...] = c * o.loss_scale * 10
        o.window_microbatches, o.window_ntokens = 1, 10
        before = {k: v.copy() for k, v in o.p.items()}
        o.apply_update(0.1)
        for k in before:
            np.testing.assert_allclose(o.p[k] - before[k], -0.1 * c / (c + 1e-8), rtol=1e-9)


def test_hand_computed_loss_scale_schedule():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    params = init_params(SHAPE, 3, generic=True)
    o = OracleTransformer(SHAPE, params, TrainConfig(init_loss_scale=128.0, scale_window=4))
    for flag, scale, nupd in rows:
        b = small_batch(SHAPE, 1)
        before = {k: v.copy() for k, v in o.p.items()}
        r = o.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens, loss_mult=float("inf") if flag == "1" else 1.0)
        assert r["overflow"] == int(flag)
        u = o.apply_update(1e-3)
        assert u["skipped"] == int(flag)
        assert u["loss_scale_after"] == float(scale)
        assert u["num_updates"] == int(nupd)
        changed = any(not np.array_equal(before[k], o.p[k]) for k in before)
        assert changed == (flag == "0")             # a skipped update leaves the parameters bit-identical


def test_accumulation_window_with_injected_overflow():
    # 16 sub-batches, 5 and 11 overflow: one skip and ONE halving for the window; the next window applies at 64
    params = init_params(SHAPE, 3, generic=True)
    o = OracleTransformer(SHAPE, params, TrainConfig(init_loss_scale=128.0, fp16_overflow=True))
    p0 = {k: v.copy() for k, v in o.p.items()}
    flags = []
    for j in range(16):
        b = small_batch(SHAPE, 200 + j)
        flags.append(o.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens,
                                  loss_mult=1e6 if j in (5, 11) else 1.0)["overflow"])
    assert flags == [1 if j in (5, 11) else 0 for j in range(16)]
    u = o.apply_update(1e-3)
    assert (u["skipped"], u["loss_scale_after"], u["num_updates"], u["clean_steps"]) == (1, 64.0, 0, 0)
    assert all(np.array_equal(p0[k], o.p[k]) for k in p0)
    assert all(not o.G[k].any() for k in o.G)
    for j in range(16):
        b = small_batch(SHAPE, 300 + j)
        assert o.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)["loss_scale"] == 64.0
    u = o.apply_update(1e-3)
    assert (u["skipped"], u["loss_scale_after"], u["num_updates"]) == (0, 64.0, 1)


def test_k_copies_of_one_batch_equal_one():
    a = OracleTransformer(SHAPE, init_params(SHAPE, 3, generic=True), TrainConfig(init_loss_scale=8.0))
    b = OracleTransformer(SHAPE, init_params(SHAPE, 3, generic=True), TrainConfig(init_loss_scale=8.0))
    bt = small_batch(SHAPE, 9)
    a.train_step(bt.src, bt.tgt, bt.src_lens, bt.tgt_lens)
    for _ in range(4):
        b.train_step(bt.src, bt.tgt, bt.src_lens, bt.tgt_lens)
    a.apply_update(1e-2)
    b.apply_update(1e-2)
    for k in a.p:
        np.testing.assert_allclose(a.p[k], b.p[k], rtol=1e-13, atol=1e-16)


def test_clip_norm():
    o = run_steps(1.0, n_updates=1, clip_norm=1e9)
    ref = run_steps(1.0, n_updates=1)
    assert all(np.array_equal(o.p[k], ref.p[k]) for k in o.p)
    # a tiny clip norm scales the gradient to that norm: with Adam step 1 the update is sign-like either way,
    # so check the first moment instead: |m| = (1-b1) * clip
    c = run_steps(1.0, n_updates=1, clip_norm=1e-3)
    tot = np.sqrt(sum(float((v * v).sum()) for v in c.m.values()))
    assert abs(tot - 0.1 * 1e-3) < 1e-12
