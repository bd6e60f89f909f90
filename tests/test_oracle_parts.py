"""Pins for the oracle's building blocks: closed forms, invariants, library special cases, brute force."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import transformer as T


# ---- loss ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("eps", [0.0, 0.1, 0.5])
def test_loss_uniform_logits_is_log_v(eps):
    V = 37
    z = np.full((5, V), 0.73)
    y = np.array([0, 3, 36, 1, 2])
    loss, nll, dz = T.label_smoothed_nll(z, y, eps)
    assert np.allclose(loss, math.log(V), atol=1e-13)
    assert np.allclose(nll, math.log(V), atol=1e-13)


def test_loss_gradient_rows_sum_to_zero_and_match_library():
    rng = np.random.default_rng(0)
    V, n, eps = 29, 7, 0.1
    z = rng.normal(0, 3, (n, V))
    y = rng.integers(0, V, n)
    loss, nll, dz = T.label_smoothed_nll(z, y, eps)
    assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-13)
    zt = torch.tensor(z, requires_grad=True)
    lt = F.cross_entropy(zt, torch.tensor(y), reduction="sum", label_smoothing=eps)
    lt.backward()
    assert abs(float(lt) - loss.sum()) < 1e-11
    np.testing.assert_allclose(dz, zt.grad.numpy(), atol=1e-13)
    l0, nll0, _ = T.label_smoothed_nll(z, y, 0.0)
    np.testing.assert_allclose(l0, nll0)
    np.testing.assert_allclose(nll0, nll)          # nll does not depend on eps
    ref = F.cross_entropy(torch.tensor(z), torch.tensor(y), reduction="none").numpy()
    np.testing.assert_allclose(nll, ref, atol=1e-12)


def test_loss_minimum_is_entropy_of_smoothed_target():
    V, eps = 11, 0.1
    q = np.full(V, eps / V)
    q[4] += 1 - eps
    z = np.log(q)[None, :] + 2.5                  # softmax(z) = q
    loss, _, dz = T.label_smoothed_nll(z, np.array([4]), eps)
    H = -(1 - eps + eps / V) * math.log(1 - eps + eps / V) - (V - 1) * (eps / V) * math.log(eps / V)
    assert abs(loss[0] - H) < 1e-12
    assert np.allclose(dz, 0.0, atol=1e-14)
    rng = np.random.default_rng(1)
    for _ in range(20):                            # any other logits give a larger loss
        l2, _, _ = T.label_smoothed_nll(z + rng.normal(0, 0.5, z.shape), np.array([4]), eps)
        assert l2[0] > H


def test_loss_large_logits_are_stable():
    z = np.array([[1000.0, 0.0, -1000.0]])
    loss, nll, dz = T.label_smoothed_nll(z, np.array([0]), 0.0)
    assert np.isfinite(loss).all() and abs(nll[0]) < 1e-12


# ---- attention ------------------------------------------------------------------------------------------------
def brute_attention(q, k, v, H, causal):
    n, d = q.shape
    m = k.shape[0]
    dh = d // H
    out = np.zeros((n, d))
    for h in range(H):
        for i in range(n):
            w = []
            for j in range(m):
                if causal and j > i:
                    w.append(0.0)
                    continue
                s = sum(q[i, h * dh + c] * k[j, h * dh + c] for c in range(dh)) / math.sqrt(dh)
                w.append(math.exp(s))
            tot = sum(w)
            for c in range(dh):
                out[i, h * dh + c] = sum(w[j] * v[j, h * dh + c] for j in range(m)) / tot
    return out


@pytest.mark.parametrize("causal", [False, True])
def test_attention_brute_force_and_rows(causal):
    rng = np.random.default_rng(2)
    n, m, d, H = 5, (5 if causal else 7), 12, 3
    q, k, v = rng.normal(size=(n, d)), rng.normal(size=(m, d)), rng.normal(size=(m, d))
    ctx, cache = T.attention_fwd(q, k, v, H, causal)
    np.testing.assert_allclose(ctx, brute_attention(q, k, v, H, causal), atol=1e-12)
    for p in cache[3]:
        assert np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
        if causal:
            assert np.all(p[np.triu_indices(n, 1)] == 0.0)


def test_attention_special_cases():
    rng = np.random.default_rng(3)
    d, H = 8, 2
    q = rng.normal(size=(4, d))
    v1 = rng.normal(size=(1, d))
    ctx, _ = T.attention_fwd(q, rng.normal(size=(1, d)), v1, H, False)
    np.testing.assert_allclose(ctx, np.repeat(v1, 4, 0), atol=1e-14)       # one key -> output = v
    v = rng.normal(size=(6, d))
    ctx, _ = T.attention_fwd(q, np.zeros((6, d)), v, H, False)               # equal scores -> mean of v
    np.testing.assert_allclose(ctx, np.repeat(v.mean(0, keepdims=True), 4, 0), atol=1e-14)
    qq = rng.normal(size=(6, d))
    ctx, _ = T.attention_fwd(qq, np.zeros((6, d)), v, H, True)               # causal: running mean
    np.testing.assert_allclose(ctx, np.cumsum(v, 0) / np.arange(1, 7)[:, None], atol=1e-14)


def test_attention_backward_against_autograd():
    rng = np.random.default_rng(4)
    n, m, d, H = 4, 6, 8, 2
    q, k, v, do = (rng.normal(size=s) for s in [(n, d), (m, d), (m, d), (n, d)])
    ctx, cache = T.attention_fwd(q, k, v, H, False)
    dq, dk, dv = T.attention_bwd(do, cache)
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, k, v))
    def heads(a):
        return a.reshape(a.shape[0], H, d // H).transpose(0, 1)
    o = F.scaled_dot_product_attention(heads(tq), heads(tk), heads(tv)).transpose(0, 1).reshape(n, d)
    np.testing.assert_allclose(ctx, o.detach().numpy(), atol=1e-12)
    (o * torch.tensor(do)).sum().backward()
    np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12)


def test_attention_weight_dropout_against_autograd_and_special_cases():
    """Dropout on the attention weights with a given keep mask: value and all three gradients against an autograd
    graph built from library primitives (softmax, masked scaling, matmul); one key -> v / (1-p) or 0; an all-true mask
    with p = 0 is the plain attention; dropped weights contribute nothing to dV."""
    rng = np.random.default_rng(14)
    n, m, d, H, pd = 5, 7, 8, 2, 0.3
    q, k, v, do = (rng.normal(size=s) for s in [(n, d), (m, d), (m, d), (n, d)])
    keep = [rng.random((n, m)) >= pd for _ in range(H)]
    for causal in (False, True):
        mm = n if causal else m
        kk, vv = k[:mm], v[:mm]
        kp = [x[:, :mm] for x in keep]
        ctx, cache = T.attention_fwd(q, kk, vv, H, causal, kp, pd)
        dq, dk, dv = T.attention_bwd(do, cache)
        tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (q, kk, vv))
        outs = []
        for h in range(H):
            sl = slice(h * d // H, (h + 1) * d // H)
            sc = tq[:, sl] @ tk[:, sl].T / math.sqrt(d // H)
            if causal:
                sc = sc.masked_fill(torch.triu(torch.ones(n, mm, dtype=torch.bool), 1), float("-inf"))
            w = torch.softmax(sc, dim=-1) * torch.tensor(kp[h], dtype=torch.float64) / (1.0 - pd)
            outs.append(w @ tv[:, sl])
        o = torch.cat(outs, dim=1)
        np.testing.assert_allclose(ctx, o.detach().numpy(), atol=1e-12)
        (o * torch.tensor(do)).sum().backward()
        np.testing.assert_allclose(dq, tq.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dk, tk.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dv, tv.grad.numpy(), atol=1e-12)
    # one key: the single weight is 1, so the output is v / (1-p) where it is kept and 0 where it is dropped
    v1 = rng.normal(size=(1, d))
    kp1 = [np.array([[True], [False], [True], [False], [True]]), np.array([[False], [False], [True], [True], [True]])]
    ctx, _ = T.attention_fwd(q, rng.normal(size=(1, d)), v1, H, False, kp1, pd)
    for h in range(H):
        sl = slice(h * d // H, (h + 1) * d // H)
        np.testing.assert_allclose(ctx[:, sl], np.where(kp1[h], v1[:, sl] / (1 - pd), 0.0), atol=1e-14)
    # nothing dropped, p = 0: the plain attention, bit for bit
    all_true = [np.ones((n, m), bool)] * H
    a, _ = T.attention_fwd(q, k, v, H, False, all_true, 0.0)
    b, _ = T.attention_fwd(q, k, v, H, False)
    assert np.array_equal(a, b)
    # a key dropped for every query receives no value gradient
    kp = [np.ones((n, m), bool) for _ in range(H)]
    for x in kp:
        x[:, 2] = False
    _, cache = T.attention_fwd(q, k, v, H, False, kp, pd)
    assert not T.attention_bwd(do, cache)[2][2].any()


def test_attention_keep_mask_generator():
    key = T.dropout_key(9, 2, T.site_id(1, 0, 3))
    p, H = 0.1, 4
    masks = [T.attention_keep(key, 11, 300, H, h, 50, p) for h in range(H)]
    allm = np.stack(masks)
    p_eff = T.dropout_threshold(p) / 65536.0
    assert abs((1.0 - allm.mean()) - p_eff) < 5 * math.sqrt(p_eff * (1 - p_eff) / allm.size)
    assert T.attention_keep(key, 11, 4, H, 0, 50, 0.0).all()
    # queries are addressed by their packed row: a window equals the same rows of the big mask; keys by their index
    np.testing.assert_array_equal(T.attention_keep(key, 20, 5, H, 2, 50, p), masks[2][9:14])
    np.testing.assert_array_equal(T.attention_keep(key, 11, 300, H, 1, 33, p), masks[1][:, :33])
    assert (masks[0] != masks[1]).mean() > 0.1                      # heads draw different bits
    # scalar re-computation with Python integers
    M = (1 << 64) - 1
    def mix(z):
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        return z ^ (z >> 31)
    for (i, h, j) in [(0, 0, 0), (7, 3, 49), (299, 1, 18), (100, 2, 5)]:
        e = (((11 + i) * H + h) << 16) + j
        w = mix((int(key) + (e >> 2) * 0x9E3779B97F4A7C15) & M)
        assert bool(masks[h][i, j]) == (((w >> (16 * (e & 3))) & 0xFFFF) >= int(p * 65536))


# ---- layer norm -------------------------------------------------------------------------------------------------
def test_layer_norm_invariants_and_library():
    rng = np.random.default_rng(5)
    x = rng.normal(2.0, 3.0, (6, 16))
    y, cache = T.layer_norm_fwd(x, np.ones(16), np.zeros(16))
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-14)
    var = x.var(axis=1)
    np.testing.assert_allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-12)
    g, b = rng.normal(size=16), rng.normal(size=16)
    y, cache = T.layer_norm_fwd(x, g, b)
    xt, gt, bt = (torch.tensor(a, requires_grad=True) for a in (x, g, b))
    yt = F.layer_norm(xt, (16,), gt, bt, 1e-5)
    np.testing.assert_allclose(y, yt.detach().numpy(), atol=1e-13)
    dy = rng.normal(size=y.shape)
    (yt * torch.tensor(dy)).sum().backward()
    dx, dg, db = T.layer_norm_bwd(dy, cache)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-12)
    assert np.allclose(dx.sum(axis=1), 0.0, atol=1e-13)
    # sum_j dx_j xhat_j vanishes only up to eps: it equals rstd * sum(dxhat*xhat) * eps / (var + eps)
    xhat, rstd = cache[0], cache[1][:, 0]
    expect = rstd * ((dy * g) * xhat).sum(axis=1) * 1e-5 / (x.var(axis=1) + 1e-5)
    np.testing.assert_allclose((dx * xhat).sum(axis=1), expect, rtol=1e-6, atol=1e-13)


# ---- positional encoding ---------------------------------------------------------------------------------------
def test_positional_encoding_identities():
    d = 16
    pe = T.positional_encoding(50, d)
    np.testing.assert_array_equal(pe[0], np.tile([0.0, 1.0], d // 2))
    np.testing.assert_allclose(pe[:, 0::2] ** 2 + pe[:, 1::2] ** 2, 1.0, atol=1e-14)
    w = 1.0 / np.power(10000.0, 2.0 * np.arange(d // 2) / d)      # PE(t+1) is a fixed rotation of PE(t)
    s, c = pe[:-1, 0::2], pe[:-1, 1::2]
    np.testing.assert_allclose(pe[1:, 0::2], s * np.cos(w) + c * np.sin(w), atol=1e-12)
    np.testing.assert_allclose(pe[1:, 1::2], c * np.cos(w) - s * np.sin(w), atol=1e-12)
    assert abs(pe[7, 0] - math.sin(7.0)) < 1e-15 and abs(pe[3, d - 1] - math.cos(3.0 / 10000 ** ((d - 2) / d))) < 1e-15


# ---- dropout ------------------------------------------------------------------------------------------------------
def splitmix64_next(state):
    """Scalar reference of the published splitmix64 step with Python integers (independent of numpy wrapping)."""
    M = (1 << 64) - 1
    state = (state + 0x9E3779B97F4A7C15) & M
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    return state, z ^ (z >> 31)


def test_mix64_is_the_splitmix64_finaliser():
    # first outputs of splitmix64 seeded with 0 are mix64(k * golden), k = 1, 2, 3
    st = 0
    for k in range(1, 6):
        st, out = splitmix64_next(st)
        got = int(T._mix64(np.uint64((k * 0x9E3779B97F4A7C15) & ((1 << 64) - 1))))
        assert got == out
    # published first output of splitmix64 with seed 0
    assert splitmix64_next(0)[1] == 0xE220A8397B1DCDAF


def test_dropout_mask_properties():
    key = T.dropout_key(5, 3, T.site_id(1, 2, 0))
    p = 0.1
    keep = T.dropout_keep(key, 0, 400, 64, p)
    n = keep.size
    rate = 1.0 - keep.mean()
    p_eff = T.dropout_threshold(p) / 65536.0
    assert abs(rate - p_eff) < 5 * math.sqrt(p_eff * (1 - p_eff) / n)
    # rows are addressed absolutely: a window of the mask equals the same rows of the big one
    np.testing.assert_array_equal(T.dropout_keep(key, 17, 5, 64, p), keep[17:22])
    assert T.dropout_keep(key, 0, 8, 64, 0.0).all()
    # another step / site / seed gives another mask
    for other in (T.dropout_key(5, 4, T.site_id(1, 2, 0)), T.dropout_key(5, 3, T.site_id(1, 2, 2)),
                  T.dropout_key(6, 3, T.site_id(1, 2, 0))):
        assert (T.dropout_keep(other, 0, 400, 64, p) != keep).mean() > 0.1
    # scalar re-computation with Python integers for a few elements
    M = (1 << 64) - 1
    def mix(z):
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        return z ^ (z >> 31)
    for (r, c) in [(0, 0), (3, 5), (399, 63), (100, 2)]:
        e = r * 64 + c
        w = mix((int(key) + (e >> 2) * 0x9E3779B97F4A7C15) & M)
        assert bool(keep[r, c]) == (((w >> (16 * (e & 3))) & 0xFFFF) >= int(p * 65536))
