"""An independent check model for the oracle pins: the same network assembled from PyTorch CPU library
routines (multi_head_attention_forward, layer_norm, linear, cross_entropy) with autograd doing the backward.
It is float64, batch-of-one, and used only by the CPU tests of the oracle.  It shares nothing with
oracle/ or with the HIP path."""
import math

import torch
import torch.nn.functional as F


def _pe(n, d):
    pe = torch.zeros(n, d, dtype=torch.float64)
    pos = torch.arange(n, dtype=torch.float64)[:, None]
    div = torch.exp(torch.arange(0, d, 2, dtype=torch.float64) * (-math.log(10000.0) / d))
    pe[:, 0::2] = torch.sin(pos * div)
    pe[:, 1::2] = torch.cos(pos * div)
    return pe


def _mha(P, pre, xq, xm, H, causal, cross):
    d = xq.shape[-1]
    if cross:
        w = torch.cat([P[pre + ".wq"], P[pre + ".wkv"]], 0)
        b = torch.cat([P[pre + ".bq"], P[pre + ".bkv"]], 0)
    else:
        w, b = P[pre + ".wqkv"], P[pre + ".bqkv"]
    mask = None
    if causal:
        n = xq.shape[0]
        mask = torch.triu(torch.full((n, n), float("-inf"), dtype=torch.float64), diagonal=1)
    out, _ = F.multi_head_attention_forward(
        xq[:, None, :], xm[:, None, :], xm[:, None, :], d, H, w, b, None, None, False, 0.0,
        P[pre + ".wo"], P[pre + ".bo"], training=False, need_weights=False, attn_mask=mask)
    return out[:, 0, :]


def _ln(P, pre, x):
    return F.layer_norm(x, (x.shape[-1],), P[pre + ".g"], P[pre + ".b"], 1e-5)


def _block(P, shape, ln, x, f):
    if shape.pre_norm:
        return x + f(_ln(P, ln, x))
    return _ln(P, ln, x + f(x))


def _ffn(P, pre, x):
    return F.linear(F.relu(F.linear(x, P[pre + ".w1"], P[pre + ".b1"])), P[pre + ".w2"], P[pre + ".b2"])


def loss_and_grads(shape, params, batch, label_smoothing):
    """Sum over sentences of the label-smoothed cross-entropy; returns (loss, {name: grad})."""
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    d, H = shape.d_model, shape.n_heads
    total = 0.0
    for b in range(len(batch.tgt_lens)):
        n = int(batch.tgt_lens[b])
        tgt = torch.tensor(batch.tgt[b, :n], dtype=torch.long)
        dec_in = torch.cat([torch.tensor([shape.eos_id]), tgt[:-1]])
        mem = None
        if shape.enc_layers:
            m = int(batch.src_lens[b])
            src = torch.tensor(batch.src[b, :m], dtype=torch.long)
            x = math.sqrt(d) * P["embed"][src] + _pe(m, d)
            for i in range(shape.enc_layers):
                pre = f"enc.{i}"
                x = _block(P, shape, pre + ".ln_self", x, lambda u: _mha(P, pre + ".self", u, u, H, False, False))
                x = _block(P, shape, pre + ".ln_ffn", x, lambda u: _ffn(P, pre + ".ffn", u))
            if shape.pre_norm:
                x = _ln(P, "enc.ln_final", x)
            mem = x
        y = math.sqrt(d) * P["embed"][dec_in] + _pe(n, d)
        for i in range(shape.dec_layers):
            pre = f"dec.{i}"
            y = _block(P, shape, pre + ".ln_self", y, lambda u: _mha(P, pre + ".self", u, u, H, True, False))
            if shape.enc_layers:
                y = _block(P, shape, pre + ".ln_cross", y, lambda u: _mha(P, pre + ".cross", u, mem, H, False, True))
            y = _block(P, shape, pre + ".ln_ffn", y, lambda u: _ffn(P, pre + ".ffn", u))
        if shape.pre_norm:
            y = _ln(P, "dec.ln_final", y)
        z = y @ P["embed"].T
        total = total + F.cross_entropy(z, tgt, reduction="sum", label_smoothing=label_smoothing)
    total.backward()
    return float(total), {k: v.grad.numpy() for k, v in P.items()}


def next_token_logprobs(shape, params, src, dec_in):
    """log-softmax over the vocabulary at every decoder position, for one sentence (no dropout)."""
    P = {k: torch.tensor(v, dtype=torch.float64) for k, v in params.items()}
    d, H = shape.d_model, shape.n_heads
    mem = None
    if shape.enc_layers:
        src = torch.tensor(src, dtype=torch.long)
        x = math.sqrt(d) * P["embed"][src] + _pe(len(src), d)
        for i in range(shape.enc_layers):
            pre = f"enc.{i}"
            x = _block(P, shape, pre + ".ln_self", x, lambda u: _mha(P, pre + ".self", u, u, H, False, False))
            x = _block(P, shape, pre + ".ln_ffn", x, lambda u: _ffn(P, pre + ".ffn", u))
        if shape.pre_norm:
            x = _ln(P, "enc.ln_final", x)
        mem = x
    dec_in = torch.tensor(dec_in, dtype=torch.long)
    y = math.sqrt(d) * P["embed"][dec_in] + _pe(len(dec_in), d)
    for i in range(shape.dec_layers):
        pre = f"dec.{i}"
        y = _block(P, shape, pre + ".ln_self", y, lambda u: _mha(P, pre + ".self", u, u, H, True, False))
        if shape.enc_layers:
            y = _block(P, shape, pre + ".ln_cross", y, lambda u: _mha(P, pre + ".cross", u, mem, H, False, True))
        y = _block(P, shape, pre + ".ln_ffn", y, lambda u: _ffn(P, pre + ".ffn", u))
    if shape.pre_norm:
        y = _ln(P, "dec.ln_final", y)
    return F.log_softmax(y @ P["embed"].T, dim=-1).numpy()
