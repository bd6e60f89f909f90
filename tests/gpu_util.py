"""Helpers of the GPU parity tests: run the same seeded inputs through the HIP path (C boundary) and the oracle."""
import numpy as np

from oracle.transformer import OracleTransformer, TrainConfig
from synth import init_params


def make_pair(shape, precision, *, dropout=0.0, seed_params=0, max_sentences=64, max_len=64, max_tokens=1024,
              init_loss_scale=1.0, scale_window=2000, clip_norm=0.0, label_smoothing=0.1, seed=0, generic=True,
              round_params=True, attn_dropout=0.0, relu_dropout=0.0, weight_decay=0.0):
    import paper_1904_01038_amd as T
    params = init_params(shape, seed_params, generic=generic)
    if round_params:
        # both sides start from parameters that are exactly representable in the compute dtype
        import torch
        tdt = {T.FP32: torch.float32, T.FP16: torch.float16, T.BF16: torch.bfloat16}[precision]
        params = {k: torch.tensor(v, dtype=torch.float32).to(tdt).to(torch.float64).numpy() for k, v in params.items()}
    cfg = T.make_config(shape, precision=precision, max_sentences=max_sentences, max_len=max_len, max_tokens=max_tokens,
                        dropout=dropout, label_smoothing=label_smoothing, init_loss_scale=init_loss_scale,
                        scale_window=scale_window, clip_norm=clip_norm, seed=seed, attn_dropout=attn_dropout,
                        relu_dropout=relu_dropout, weight_decay=weight_decay)
    gpu = T.Tfm(cfg)
    assert sorted(gpu.param_names) == sorted(params.keys())          # same names; the library orders them by its own memory layout
    gpu.set_params(params)
    ocfg = TrainConfig(weight_decay=weight_decay, dropout=dropout, attn_dropout=attn_dropout, relu_dropout=relu_dropout, label_smoothing=label_smoothing, init_loss_scale=init_loss_scale,
                       scale_window=scale_window, clip_norm=clip_norm, fp16_overflow=(precision == T.FP16),
                       dynamic_scale=(precision == T.FP16), seed=seed)
    return gpu, OracleTransformer(shape, params, ocfg)


def max_rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = max(float(np.max(np.abs(b))), 1e-30)
    return float(np.max(np.abs(a - b))) / den


def cosine(a, b):
    a, b = np.asarray(a, dtype=np.float64).ravel(), np.asarray(b, dtype=np.float64).ravel()
    na, nb = np.linalg.norm(a), np.linalg.norm(b)
    if na == 0.0 and nb == 0.0:
        return 1.0
    return float(a @ b / max(na * nb, 1e-300))


def step_both(gpu, oracle, batch, loss_mult=None):
    if loss_mult is not None:
        gpu.debug_set_loss_multiplier(loss_mult)
    rg = gpu.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    ro = oracle.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens,
                           loss_mult=1.0 if loss_mult is None else loss_mult)
    return rg, ro


def check_params_after_update(pg, oracle, grads_before, lr, rel=2e-2, solid_frac=1e-3):
    """Adam divides by |g|: where the true gradient is (numerically) zero, e.g. the key bias of an attention
    layer, rounding noise decides the sign of the step.  Elements with a meaningful gradient must agree to a
    small fraction of the step; the others may differ by at most a full step in either direction."""
    for k, v in oracle.p.items():
        g = np.abs(grads_before[k])
        solid = g >= solid_frac * max(float(g.max()), 1e-300)
        err = np.abs(np.asarray(pg[k], dtype=np.float64) - v)
        assert np.all(err[solid] <= rel * lr + 1e-6 * np.abs(v[solid])), (k, float(err[solid].max()))
        assert np.all(err <= 2.1 * lr + 1e-6 * np.abs(v)), (k, float(err.max()))
