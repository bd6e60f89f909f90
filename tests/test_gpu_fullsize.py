"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (same shapes, same kernels):
one sub-batch of the named workload with dropout off, loss and every gradient tensor against the float64 oracle."""
import numpy as np
import pytest

from synth import PRESETS, WORKLOADS, make_batches, init_params
from tests.gpu_util import cosine

pytestmark = pytest.mark.gpu


def run_workload(workload, precision_name, n_sentences=None):
    import paper_1904_01038_amd as T
    from oracle.transformer import OracleTransformer, TrainConfig
    import torch
    shape = PRESETS[WORKLOADS[workload]["model"]]
    batch = make_batches(workload, 1)[0]
    prec = {"fp16": T.FP16, "bf16": T.BF16}[precision_name]
    tdt = {"fp16": torch.float16, "bf16": torch.bfloat16}[precision_name]
    scale = 8.0 if precision_name == "fp16" else 1.0
    params = init_params(shape, 0)
    params = {k: torch.tensor(v, dtype=torch.float32).to(tdt).to(torch.float64).numpy() for k, v in params.items()}
    max_tok = max(batch.ntokens, 0 if batch.src is None else int(batch.src_lens.sum()))
    cfg = T.make_config(shape, precision=prec, max_sentences=len(batch.tgt_lens), max_tokens=(max_tok + 63) // 64 * 64,
                        max_len=max(batch.tgt.shape[1], 0 if batch.src is None else batch.src.shape[1]),
                        dropout=0.0, init_loss_scale=scale, label_smoothing=0.0 if shape.cutoffs else 0.1)
    gpu = T.Tfm(cfg)
    gpu.set_params(params)
    rg = gpu.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    gg = gpu.get_grads()
    gpu.close()
    oracle = OracleTransformer(shape, params, TrainConfig(init_loss_scale=scale, fp16_overflow=False,
                                                          label_smoothing=0.0 if shape.cutoffs else 0.1))
    del params
    ro = oracle.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    return rg, ro, gg, oracle.G


def check(rg, ro, gg, G):
    assert rg["ntokens"] == ro["ntokens"]
    assert rg["overflow"] == 0
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-2 * abs(ro["loss_sum"])
    assert abs(rg["nll_sum"] - ro["nll_sum"]) <= 1e-2 * abs(ro["nll_sum"])
    worst = min((cosine(gg[k], v), k) for k, v in G.items())
    assert worst[0] >= 0.999, worst


def test_big_fp16_full_size_subbatch():
    check(*run_workload("big", "fp16"))


def test_base_bf16_full_size_subbatch():
    check(*run_workload("base", "bf16"))


def test_lm16_fp16_full_size_subbatch():
    check(*run_workload("lm16", "fp16"))


def test_lm16_adaptive_fp16_full_size_subbatch():
    """267.7 K types in three clusters: every tail GEMM at its real shape."""
    check(*run_workload("lm16a", "fp16"))
