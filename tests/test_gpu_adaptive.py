"""Adaptive input embeddings and adaptive softmax on the GPU against the oracle (language model only)."""
import numpy as np
import pytest

from synth import ModelShape, Batch
from tests.gpu_util import make_pair, step_both, max_rel, cosine, check_params_after_update

pytestmark = pytest.mark.gpu

SMALL = ModelShape(0, 2, 32, 2, 64, 120, pre_norm=1, cutoffs=(22, 56), factor=2)          # clusters 22 / 34 / 64, widths 32 / 16 / 8
HALF = ModelShape(0, 2, 128, 2, 256, 254, pre_norm=1, cutoffs=(62, 126), factor=4)        # 62+2 / 64 / 128 rows, widths 128 / 32 / 8
POST = ModelShape(0, 1, 32, 4, 48, 90, pre_norm=0, cutoffs=(30,), factor=4)               # one tail cluster of width 8


def lm_batch(shape, seed, lens, lo=0, hi=None):
    rng = np.random.default_rng(seed)
    lens = np.array(lens, dtype=np.int32)
    tgt = np.full((len(lens), lens.max()), shape.pad_id, dtype=np.int32)
    for i, n in enumerate(lens):
        tgt[i, :n] = rng.integers(lo, hi or shape.vocab, n)
    return Batch(None, tgt, None, lens)


@pytest.mark.parametrize("shape", [SMALL, POST], ids=["three_clusters", "post_norm"])
@pytest.mark.parametrize("dropout", [0.0, 0.2])
def test_fp32_window_and_update(shape, dropout):
    import paper_1904_01038_amd as T
    gpu, oracle = make_pair(shape, T.FP32, dropout=dropout, label_smoothing=0.0, max_sentences=8, max_len=24, max_tokens=96)
    for seed, lens in [(1, (9, 14, 5, 20)), (2, (24, 3, 3))]:
        rg, ro = step_both(gpu, oracle, lm_batch(shape, seed, lens))
        assert rg["ntokens"] == ro["ntokens"] and rg["overflow"] == 0
        assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"])
        assert abs(rg["nll_sum"] - ro["nll_sum"]) <= 1e-4 * abs(ro["nll_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert max_rel(gg[k], v) <= 1e-3, (k, max_rel(gg[k], v))
    grads = {k: v.copy() for k, v in oracle.unscaled_grads().items()}
    ug, uo = gpu.apply_update(1e-3), oracle.apply_update(1e-3)
    assert ug["skipped"] == uo["skipped"] == 0 and abs(ug["grad_norm"] - uo["grad_norm"]) <= 1e-4 * uo["grad_norm"]
    check_params_after_update(gpu.get_params(), oracle, grads, 1e-3)
    gpu.close()


@pytest.mark.parametrize("prec", ["fp16", "bf16"])
def test_half_precision_step(prec):
    import paper_1904_01038_amd as T
    p = T.FP16 if prec == "fp16" else T.BF16
    gpu, oracle = make_pair(HALF, p, dropout=0.1, label_smoothing=0.0, init_loss_scale=8.0, max_sentences=16, max_len=96, max_tokens=512)
    rg, ro = step_both(gpu, oracle, lm_batch(HALF, 3, (90, 64, 33, 96, 70, 81)))
    assert rg["overflow"] == 0
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-2 * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert cosine(gg[k], v) >= 0.999, (k, cosine(gg[k], v))
    gpu.close()


def test_clusters_that_do_not_occur_get_exactly_zero_gradients():
    import paper_1904_01038_amd as T
    gpu, oracle = make_pair(SMALL, T.FP32, label_smoothing=0.0, max_sentences=8, max_len=24, max_tokens=96)
    # first a batch that touches everything, so that stale values would show
    step_both(gpu, oracle, lm_batch(SMALL, 1, (12, 12)))
    gpu.apply_update(1e-3)
    oracle.apply_update(1e-3)
    # head tokens only: as inputs and as targets
    rg, ro = step_both(gpu, oracle, lm_batch(SMALL, 2, (10, 7), lo=0, hi=22))
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k in ("embed.1", "embed.1.proj", "embed.2", "embed.2.proj"):
        assert not gg[k].any() and not oracle.G[k].any(), k
    assert max_rel(gg["embed"], oracle.G["embed"]) <= 1e-3
    gpu.apply_update(1e-3)
    oracle.apply_update(1e-3)
    # cluster 2 only among the targets, cluster 1 only among the inputs: each side alone feeds a projection
    b = lm_batch(SMALL, 3, (8, 8), lo=56, hi=120)
    b.tgt[:, 0::2] = np.random.default_rng(4).integers(22, 56, b.tgt[:, 0::2].shape)     # inputs at odd positions come from cluster 1
    rg, ro = step_both(gpu, oracle, b)
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert max_rel(gg[k], v) <= 1e-3, k
    gpu.close()


def test_configuration_checks():
    import ctypes as C
    import paper_1904_01038_amd as T
    L, n = T.lib(), C.c_size_t()
    ok = T.make_config(SMALL, precision=T.FP32, max_sentences=4, max_len=16, max_tokens=64, label_smoothing=0.0)
    assert L.tfm_workspace_bytes(C.byref(ok), C.byref(n)) == 0
    bad = [ModelShape(1, 1, 32, 2, 64, 120, cutoffs=(22,)),                    # an encoder
           ModelShape(0, 1, 32, 2, 64, 120, cutoffs=(56, 22)),                 # not ascending
           ModelShape(0, 1, 32, 2, 64, 120, cutoffs=(22, 120)),                # reaches the vocabulary's end
           ModelShape(0, 1, 32, 2, 64, 120, cutoffs=(22, 56), factor=8),       # width 32 / 64 is no integer
           ModelShape(0, 1, 32, 2, 64, 120, cutoffs=(1,))]                     # eos outside the head
    for shape in bad:
        cfg = T.make_config(shape, precision=T.FP32, max_sentences=4, max_len=16, max_tokens=64, label_smoothing=0.0)
        assert L.tfm_workspace_bytes(C.byref(cfg), C.byref(n)) == -1, shape
    cfg = T.make_config(SMALL, precision=T.FP32, max_sentences=4, max_len=16, max_tokens=64, label_smoothing=0.1)
    assert L.tfm_workspace_bytes(C.byref(cfg), C.byref(n)) == -1
