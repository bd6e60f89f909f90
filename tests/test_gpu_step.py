"""GPU parity of the whole training step against the oracle, through the C boundary."""
import numpy as np
import pytest

from synth import ModelShape, PRESETS, make_batches
from tests.gpu_util import make_pair, max_rel, cosine, step_both, check_params_after_update
from tests.test_oracle_model import small_batch

pytestmark = pytest.mark.gpu

# tolerances of the fp32 path and of the half-precision paths (loss relative, gradient max-relative / cosine)
FP32_LOSS, FP32_GRAD = 1e-4, 1e-3
HALF_LOSS, HALF_COS = 1e-2, 0.999


def check_fp32(gpu, oracle, rg, ro):
    assert rg["ntokens"] == ro["ntokens"]
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= FP32_LOSS * abs(ro["loss_sum"])
    assert abs(rg["nll_sum"] - ro["nll_sum"]) <= FP32_LOSS * abs(ro["nll_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert max_rel(gg[k], v) <= FP32_GRAD, (k, max_rel(gg[k], v))


def test_tiny_config_fp32_step_and_update():
    import paper_1904_01038_amd as T
    shape = PRESETS["tiny"]
    gpu, oracle = make_pair(shape, T.FP32, generic=False, max_sentences=8, max_len=16, max_tokens=128)
    batch = make_batches("tiny", 1)[0]
    rg, ro = step_both(gpu, oracle, batch)
    assert rg["overflow"] == 0 and ro["overflow"] == 0
    check_fp32(gpu, oracle, rg, ro)
    gb = oracle.unscaled_grads()
    ug, uo = gpu.apply_update(1e-3), oracle.apply_update(1e-3)
    assert (ug["skipped"], ug["num_updates"], ug["ntokens_total"]) == (0, 1, 128)
    assert abs(ug["grad_norm"] - uo["grad_norm"]) <= 1e-3 * uo["grad_norm"]
    check_params_after_update(gpu.get_params(), oracle, gb, 1e-3)
    m, v2 = gpu.get_adam(0), gpu.get_adam(1)
    for k in oracle.m:
        assert max_rel(m[k], oracle.m[k]) <= FP32_GRAD, k
        assert max_rel(v2[k], oracle.v[k]) <= 2 * FP32_GRAD, k


SMALL = {
    "post": ModelShape(2, 2, 32, 4, 64, 48),
    "pre": ModelShape(1, 2, 32, 2, 40, 51, pre_norm=1),
    "lm_pre": ModelShape(0, 2, 32, 4, 64, 48, pre_norm=1),
    "lm_post": ModelShape(0, 1, 24, 3, 32, 40, pre_norm=0),
}


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("dropout", [0.0, 0.25])
def test_small_models_fp32(name, dropout):
    import paper_1904_01038_amd as T
    shape = SMALL[name]
    gpu, oracle = make_pair(shape, T.FP32, dropout=dropout, seed=5)
    lm = shape.enc_layers == 0
    for it in range(2):                      # second step: dropout masks of step 1, accumulation into G
        batch = small_batch(shape, 20 + it, lm=lm)
        rg, ro = step_both(gpu, oracle, batch)
        check_fp32(gpu, oracle, rg, ro)
    gb = oracle.unscaled_grads()
    ug, uo = gpu.apply_update(5e-3), oracle.apply_update(5e-3)
    assert ug["ntokens_total"] == uo["ntokens_total"]
    check_params_after_update(gpu.get_params(), oracle, gb, 5e-3)


@pytest.mark.parametrize("name", list(SMALL))
def test_small_models_fp32_with_attention_and_relu_dropout(name):
    """All three dropout kinds at once (sub-layer outputs, attention weights, feed-forward hidden activations): the
    generic kernels, two steps, then the update."""
    import paper_1904_01038_amd as T
    shape = SMALL[name]
    gpu, oracle = make_pair(shape, T.FP32, dropout=0.2, attn_dropout=0.25, relu_dropout=0.3, seed=7)
    lm = shape.enc_layers == 0
    for it in range(2):
        batch = small_batch(shape, 40 + it, lm=lm)
        rg, ro = step_both(gpu, oracle, batch)
        check_fp32(gpu, oracle, rg, ro)
    gb = oracle.unscaled_grads()
    ug, uo = gpu.apply_update(5e-3), oracle.apply_update(5e-3)
    check_params_after_update(gpu.get_params(), oracle, gb, 5e-3)


@pytest.mark.parametrize("precision", ["fp16", "bf16"])
@pytest.mark.parametrize("name", ["post", "lm_pre"])
def test_half_precision_models_with_attention_and_relu_dropout(precision, name):
    """The matrix-core kernels with dropout on the attention weights (heads of width 64, sentences of one and of several
    64-row chunks) and on the feed-forward hidden activations (GEMM epilogue and the masked input gradient)."""
    import paper_1904_01038_amd as T
    shape = {"post": ModelShape(2, 2, 128, 2, 256, 512), "lm_pre": ModelShape(0, 2, 128, 2, 256, 512, pre_norm=1)}[name]
    prec = T.FP16 if precision == "fp16" else T.BF16
    scale = 128.0 if precision == "fp16" else 1.0
    for hi in (40, 150):                      # every sentence within one chunk / up to three chunks
        gpu, oracle = make_pair(shape, prec, generic=True, init_loss_scale=scale, max_sentences=64, max_len=160, max_tokens=2048,
                                dropout=0.1, attn_dropout=0.2, relu_dropout=0.15, seed=3)
        if shape.enc_layers:
            batch = make_batches("base", 1, shape=shape, max_tokens=600, lo=5, hi=hi)[0]
        else:
            batch = make_batches("lm16", 1, shape=shape, hi=hi, max_sentences=6)[0]
        rg, ro = step_both(gpu, oracle, batch)
        assert rg["overflow"] == 0 and ro["overflow"] == 0
        assert abs(rg["loss_sum"] - ro["loss_sum"]) <= HALF_LOSS * abs(ro["loss_sum"])
        gg = gpu.get_grads()
        for k, v in oracle.G.items():
            assert cosine(gg[k], v) >= HALF_COS, (hi, k, cosine(gg[k], v))
        gpu.close()


@pytest.mark.parametrize("precision", ["fp16", "bf16"])
@pytest.mark.parametrize("name", ["post", "lm_pre"])
def test_half_precision_models(precision, name):
    import paper_1904_01038_amd as T
    shape = {"post": ModelShape(2, 2, 128, 2, 256, 512), "lm_pre": ModelShape(0, 2, 128, 2, 256, 512, pre_norm=1)}[name]
    prec = T.FP16 if precision == "fp16" else T.BF16
    scale = 128.0 if precision == "fp16" else 1.0
    gpu, oracle = make_pair(shape, prec, generic=True, init_loss_scale=scale, max_sentences=64, max_len=64, max_tokens=2048)
    if shape.enc_layers:
        batch = make_batches("base", 1, shape=shape, max_tokens=600, lo=5, hi=40)[0]
    else:
        batch = make_batches("lm16", 1, shape=shape, hi=48, max_sentences=6)[0]
    rg, ro = step_both(gpu, oracle, batch)
    assert rg["overflow"] == 0 and ro["overflow"] == 0
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= HALF_LOSS * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert cosine(gg[k], v) >= HALF_COS, (k, cosine(gg[k], v))


def test_padding_invariance_and_determinism():
    import paper_1904_01038_amd as T
    shape = SMALL["post"]
    gpu, _ = make_pair(shape, T.FP32)
    batch = small_batch(shape, 3)
    r1 = gpu.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
    g1 = gpu.get_grads()
    gpu.apply_update(0.0)
    # same batch with extra padding columns of junk-free pad ids: bit-identical
    pad = lambda a: np.concatenate([a, np.full((a.shape[0], 5), shape.pad_id, np.int32)], axis=1)
    r2 = gpu.train_step(pad(batch.src), pad(batch.tgt), batch.src_lens, batch.tgt_lens)
    g2 = gpu.get_grads()
    assert r1["loss_sum"] == r2["loss_sum"]
    for k in g1:
        assert np.array_equal(g1[k], g2[k]), k


def test_bad_arguments_are_rejected_without_side_effects():
    import paper_1904_01038_amd as T
    shape = SMALL["post"]
    gpu, _ = make_pair(shape, T.FP32, max_sentences=4, max_len=8, max_tokens=16)
    before = gpu.get_params()
    b = small_batch(shape, 3)
    bad = b.tgt.copy()
    bad[0, 0] = shape.vocab
    for args in [(b.src, bad, b.src_lens, b.tgt_lens),
                 (b.src, b.tgt, b.src_lens, np.array([9, 1, 1], np.int32)),
                 (b.src, b.tgt, np.array([0, 1, 1], np.int32), b.tgt_lens),
                 (None, b.tgt, None, b.tgt_lens)]:
        with pytest.raises(T.TfmError) as e:
            gpu.train_step(*args)
        assert e.value.code == -1
    with pytest.raises(T.TfmError) as e:
        gpu.apply_update(1e-3)
    assert e.value.code == -4
    after = gpu.get_params()
    assert all(np.array_equal(before[k], after[k]) for k in before)
    big = small_batch(shape, 3)
    with pytest.raises(T.TfmError):     # 3 sentences fit, but not with > max_tokens tokens
        gpu.train_step(np.tile(big.src, (2, 1)), np.tile(big.tgt, (2, 1)), np.tile(big.src_lens, 2), np.tile(big.tgt_lens, 2))


def test_weight_decay_fp32_update_matches_the_oracle():
    import paper_1904_01038_amd as T
    shape = SMALL["post"]
    gpu, oracle = make_pair(shape, T.FP32, weight_decay=0.1, seed=2)
    for it in range(3):
        rg, ro = step_both(gpu, oracle, small_batch(shape, 60 + it))
        check_fp32(gpu, oracle, rg, ro)
        gb = oracle.unscaled_grads()
        gb = {k: v + 0.1 * oracle.p[k] for k, v in gb.items()}      # what the step divides by: gradient plus decay term
        ug, uo = gpu.apply_update(5e-3), oracle.apply_update(5e-3)
        assert abs(ug["grad_norm"] - uo["grad_norm"]) <= 1e-4 * uo["grad_norm"]     # the reported norm excludes the decay term
        check_params_after_update(gpu.get_params(), oracle, gb, 5e-3)
