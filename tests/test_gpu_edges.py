"""Edge cases of the C boundary on the GPU: degenerate batches, capacity limits, determinism of the half-precision
path, clipping, state round trips and the loss-scale floor."""
import numpy as np
import pytest

from synth import ModelShape, Batch, make_batches
from tests.gpu_util import make_pair, step_both, cosine, max_rel
from tests.test_oracle_model import small_batch

pytestmark = pytest.mark.gpu
SHAPE = ModelShape(1, 1, 32, 2, 64, 48)
HSHAPE = ModelShape(1, 2, 128, 2, 256, 512)


def test_single_token_sentences_and_single_sentence_batches():
    import paper_1904_01038_amd as T
    gpu, oracle = make_pair(SHAPE, T.FP32)
    one = Batch(np.array([[2]], np.int32), np.array([[2]], np.int32), np.array([1], np.int32), np.array([1], np.int32))
    rg, ro = step_both(gpu, oracle, one)
    assert rg["ntokens"] == 1 and abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"])
    mixed = Batch(np.array([[5, 2, 1, 1], [7, 8, 9, 2], [2, 1, 1, 1]], np.int32), np.array([[2, 1, 1], [6, 7, 2], [9, 2, 1]], np.int32),
                  np.array([2, 4, 1], np.int32), np.array([1, 3, 2], np.int32))
    rg, ro = step_both(gpu, oracle, mixed)
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert max_rel(gg[k], v) <= 1e-3, k


def test_capacity_is_usable_to_the_last_token_and_sentence():
    import paper_1904_01038_amd as T
    gpu, oracle = make_pair(SHAPE, T.FP32, max_sentences=3, max_len=6, max_tokens=12)
    b = small_batch(SHAPE, 1)                      # 3 sentences, 12 source tokens, 12 target tokens, longest 6
    assert int(b.src_lens.sum()) == 12 and int(b.tgt_lens.sum()) == 12 and max(b.src.shape[1], b.tgt.shape[1]) == 6
    rg, ro = step_both(gpu, oracle, b)
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"])
    with pytest.raises(T.TfmError):                # a fourth sentence does not fit
        gpu.train_step(np.tile(b.src[:1], (4, 1)), np.tile(b.tgt[:1], (4, 1)), np.tile(b.src_lens[:1], 4), np.tile(b.tgt_lens[:1], 4))
    with pytest.raises(T.TfmError):                # no sentences at all
        gpu.train_step(b.src[:0], b.tgt[:0], b.src_lens[:0], b.tgt_lens[:0])


@pytest.mark.parametrize("prec", ["fp16", "bf16"])
def test_half_precision_path_is_bit_reproducible(prec):
    import paper_1904_01038_amd as T
    p = T.FP16 if prec == "fp16" else T.BF16
    batch = make_batches("base", 1, shape=HSHAPE, max_tokens=1500, lo=20, hi=90)[0]      # > 64 tokens: several attention chunks
    runs = []
    for _ in range(2):
        gpu, _ = make_pair(HSHAPE, p, dropout=0.1, init_loss_scale=4.0, max_sentences=64, max_len=96, max_tokens=2048, seed=3)
        r = gpu.train_step(batch.src, batch.tgt, batch.src_lens, batch.tgt_lens)
        g = gpu.get_grads()
        gpu.apply_update(1e-3)
        runs.append((r, g, gpu.get_params()))
        gpu.close()
    assert runs[0][0] == runs[1][0]
    for k in runs[0][1]:
        assert np.array_equal(runs[0][1][k], runs[1][1][k]), k
        assert np.array_equal(runs[0][2][k], runs[1][2][k]), k


def test_long_sentences_cross_attention_chunks_fp16():
    import paper_1904_01038_amd as T
    gpu, oracle = make_pair(HSHAPE, T.FP16, init_loss_scale=8.0, max_sentences=16, max_len=160, max_tokens=2048)
    batch = make_batches("base", 1, shape=HSHAPE, max_tokens=1200, lo=70, hi=150)[0]
    rg, ro = step_both(gpu, oracle, batch)
    assert rg["overflow"] == 0
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-2 * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert cosine(gg[k], v) >= 0.999, (k, cosine(gg[k], v))


def test_gradient_clipping_matches_the_oracle():
    import paper_1904_01038_amd as T
    gpu, oracle = make_pair(SHAPE, T.FP32, clip_norm=0.05)
    b = small_batch(SHAPE, 4)
    step_both(gpu, oracle, b)
    ug, uo = gpu.apply_update(1e-2), oracle.apply_update(1e-2)
    assert uo["grad_norm"] > 0.05                          # the clip is active
    assert abs(ug["grad_norm"] - uo["grad_norm"]) <= 1e-4 * uo["grad_norm"]
    m = gpu.get_adam(0)
    for k, v in oracle.m.items():
        assert max_rel(m[k], v) <= 1e-3, k
    tot = np.sqrt(sum(float((v.astype(np.float64) ** 2).sum()) for v in m.values()))
    assert abs(tot - 0.1 * 0.05) <= 1e-3 * 0.005         # |m| = (1 - beta1) * clip after the first step


def test_state_round_trips_and_loss_scale_floor():
    import paper_1904_01038_amd as T
    gpu, _ = make_pair(SHAPE, T.FP16, init_loss_scale=4.0)
    gpu.set_scaler(2.0 ** -13, 7, 123)
    assert gpu.get_scaler() == dict(loss_scale=2.0 ** -13, clean_steps=7, num_updates=123)
    b = small_batch(SHAPE, 5)
    gpu.debug_set_loss_multiplier(float("inf"))
    assert gpu.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)["overflow"] == 1
    u = gpu.apply_update(1e-3)                             # 2^-13 -> 2^-14: still at the floor, no error
    assert u["skipped"] == 1 and u["loss_scale_after"] == 2.0 ** -14 and u["num_updates"] == 123
    gpu.debug_set_loss_multiplier(float("inf"))
    gpu.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens)
    with pytest.raises(T.TfmError) as e:                   # 2^-15 is below min_loss_scale
        gpu.apply_update(1e-3)
    assert e.value.code == -5
    # Adam moments: set, read back
    gpu2, _ = make_pair(SHAPE, T.FP32)
    L = T.lib()
    import ctypes as C
    i = gpu2.index["dec.0.ffn.w1"]
    a = np.arange(64 * 32, dtype=np.float32) / 1000.0
    assert L.tfm_set_adam(gpu2._h, i, 1, a.ctypes.data_as(C.c_void_p), a.size) == 0
    assert np.array_equal(gpu2.get_adam(1)["dec.0.ffn.w1"].ravel(), a)
    assert not gpu2.get_adam(0)["dec.0.ffn.w1"].any()


def test_side_stream_gives_bit_identical_gradients():
    import paper_1904_01038_amd as T
    batches = make_batches("base", 3, shape=HSHAPE, max_tokens=1500, lo=20, hi=90)
    runs = []
    for on in (True, False):
        gpu, _ = make_pair(HSHAPE, T.FP16, dropout=0.1, init_loss_scale=4.0, max_sentences=64, max_len=96, max_tokens=2048, seed=5)
        gpu.set_overlap(on)
        outs = []
        for b in batches:                               # two accumulated sub-batches, an update, then a third step
            outs.append(gpu.train_step(b.src, b.tgt, b.src_lens, b.tgt_lens, sync=False))
            if len(outs) == 2:
                gpu.apply_update(1e-3, sync=False)
        runs.append((gpu.get_grads(), gpu.get_params()))
        gpu.close()
    for k in runs[0][0]:
        assert np.array_equal(runs[0][0][k], runs[1][0][k]), k
        assert np.array_equal(runs[0][1][k], runs[1][1][k]), k


@pytest.mark.parametrize("prec", ["fp32", "fp16"])
def test_model_width_1536(prec):
    """The larger language model's width: three 512-column chunks per row in the normalisation and embedding kernels,
    24 heads of width 64."""
    import paper_1904_01038_amd as T
    shape = ModelShape(0, 1, 1536, 24, 256, 96, pre_norm=1)
    p = T.FP32 if prec == "fp32" else T.FP16
    gpu, oracle = make_pair(shape, p, dropout=0.1, init_loss_scale=4.0 if prec == "fp16" else 1.0, max_sentences=4, max_len=80,
                            max_tokens=256)
    rng = np.random.default_rng(0)
    lens = np.array([70, 9, 33], np.int32)
    tgt = np.full((3, 70), shape.pad_id, np.int32)
    for i, n in enumerate(lens):
        tgt[i, :n] = rng.integers(4, shape.vocab, n)
    rg, ro = step_both(gpu, oracle, Batch(None, tgt, None, lens))
    assert rg["overflow"] == 0
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= (1e-4 if prec == "fp32" else 1e-2) * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        if prec == "fp32":
            assert max_rel(gg[k], v) <= 1e-3, (k, max_rel(gg[k], v))
        else:
            assert cosine(gg[k], v) >= 0.999, (k, cosine(gg[k], v))
    gpu.close()


@pytest.mark.parametrize("prec", ["fp16", "bf16"])
def test_half_precision_with_head_widths_other_than_64(prec):
    """Head widths 16 and 128 take the generic attention kernels; odd sizes take the generic GEMM."""
    import paper_1904_01038_amd as T
    p = T.FP16 if prec == "fp16" else T.BF16
    for shape in (ModelShape(1, 1, 64, 4, 136, 88), ModelShape(1, 1, 256, 2, 64, 72, pre_norm=1)):
        gpu, oracle = make_pair(shape, p, dropout=0.1, init_loss_scale=4.0, max_sentences=8, max_len=40, max_tokens=256)
        batch = make_batches("base", 1, shape=shape, max_tokens=200, lo=5, hi=38)[0]
        rg, ro = step_both(gpu, oracle, batch)
        assert rg["overflow"] == 0
        assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-2 * abs(ro["loss_sum"])
        gg = gpu.get_grads()
        for k, v in oracle.G.items():
            assert cosine(gg[k], v) >= 0.999, (shape, k, cosine(gg[k], v))
        gpu.close()


def test_more_weight_gradients_than_one_grouped_launch_holds():
    """A deep, narrow encoder-decoder has more weight gradients per backward pass (4 per encoder layer, 7 per decoder
    layer, 1 for the vocabulary) than the 48 products one grouped launch takes: the queue must flush on its own in the
    middle of the decoder and again later, and every gradient must still match the oracle.  (fp16 only: through 14 layers
    bf16's 8-bit mantissa alone takes the first layers' gradients to a cosine of 0.9989.)"""
    import paper_1904_01038_amd as T
    p = T.FP16
    shape = ModelShape(5, 9, 64, 1, 128, 96)                 # 20 + 63 + 1 = 84 products; head width 64
    gpu, oracle = make_pair(shape, p, dropout=0.1, init_loss_scale=4.0, max_sentences=8, max_len=40, max_tokens=256)
    batch = make_batches("base", 1, shape=shape, max_tokens=200, lo=5, hi=38)[0]
    rg, ro = step_both(gpu, oracle, batch)
    assert rg["overflow"] == 0
    assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-2 * abs(ro["loss_sum"])
    gg = gpu.get_grads()
    for k, v in oracle.G.items():
        assert cosine(gg[k], v) >= 0.999, (k, cosine(gg[k], v))
    gpu.close()
