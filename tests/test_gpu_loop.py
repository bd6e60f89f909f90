"""A short training run assembled from the library's pieces (batching, epoch shuffle, learning-rate schedule,
accumulated training steps, update) against the same run assembled from the oracle's pieces."""
import numpy as np
import pytest

from oracle.schedule_batching import batch_by_length, lr_inverse_sqrt, shuffle_batches
from synth import ModelShape
from synth.batches import zipf_ids
from tests.gpu_util import make_pair, max_rel

pytestmark = pytest.mark.gpu
SHAPE = ModelShape(1, 1, 32, 2, 64, 48)


def pool(seed, n, lo, hi):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        m = int(rng.integers(lo, hi + 1))
        k = int(np.clip(m + rng.integers(-2, 3), lo, hi))
        out.append((np.append(zipf_ids(rng, m - 1, SHAPE.vocab), SHAPE.eos_id).astype(np.int32),
                    np.append(zipf_ids(rng, k - 1, SHAPE.vocab), SHAPE.eos_id).astype(np.int32)))
    return out


def collate(sents, idx):
    def pad(rows):
        out = np.full((len(rows), max(len(r) for r in rows)), SHAPE.pad_id, np.int32)
        for i, r in enumerate(rows):
            out[i, :len(r)] = r
        return out
    s, t = [sents[i][0] for i in idx], [sents[i][1] for i in idx]
    return pad(s), pad(t), np.array([len(r) for r in s], np.int32), np.array([len(r) for r in t], np.int32)


def test_two_epochs_with_accumulation_match_the_oracle():
    import paper_1904_01038_amd as T
    sents = pool(0, 60, 2, 12)
    src_lens, tgt_lens = [len(s) for s, _ in sents], [len(t) for _, t in sents]
    cap, max_sent, warmup, peak, freq = 48, 6, 4, 5e-3, 2
    gpu, oracle = make_pair(SHAPE, T.FP32, dropout=0.1, max_sentences=max_sent, max_len=12, max_tokens=cap, clip_norm=1.0)
    lib_batches = T.batch_by_length(src_lens, tgt_lens, cap, max_sent, 2)
    ora_batches = batch_by_length(src_lens, tgt_lens, cap, max_sent, 2)
    assert [b.tolist() for b in lib_batches] == ora_batches and len(ora_batches) >= 10
    update = 0
    for epoch in range(2):
        lib_perm = T.shuffle_batches(len(lib_batches), 7, epoch)
        ora_perm = shuffle_batches(len(ora_batches), 7, epoch)
        assert lib_perm.tolist() == ora_perm
        for k in range(0, len(ora_perm) - freq + 1, freq):
            for j in range(freq):
                rg = gpu.train_step(*collate(sents, lib_batches[lib_perm[k + j]]))
                ro = oracle.train_step(*collate(sents, ora_batches[ora_perm[k + j]]))
                assert abs(rg["loss_sum"] - ro["loss_sum"]) <= 1e-4 * abs(ro["loss_sum"]), (epoch, k, j)
            update += 1
            ug = gpu.apply_update(T.lr_inverse_sqrt(update, warmup, peak, 0.0))
            uo = oracle.apply_update(lr_inverse_sqrt(update, warmup, peak, 0.0))
            assert abs(ug["grad_norm"] - uo["grad_norm"]) <= 1e-3 * uo["grad_norm"]
    assert update >= 10
    pg = gpu.get_params()
    start = make_pair(SHAPE, T.FP32)[1].p
    for name, v in oracle.p.items():
        moved = float(np.max(np.abs(v - start[name])))
        assert moved > 0.0
        keep = np.ones(v.shape, bool)
        # A bias added to every key shifts all scores of a softmax row alike: its true gradient is zero, what both
        # sides hold there is rounding noise, and Adam turns the sign of that noise into full-size steps.
        d = SHAPE.d_model
        if name.endswith(".bqkv"):
            keep[d:2 * d] = False
        if name.endswith(".bkv"):
            keep[:d] = False
        # the run moved every tensor; the two runs agree to a small fraction of that movement
        assert float(np.max(np.abs(pg[name] - v)[keep])) <= 2e-2 * moved + 1e-7, name
