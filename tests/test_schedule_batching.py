"""Learning-rate schedule, batching and epoch shuffle: the oracle against what the text and arithmetic fix, then the
library's host code against the oracle, bit for bit.  No GPU."""
import math
import os
from collections import Counter

import numpy as np
import pytest

from oracle.schedule_batching import lr_inverse_sqrt, lr_cosine_restarts, batch_by_length, shuffle_batches, _finalise

HERE = os.path.dirname(os.path.abspath(__file__))


# ---- oracle pins ---------------------------------------------------------------------------------------------------------
def test_lr_is_the_cited_schedule():
    # lr = d^-1/2 * min(t^-1/2, t * w^-3/2)
    for d, w in [(512, 4000), (1024, 4000), (1024, 16000)]:
        peak = (d * w) ** -0.5
        for t in [1, 2, 10, w - 1, w, w + 1, 3 * w, 100 * w]:
            want = d ** -0.5 * min(t ** -0.5, t * w ** -1.5)
            assert math.isclose(lr_inverse_sqrt(t, w, peak), want, rel_tol=1e-12), (d, w, t)


def test_lr_shape():
    w, peak, init = 4000, 1e-3, 1e-7
    assert lr_inverse_sqrt(w, w, peak, init) == peak                      # the peak is reached at the end of warm-up
    assert math.isclose(lr_inverse_sqrt(4 * w, w, peak, init), peak / 2, rel_tol=1e-15)
    assert math.isclose(lr_inverse_sqrt(w // 2, w, peak, init), (peak + init) / 2, rel_tol=1e-12)
    assert lr_inverse_sqrt(0, w, peak, init) == init
    up = [lr_inverse_sqrt(t, w, peak, init) for t in range(0, w + 1, 100)]
    down = [lr_inverse_sqrt(t, w, peak, init) for t in range(w, 20 * w, 500)]
    assert all(a < b for a, b in zip(up, up[1:])) and all(a > b for a, b in zip(down, down[1:]))
    assert math.isnan(lr_inverse_sqrt(-1, w, peak)) and math.isnan(lr_inverse_sqrt(1, -1, peak))
    assert lr_inverse_sqrt(9, 0, 3.0) == 1.0 and lr_inverse_sqrt(0, 0, 3.0) == 3.0


def test_cosine_restarts_is_the_cited_schedule():
    """eta_t = eta_min + (eta_max - eta_min) (1 + cos(pi T_cur / T_i)) / 2 with T_cur = 0 at a (re)start: checked on values
    the formula fixes by hand, on periodicity, monotonicity inside a cycle, doubling periods and shrinking maxima."""
    mx, mn, T0 = 1e-3, 1e-5, 100
    f = lambda t, **kw: lr_cosine_restarts(t, 0, mx, mn, T0, **kw)
    assert f(1) == mx                                              # T_cur = 0: the maximum
    assert math.isclose(f(1 + T0 // 2), (mx + mn) / 2, rel_tol=1e-12)      # half-way: the mean of the two
    assert math.isclose(f(1 + T0 // 4), mn + (mx - mn) * (1 + math.sqrt(0.5)) / 2, rel_tol=1e-12)   # cos(pi/4)
    assert f(T0) > mn and math.isclose(f(T0), mn + (mx - mn) * (1 + math.cos(math.pi * 0.99)) / 2, rel_tol=1e-9)
    assert f(T0 + 1) == mx                                         # warm restart
    for t in range(1, 3 * T0):                                     # fixed period: periodic, decreasing inside a cycle
        assert math.isclose(f(t), f(t + T0), rel_tol=1e-12)
        if t % T0:
            assert f(t + 1) < f(t)
    # periods 100, 200, 400 with maxima 1, 1/2, 1/4: restarts at updates 1, 101, 301, 701
    g = lambda t: lr_cosine_restarts(t, 0, mx, mn, T0, 2.0, 0.5)
    for start, i in [(1, 0), (101, 1), (301, 2), (701, 3)]:
        assert g(start) == mx * 0.5 ** i, (start, g(start))
        assert g(start - 1) < g(start) or start == 1
        half = start + (T0 * 2 ** i) // 2
        assert math.isclose(g(half), (mx * 0.5 ** i + mn) / 2, rel_tol=1e-12)
    # warm-up first: linear to the maximum, the first cycle begins right after it
    h = lambda t: lr_cosine_restarts(t, 50, mx, mn, T0, 1.0, 1.0, 1e-7)
    assert h(0) == 1e-7 and h(50) == mx and math.isclose(h(25), (mx + 1e-7) / 2, rel_tol=1e-12)
    assert h(51) == mx and math.isclose(h(51 + T0 // 2), (mx + mn) / 2, rel_tol=1e-12) and h(151) == mx
    # a period that is not an integer number of updates
    k = lambda t: lr_cosine_restarts(t, 0, 1.0, 0.0, 2.5, 1.5)
    assert k(1) == 1.0 and math.isclose(k(2), (1 + math.cos(math.pi / 2.5)) / 2) and math.isclose(k(4), (1 + math.cos(math.pi * 0.5 / 3.75)) / 2)
    assert all(math.isnan(x) for x in (lr_cosine_restarts(-1, 0, mx, mn, T0), lr_cosine_restarts(1, -1, mx, mn, T0),
                                       lr_cosine_restarts(1, 0, mx, mn, 0), lr_cosine_restarts(1, 0, mx, mn, T0, 0.5)))


def read_example():
    ex = {"expect": {}}
    for line in open(os.path.join(HERE, "golden", "batching_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, rest = line.split(None, 1)
        if key == "multiple":
            m, spec = rest.split(":")
            ex["expect"][int(m)] = [[int(x) for x in part.split()] for part in spec.split("|")]
        elif key in ("src_lens", "tgt_lens"):
            ex[key] = [int(x) for x in rest.split()]
        else:
            ex[key] = int(rest)
    return ex


def test_batching_hand_worked_example():
    ex = read_example()
    for multiple, want in ex["expect"].items():
        assert batch_by_length(ex["src_lens"], ex["tgt_lens"], ex["max_tokens"], ex["max_sentences"], multiple) == want


def random_lengths(seed, n, lo, hi, lm=False):
    rng = np.random.default_rng(seed)
    src = rng.integers(lo, hi + 1, n)
    tgt = np.clip(src + rng.integers(-3, 4, n), lo, hi)
    return (None if lm else src.tolist()), tgt.tolist()


@pytest.mark.parametrize("seed,n,cap,max_sent,multiple", [(0, 500, 400, 64, 1), (1, 800, 3584, 1024, 8), (2, 300, 120, 7, 2),
                                                          (3, 1, 50, 4, 8), (4, 257, 80, 1, 1)])
def test_batching_invariants(seed, n, cap, max_sent, multiple):
    src, tgt = random_lengths(seed, n, 1, min(80, cap), lm=seed == 2)
    length = [max(s, t) for s, t in zip(src, tgt)] if src else tgt
    batches = batch_by_length(src, tgt, cap, max_sent, multiple)
    flat = [i for b in batches for i in b]
    assert sorted(flat) == list(range(n))                                  # every sentence exactly once
    assert [length[i] for i in flat] == sorted(length)                     # similar lengths are neighbours
    for k, b in enumerate(batches):
        assert 1 <= len(b) <= max_sent
        assert len(b) * max(length[i] for i in b) <= cap                   # padded token count under the cap
        if k + 1 < len(batches):
            nxt = batches[k + 1][0]
            if multiple == 1:                                              # greedy: the next sentence did not fit
                assert (len(b) + 1) * length[nxt] > cap or len(b) == max_sent
            elif len(b) >= multiple:
                assert len(b) % multiple == 0
    # the content of the batches is a function of the lengths alone
    assert batch_by_length(src, tgt, cap, max_sent, multiple) == batches


def test_batching_rejects_bad_lengths():
    with pytest.raises(ValueError):
        batch_by_length([3, 0], [3, 2], 10, 4)
    with pytest.raises(ValueError):
        batch_by_length(None, [3, 11], 10, 4)
    assert batch_by_length(None, [], 10, 4) == []


def test_shuffle_is_a_seeded_uniform_permutation():
    assert _finalise(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF              # first output of splitmix64 seeded with 0
    for n in (0, 1, 2, 17, 1000):
        p = shuffle_batches(n, 5, 3)
        assert sorted(p) == list(range(n))
        assert p == shuffle_batches(n, 5, 3)
    assert shuffle_batches(1000, 5, 3) != shuffle_batches(1000, 5, 4) != shuffle_batches(1000, 6, 4)
    counts = Counter(tuple(shuffle_batches(4, 11, e)) for e in range(24000))
    assert len(counts) == 24
    chi2 = sum((c - 1000.0) ** 2 / 1000.0 for c in counts.values())
    assert chi2 < 60.0                                                     # 23 degrees of freedom: P(chi2 > 60) ~ 3e-5
    first = Counter(shuffle_batches(50, 1, e)[0] for e in range(20000))
    assert len(first) == 50 and max(first.values()) < 520 and min(first.values()) > 290


# ---- the library's host code against the oracle ---------------------------------------------------------------------
@pytest.fixture(scope="module")
def T():
    import paper_1904_01038_amd as T
    if not os.path.exists(T.lib_path()):
        from paper_1904_01038_amd import build
        build.build(verbose=False)
    return T


def test_library_lr_matches(T):
    for w, peak, init in [(4000, 1e-3, 1e-7), (16000, 7e-4, 0.0), (0, 0.5, 0.0), (1, 1.0, 0.25)]:
        for t in [0, 1, 2, 3, 999, 4000, 4001, 16000, 10 ** 6, 10 ** 12]:
            assert T.lr_inverse_sqrt(t, w, peak, init) == lr_inverse_sqrt(t, w, peak, init), (w, t)
    assert math.isnan(T.lr_inverse_sqrt(-1, 10, 1.0)) and math.isnan(T.lr_inverse_sqrt(1, -2, 1.0))


def test_library_cosine_restarts_matches(T):
    """The library inverts the geometric sum of the cycle lengths in closed form; the oracle walks the cycles."""
    cases = [(0, 1e-3, 1e-5, 100, 1.0, 1.0, 0.0), (50, 1e-3, 1e-5, 100, 2.0, 0.5, 1e-7), (10, 2e-3, 0.0, 37.5, 1.3, 0.9, 1e-4),
             (0, 1.0, 0.1, 1, 1.0, 1.0, 0.0), (4000, 7e-4, 1e-9, 25000, 1.0, 0.75, 1e-7)]
    for (w, mx, mn, per, tm, sh, init) in cases:
        ts = list(range(0, 400)) + [1000, 4001, 29000, 29001, 54001, 10 ** 6, 10 ** 7 + 3]
        for t in ts:
            a, b = T.lr_cosine_restarts(t, w, mx, mn, per, tm, sh, init), lr_cosine_restarts(t, w, mx, mn, per, tm, sh, init)
            assert math.isclose(a, b, rel_tol=1e-9, abs_tol=1e-15), (w, per, tm, t, a, b)
    assert math.isnan(T.lr_cosine_restarts(-1, 0, 1.0, 0.0, 10)) and math.isnan(T.lr_cosine_restarts(1, 0, 1.0, 0.0, 10, 0.9))


def test_library_batching_matches(T):
    ex = read_example()
    for multiple, want in ex["expect"].items():
        got = T.batch_by_length(ex["src_lens"], ex["tgt_lens"], ex["max_tokens"], ex["max_sentences"], multiple)
        assert [b.tolist() for b in got] == want
    cases = [(0, 500, 400, 64, 1, 80), (1, 20000, 3584, 1024, 8, 120), (2, 300, 120, 7, 2, 60), (3, 1, 50, 4, 8, 50),
             (4, 257, 80, 1, 1, 80), (5, 4000, 4096, 100000, 1, 50), (6, 3000, 64, 9, 4, 64), (7, 999, 512, 33, 16, 1)]
    for seed, n, cap, max_sent, multiple, hi in cases:
        src, tgt = random_lengths(seed, n, 1, hi, lm=seed % 3 == 2)
        want = batch_by_length(src, tgt, cap, max_sent, multiple)
        got = T.batch_by_length(src, tgt, cap, max_sent, multiple)
        assert [b.tolist() for b in got] == want, (seed, n)
    assert T.batch_by_length(None, [], 10, 4) == []
    for bad in [([3, 0], [3, 2]), (None, [3, 11]), (None, [0])]:
        with pytest.raises(T.TfmError):
            T.batch_by_length(bad[0], bad[1], 10, 4)
    with pytest.raises(T.TfmError):
        T.batch_by_length(None, [1], 0, 4)


def test_library_shuffle_matches(T):
    for n, seed, epoch in [(0, 1, 1), (1, 1, 1), (2, 0, 0), (17, 5, 3), (1000, 2 ** 63 + 12345, 7), (4096, 9, 2 ** 31 + 5)]:
        assert T.shuffle_batches(n, seed, epoch).tolist() == shuffle_batches(n, seed, epoch)
