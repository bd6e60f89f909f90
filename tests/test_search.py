"""The beam-search driver (host bookkeeping used by the benchmark and the decoding tests) on a toy predictor: with a
beam wide enough to keep every prefix alive it must return the exhaustive optimum."""
import itertools

import numpy as np

from tests.beam_search import beam_search


def test_wide_beam_is_exhaustive():
    V, eos, steps = 4, 2, 3
    for seed in range(5):
        rng = np.random.default_rng(seed)
        table = np.log(rng.dirichlet(np.ones(V), size=V))          # first-order model: logp(next | prev)

        def step(prev, parent):
            lp = table[prev]
            ids = np.argsort(-lp, axis=1, kind="stable")
            return np.take_along_axis(lp, ids, 1).astype(np.float32), ids.astype(np.int32)

        for lenpen in (0.0, 0.6):
            got = beam_search(step, 2, 16, steps, eos, len_penalty=lenpen)
            best = []
            for n in range(1, steps + 1):
                for seq in itertools.product(range(V), repeat=n):
                    if eos in seq[:-1] or (seq[-1] != eos and n < steps):
                        continue
                    p, s = eos, 0.0
                    for tok in seq:
                        s += float(np.float32(table[p, tok]))
                        p = tok
                    best.append((s / n ** lenpen, list(seq)))
            best.sort(key=lambda x: -x[0])
            for s in range(2):
                assert got[s][0][1] == best[0][1]
                assert abs(got[s][0][0] - best[0][0]) < 1e-6
                assert len(got[s]) == 16 and all(a[0] >= b[0] for a, b in zip(got[s], got[s][1:]))
