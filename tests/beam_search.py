"""A plain beam search over a step-wise predictor (host bookkeeping only; the model runs behind `step`).

The library's part of inference is the decoding step with cached states; which hypotheses continue is the caller's
business.  This driver is what the benchmark and the tests use: it works on any `step(prev, parent) -> (top_logp,
top_id)` with `top_logp`/`top_id` of shape [sentences * beam, k], k >= 2 * beam, best first.
"""
import numpy as np


def beam_search(step, n_sentences, beam, max_steps, eos_id, len_penalty=0.6):
    """Returns, per sentence, a list of (score, tokens) sorted best first; score = sum of log-probabilities divided
    by len(tokens) ** len_penalty.  A hypothesis ends with eos or is cut after max_steps tokens.

    Per step and sentence the beam * k candidates (row score + token log-probability) are ranked, ties by (row,
    rank within the row); walking down the ranking, eos candidates become finished hypotheses and the others fill
    the `beam` slots of the next step; candidates after the slots are full are dropped.  A sentence stops once it
    has `beam` finished hypotheses (its rows are then fed eos so that shapes stay fixed)."""
    B, rows = n_sentences, n_sentences * beam
    prev = np.full(rows, eos_id, dtype=np.int32)
    parent = np.arange(rows, dtype=np.int32)
    score = np.full((B, beam), -np.inf)
    score[:, 0] = 0.0                                    # at the first step only slot 0 of a sentence is alive
    tokens = np.zeros((rows, max_steps), dtype=np.int32)
    finished = [[] for _ in range(B)]
    n_finished = np.zeros(B, dtype=np.int64)
    base = (np.arange(B) * beam)[:, None]
    for t in range(max_steps):
        top_logp, top_id = step(prev, parent if t else None)
        k = top_logp.shape[1]
        last = t == max_steps - 1
        cand = (score[:, :, None] + top_logp.reshape(B, beam, k).astype(np.float64)).reshape(B, beam * k)
        order = np.argsort(-cand, axis=1, kind="stable")[:, :2 * beam]          # stable: ties by (row, rank)
        c_score = np.take_along_axis(cand, order, axis=1)
        c_slot = order // k                                                       # beam slot the candidate extends
        c_tok = np.take_along_axis(top_id.reshape(B, beam * k), order, axis=1)
        alive = np.isfinite(c_score) & (n_finished < beam)[:, None]
        ends = alive & ((c_tok == eos_id) | last)
        goes_on = alive & ~ends
        rank = np.cumsum(goes_on, axis=1) - 1                                     # slot of a continuing candidate
        goes_on &= rank < beam
        before = np.cumsum(goes_on, axis=1) - goes_on                             # continuing candidates ranked above
        ends &= before < beam
        for s, j in zip(*np.nonzero(ends)):                                       # rare: hypotheses that end here
            if len(finished[s]) < beam:
                seq = tokens[base[s, 0] + c_slot[s, j], :t].tolist() + [int(c_tok[s, j])]
                finished[s].append((float(c_score[s, j]) / len(seq) ** len_penalty, seq))
        n_finished = np.array([len(f) for f in finished])
        # next step's rows: slot r of sentence s <- the continuing candidate of rank r (or a dead filler)
        new_prev = np.full((B, beam), eos_id, dtype=np.int32)
        new_parent = base + np.arange(beam)[None, :]
        new_score = np.full((B, beam), -np.inf)
        ss, jj = np.nonzero(goes_on)
        rr = rank[ss, jj]
        new_prev[ss, rr] = c_tok[ss, jj]
        new_parent[ss, rr] = base[ss, 0] + c_slot[ss, jj]
        new_score[ss, rr] = c_score[ss, jj]
        new_parent = new_parent.reshape(-1).astype(np.int32)
        tokens = tokens[new_parent]
        tokens[:, t] = new_prev.reshape(-1)
        prev, parent, score = new_prev.reshape(-1), new_parent, new_score
        if np.all(n_finished >= beam):
            break
    return [sorted(f, key=lambda x: -x[0]) for f in finished]
