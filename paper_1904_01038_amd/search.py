"""A plain beam search over a step-wise predictor (host bookkeeping only; the model runs behind `step`).

The library's part of inference is the decoding step with cached states; which hypotheses continue is the caller's
business.  This driver is what the benchmark and the tests use: it works on any `step(prev, parent) -> (top_logp,
top_id)` with `top_logp`/`top_id` of shape [sentences * beam, k], k >= 2 * beam, best first.
"""
import numpy as np


def beam_search(step, n_sentences, beam, max_steps, eos_id, len_penalty=0.6):
    """Returns, per sentence, a list of (score, tokens) sorted best first; score = sum of log-probabilities divided
    by len(tokens) ** len_penalty.  A hypothesis ends with eos or is cut after max_steps tokens."""
    rows = n_sentences * beam
    prev = np.full(rows, eos_id, dtype=np.int32)
    parent = np.arange(rows, dtype=np.int32)
    score = np.full(rows, -np.inf)
    score[::beam] = 0.0                                  # at the first step only slot 0 of a sentence is alive
    tokens = [[] for _ in range(rows)]
    finished = [[] for _ in range(n_sentences)]
    for t in range(max_steps):
        top_logp, top_id = step(prev, parent if t else None)
        k = top_logp.shape[1]
        new_tokens = [None] * rows
        last = t == max_steps - 1
        for s in range(n_sentences):
            base = s * beam
            if len(finished[s]) >= beam:                 # done: keep its rows fed so that shapes stay fixed
                for j in range(beam):
                    prev[base + j], parent[base + j], new_tokens[base + j] = eos_id, base + j, tokens[base + j]
                continue
            cand = []
            for j in range(beam):
                if score[base + j] == -np.inf:
                    continue
                for c in range(k):
                    cand.append((score[base + j] + float(top_logp[base + j, c]), base + j, int(top_id[base + j, c])))
            cand.sort(key=lambda x: (-x[0], x[1], x[2]))
            slot = 0
            new_score = np.full(beam, -np.inf)
            for sc, row, tok in cand:
                seq = tokens[row] + [tok]
                if tok == eos_id or last:
                    if len(finished[s]) < beam:
                        finished[s].append((sc / len(seq) ** len_penalty, seq))
                    continue
                if slot < beam:
                    prev[base + slot], parent[base + slot], new_tokens[base + slot] = tok, row, seq
                    new_score[slot] = sc
                    slot += 1
                if slot == beam:
                    break
            for j in range(slot, beam):                  # unused slots repeat slot 0's history and stay dead
                prev[base + j], parent[base + j], new_tokens[base + j] = eos_id, base + j, tokens[base + j]
            score[base:base + beam] = new_score
        tokens = new_tokens
        if all(len(f) >= beam for f in finished):
            break
    return [sorted(f, key=lambda x: -x[0]) for f in finished]
