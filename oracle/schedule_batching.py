"""Oracle for the steps on either side of the training step: learning-rate schedule, batching, epoch shuffle.

TEST INFRASTRUCTURE ONLY: plain Python, written from the paper; only tests/, the smoke check and the bench's CPU
baseline may import it.  It shares no code with the HIP/C++ library.

  lr_inverse_sqrt   Components, Learning Rate Schedulers: the inverse square-root schedule of the Transformer paper the
                    text cites, lr = d^-1/2 * min(t^-1/2, t * w^-3/2), generalised to a peak rate and a start rate.
  lr_cosine_restarts  Components, Learning Rate Schedulers: the cyclical schedule "based on warm restarts" of the work
                    the text cites: inside cycle i, lr = min + (max_i - min) (1 + cos(pi T_cur / T_i)) / 2.
  batch_by_length   Implementation, Batching: mini-batches group sentences of similar length, hold up to a given
                    number of tokens and keep their content from epoch to epoch.
  shuffle_batches   Implementation, Batching: the batches themselves are visited in a new random order every epoch.

The paper fixes none of the details (sort key, what the token cap counts, the random generator); the readings taken
here are the ones the library documents in its header.
"""
import math

MASK = (1 << 64) - 1


def lr_inverse_sqrt(t, warmup, peak_lr, init_lr=0.0):
    if t < 0 or warmup < 0:
        return math.nan
    if warmup == 0:
        return peak_lr / math.sqrt(max(t, 1))
    if t <= warmup:
        return init_lr + (peak_lr - init_lr) * (t / warmup)
    return peak_lr * math.sqrt(warmup / t)


def lr_cosine_restarts(t, warmup, max_lr, min_lr, period, t_mult=1.0, shrink=1.0, init_lr=0.0):
    """Update t = 1, 2, ...: linear warm-up from init_lr to max_lr over `warmup` updates, then cosine cycles with warm
    restarts.  Cycle i = 0, 1, ... lasts T_i = period * t_mult^i updates (a real number when t_mult is not an integer)
    and starts at max_i = max_lr * shrink^i; T_cur counts the updates since the cycle began, so the first update after
    the warm-up (and after every restart) runs at max_i."""
    if t < 0 or warmup < 0 or period <= 0 or t_mult < 1.0:
        return math.nan
    if t <= warmup:
        return max_lr if warmup == 0 else init_lr + (max_lr - init_lr) * (t / warmup)
    t_cur = float(t - warmup - 1)                     # 0 at the first update of the first cycle
    i, length = 0, float(period)
    while t_cur >= length:                            # walk the cycles one by one
        t_cur -= length
        length *= t_mult
        i += 1
    top = max_lr * shrink ** i
    return min_lr + 0.5 * (top - min_lr) * (1.0 + math.cos(math.pi * t_cur / length))


def batch_by_length(src_lens, tgt_lens, max_tokens, max_sentences, multiple=1):
    """Returns a list of batches, each a list of sentence indices."""
    n = len(tgt_lens)
    length = [max(src_lens[i], tgt_lens[i]) if src_lens is not None else tgt_lens[i] for i in range(n)]
    for i in range(n):
        lo = min(src_lens[i], tgt_lens[i]) if src_lens is not None else tgt_lens[i]
        if lo < 1 or length[i] > max_tokens:
            raise ValueError("sentence %d has a length outside [1, max_tokens]" % i)
    queue = sorted(range(n), key=lambda i: (length[i], i))      # similar lengths next to each other
    batches = []
    current = []
    while queue:
        i = queue[0]
        grown = current + [i]
        padded = len(grown) * max(length[j] for j in grown)      # tokens of the padded batch if i joined
        if current and (padded > max_tokens or len(current) >= max_sentences):
            keep = len(current)
            if multiple > 1 and keep >= multiple:
                keep -= keep % multiple
            batches.append(current[:keep])
            current = current[keep:]                            # the remainder opens the next batch
            continue
        current = grown
        queue.pop(0)
    if current:
        batches.append(current)
    return batches


def _finalise(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def shuffle_batches(n_batches, seed, epoch):
    perm = list(range(n_batches))
    for i in range(n_batches - 1, 0, -1):
        r = _finalise((seed + 0x9E3779B97F4A7C15 * ((epoch << 32) + i + 1)) & MASK)
        j = r % (i + 1)
        perm[i], perm[j] = perm[j], perm[i]
    return perm
