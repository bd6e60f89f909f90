// Host-side steps on either side of the training step: the learning-rate schedule, token-capped batching of
// sentences of similar length and the per-epoch shuffle of the batch order (Components, Learning Rate Schedulers;
// Implementation, Batching).  No device code.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/tfm.h"

namespace {

inline uint64_t finalise64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

}  // namespace

extern "C" {

double tfm_lr_inverse_sqrt(int64_t t, int64_t warmup, double peak_lr, double init_lr) {
  if (t < 0 || warmup < 0) return std::numeric_limits<double>::quiet_NaN();
  if (warmup == 0) return peak_lr / std::sqrt((double)std::max<int64_t>(t, 1));
  if (t <= warmup) return init_lr + (peak_lr - init_lr) * ((double)t / (double)warmup);
  return peak_lr * std::sqrt((double)warmup / (double)t);
}

double tfm_lr_cosine_restarts(int64_t t, int64_t warmup, double max_lr, double min_lr, double period, double t_mult, double shrink,
                              double init_lr) {
  const double nan = std::numeric_limits<double>::quiet_NaN();
  if (t < 0 || warmup < 0 || !(period > 0.0) || !(t_mult >= 1.0)) return nan;
  if (t <= warmup) return warmup == 0 ? max_lr : init_lr + (max_lr - init_lr) * ((double)t / (double)warmup);
  const double u = (double)(t - warmup - 1);             // updates since the first cycle began
  double cycle, start, length;
  if (t_mult == 1.0) {
    cycle = std::floor(u / period);
    start = cycle * period;
    length = period;
  } else {
    // cycles end at period * (t_mult^(i+1) - 1) / (t_mult - 1): invert the geometric sum, then settle rounding at the edges
    cycle = std::floor(std::log1p(u * (t_mult - 1.0) / period) / std::log(t_mult));
    auto begin_of = [&](double i) { return period * (std::pow(t_mult, i) - 1.0) / (t_mult - 1.0); };
    while (cycle > 0 && begin_of(cycle) > u) cycle -= 1.0;
    while (begin_of(cycle + 1.0) <= u) cycle += 1.0;
    start = begin_of(cycle);
    length = period * std::pow(t_mult, cycle);
  }
  const double top = max_lr * std::pow(shrink, cycle);
  const double pi = 3.14159265358979323846;
  return min_lr + 0.5 * (top - min_lr) * (1.0 + std::cos(pi * (u - start) / length));
}

int tfm_batch_by_length(const int32_t* src_lens, const int32_t* tgt_lens, int64_t n, int32_t max_tokens,
                        int32_t max_sentences, int32_t multiple, int64_t* order, int64_t* batch_begin,
                        int64_t* n_batches) {
  if (!tgt_lens || !order || !batch_begin || !n_batches || n < 0 || max_tokens < 1 || max_sentences < 1 || multiple < 1)
    return TFM_EINVAL;
  std::vector<int32_t> len((size_t)n);
  for (int64_t i = 0; i < n; ++i) {
    const int32_t s = src_lens ? src_lens[i] : 1, t = tgt_lens[i];
    if (s < 1 || t < 1 || s > max_tokens || t > max_tokens) return TFM_EINVAL;
    len[(size_t)i] = std::max(src_lens ? s : 0, t);
  }
  {
    // stable counting sort by length (1 .. max_tokens): ties keep index order
    std::vector<int64_t> start((size_t)max_tokens + 2, 0);
    for (int64_t i = 0; i < n; ++i) ++start[(size_t)len[(size_t)i] + 1];
    for (size_t l = 1; l < start.size(); ++l) start[l] += start[l - 1];
    for (int64_t i = 0; i < n; ++i) order[start[(size_t)len[(size_t)i]]++] = i;
  }
  int64_t nb = 0, begin = 0;          // the open batch is order[begin .. pos)
  batch_begin[0] = 0;
  int64_t pos = 0;
  int32_t longest = 0;
  while (pos < n || begin < pos) {
    bool close = pos == n;
    if (!close) {
      const int32_t L = std::max(longest, len[(size_t)order[pos]]);      // sorted: the candidate is the longest
      const int64_t count = pos - begin;
      if (count > 0 && ((count + 1) * (int64_t)L > max_tokens || count >= max_sentences)) close = true;
      else { longest = L; ++pos; }
    }
    if (close) {
      int64_t count = pos - begin;
      if (multiple > 1 && count >= multiple && pos < n) count = count / multiple * multiple;   // the rest opens the next batch
      begin += count;
      batch_begin[++nb] = begin;
      pos = std::max(pos, begin);
      longest = 0;
      for (int64_t i = begin; i < pos; ++i) longest = std::max(longest, len[(size_t)order[i]]);
    }
  }
  *n_batches = nb;
  return TFM_OK;
}

int tfm_shuffle_batches(int64_t n_batches, uint64_t seed, uint64_t epoch, int64_t* perm) {
  if (n_batches < 0 || !perm || n_batches > ((int64_t)1 << 32)) return TFM_EINVAL;
  for (int64_t i = 0; i < n_batches; ++i) perm[i] = i;
  for (int64_t i = n_batches - 1; i >= 1; --i) {
    const uint64_t r = finalise64(seed + 0x9E3779B97F4A7C15ull * ((epoch << 32) + (uint64_t)i + 1));
    std::swap(perm[i], perm[(int64_t)(r % (uint64_t)(i + 1))]);
  }
  return TFM_OK;
}

}  // extern "C"
