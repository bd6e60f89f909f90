// Shape-agnostic multi-head attention forward/backward on the vector ALUs, fp32 arithmetic.  It serves the fp32
// precision mode and head widths the MFMA kernels do not take.  One block per (sentence, head, query row) in the
// forward and dQ passes and per (sentence, head, key row) in the dK/dV pass; no atomics.
#include "common.h"
#include "kernels.h"

namespace tfm {

constexpr int AN_THREADS = 128;

// Dropout on the attention weights (thr = 0: off): weight (packed query row, head h, key j) uses element
// ((row * H + h) << 16) + j of the counter-based generator.
struct AttnDrop { uint64_t key; uint32_t thr; float inv_keep; int H; };
__device__ __forceinline__ bool attn_keep(const AttnDrop& d, int qrow, int h, int j) {
  const uint64_t e = (((uint64_t)qrow * (uint64_t)d.H + (uint64_t)h) << 16) + (uint64_t)j;
  return drop_keep(drop_word(d.key, e >> 2), (int)(e & 3), d.thr);
}

// grid: (max_lq, H, B).  LDS: q row [dh] + scores [max_lk].
template <typename T>
__global__ __launch_bounds__(AN_THREADS) void attn_fwd_naive_kernel(const T* __restrict__ q, int ldq, const T* __restrict__ k, int ldk,
                                                                    const T* __restrict__ v, int ldv, T* __restrict__ o, int ldo,
                                                                    float* __restrict__ lse, const int* __restrict__ q_off,
                                                                    const int* __restrict__ k_off, int dh, int total_q, int causal,
                                                                    float scale, AttnDrop drop) {
  extern __shared__ float lds[];
  __shared__ float sh[16];
  const int b = blockIdx.z, h = blockIdx.y, i = blockIdx.x;
  const int q0 = q_off[b], lq = q_off[b + 1] - q0, k0 = k_off[b], lk = k_off[b + 1] - k0;
  if (i >= lq) return;
  float* qs = lds;
  float* sc = lds + dh;
  const int nk = causal ? min(lk, i + 1) : lk;
  for (int c = threadIdx.x; c < dh; c += AN_THREADS) qs[c] = to_f<T>(q[(size_t)(q0 + i) * ldq + h * dh + c]);
  __syncthreads();
  float lmax = -INFINITY;
  for (int j = threadIdx.x; j < nk; j += AN_THREADS) {
    const T* kr = k + (size_t)(k0 + j) * ldk + h * dh;
    float s = 0.f;
    for (int c = 0; c < dh; ++c) s += qs[c] * to_f<T>(kr[c]);
    s *= scale;
    sc[j] = s;
    lmax = fmaxf(lmax, s);
  }
  const float m = block_max(lmax, sh);
  float se = 0.f;
  for (int j = threadIdx.x; j < nk; j += AN_THREADS) {
    const float e = __expf(sc[j] - m);
    se += e;                                         // the row sum keeps every weight; only those that average V are dropped
    sc[j] = !drop.thr ? e : (attn_keep(drop, q0 + i, h, j) ? e * drop.inv_keep : 0.f);
  }
  se = block_sum(se, sh);
  __syncthreads();
  const float inv = 1.f / se;
  if (threadIdx.x == 0) lse[(size_t)h * total_q + q0 + i] = m + logf(se);
  for (int c = threadIdx.x; c < dh; c += AN_THREADS) {
    float acc = 0.f;
    for (int j = 0; j < nk; ++j) acc += sc[j] * to_f<T>(v[(size_t)(k0 + j) * ldv + h * dh + c]);
    o[(size_t)(q0 + i) * ldo + h * dh + c] = from_f<T>(acc * inv);
  }
}

// dQ pass.  grid (max_lq, H, B).  LDS: q, dO rows [dh] each + ds [max_lk].
template <typename T>
__global__ __launch_bounds__(AN_THREADS) void attn_bwd_dq_naive_kernel(
    const T* __restrict__ q, int ldq, const T* __restrict__ k, int ldk, const T* __restrict__ v, int ldv, const T* __restrict__ o,
    int ldo, const T* __restrict__ d_o, int lddo, const float* __restrict__ lse, T* __restrict__ dq, int lddq,
    const int* __restrict__ q_off, const int* __restrict__ k_off, int dh, int total_q, int causal, float scale, AttnDrop drop) {
  extern __shared__ float lds[];
  __shared__ float sh[16];
  const int b = blockIdx.z, h = blockIdx.y, i = blockIdx.x;
  const int q0 = q_off[b], lq = q_off[b + 1] - q0, k0 = k_off[b], lk = k_off[b + 1] - k0;
  if (i >= lq) return;
  float* qs = lds;
  float* dos = lds + dh;
  float* dsv = lds + 2 * dh;
  const int nk = causal ? min(lk, i + 1) : lk;
  float dl = 0.f;
  for (int c = threadIdx.x; c < dh; c += AN_THREADS) {
    qs[c] = to_f<T>(q[(size_t)(q0 + i) * ldq + h * dh + c]);
    const float g = to_f<T>(d_o[(size_t)(q0 + i) * lddo + h * dh + c]);
    dos[c] = g;
    dl += g * to_f<T>(o[(size_t)(q0 + i) * ldo + h * dh + c]);
  }
  const float delta = block_sum(dl, sh);
  __syncthreads();
  const float L = lse[(size_t)h * total_q + q0 + i];
  for (int j = threadIdx.x; j < nk; j += AN_THREADS) {
    const T* kr = k + (size_t)(k0 + j) * ldk + h * dh;
    const T* vr = v + (size_t)(k0 + j) * ldv + h * dh;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) { s += qs[c] * to_f<T>(kr[c]); dp += dos[c] * to_f<T>(vr[c]); }
    const float p = __expf(s * scale - L);
    if (drop.thr) dp = attn_keep(drop, q0 + i, h, j) ? dp * drop.inv_keep : 0.f;
    dsv[j] = p * (dp - delta);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += AN_THREADS) {
    float acc = 0.f;
    for (int j = 0; j < nk; ++j) acc += dsv[j] * to_f<T>(k[(size_t)(k0 + j) * ldk + h * dh + c]);
    dq[(size_t)(q0 + i) * lddq + h * dh + c] = from_f<T>(acc * scale);
  }
}

// dK/dV pass.  grid (max_lk, H, B).  LDS: k, v rows [dh] + p [max_lq] + ds [max_lq].
template <typename T>
__global__ __launch_bounds__(AN_THREADS) void attn_bwd_dkv_naive_kernel(
    const T* __restrict__ q, int ldq, const T* __restrict__ k, int ldk, const T* __restrict__ v, int ldv, const T* __restrict__ o,
    int ldo, const T* __restrict__ d_o, int lddo, const float* __restrict__ lse, T* __restrict__ dk, int lddk, T* __restrict__ dv,
    int lddv, const int* __restrict__ q_off, const int* __restrict__ k_off, int dh, int total_q, int max_lq, int causal,
    float scale, AttnDrop drop) {
  extern __shared__ float lds[];
  const int b = blockIdx.z, h = blockIdx.y, j = blockIdx.x;
  const int q0 = q_off[b], lq = q_off[b + 1] - q0, k0 = k_off[b], lk = k_off[b + 1] - k0;
  if (j >= lk) return;
  float* ks = lds;
  float* vs = lds + dh;
  float* ps = lds + 2 * dh;
  float* dss = ps + max_lq;
  for (int c = threadIdx.x; c < dh; c += AN_THREADS) {
    ks[c] = to_f<T>(k[(size_t)(k0 + j) * ldk + h * dh + c]);
    vs[c] = to_f<T>(v[(size_t)(k0 + j) * ldv + h * dh + c]);
  }
  __syncthreads();
  const int i0 = causal ? j : 0;
  for (int i = i0 + threadIdx.x; i < lq; i += AN_THREADS) {
    const T* qr = q + (size_t)(q0 + i) * ldq + h * dh;
    const T* gr = d_o + (size_t)(q0 + i) * lddo + h * dh;
    const T* orow = o + (size_t)(q0 + i) * ldo + h * dh;
    float s = 0.f, dp = 0.f, delta = 0.f;
    for (int c = 0; c < dh; ++c) {
      const float g = to_f<T>(gr[c]);
      s += to_f<T>(qr[c]) * ks[c];
      dp += g * vs[c];
      delta += g * to_f<T>(orow[c]);
    }
    const float p = __expf(s * scale - lse[(size_t)h * total_q + q0 + i]);
    const bool keep = !drop.thr || attn_keep(drop, q0 + i, h, j);
    if (drop.thr) dp = keep ? dp * drop.inv_keep : 0.f;
    ps[i] = !drop.thr ? p : (keep ? p * drop.inv_keep : 0.f);      // dV averages dO with the dropped weights
    dss[i] = p * (dp - delta);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += AN_THREADS) {
    float av = 0.f, ak = 0.f;
    for (int i = i0; i < lq; ++i) {
      av += ps[i] * to_f<T>(d_o[(size_t)(q0 + i) * lddo + h * dh + c]);
      ak += dss[i] * to_f<T>(q[(size_t)(q0 + i) * ldq + h * dh + c]);
    }
    dv[(size_t)(k0 + j) * lddv + h * dh + c] = from_f<T>(av);
    dk[(size_t)(k0 + j) * lddk + h * dh + c] = from_f<T>(ak * scale);
  }
}

static AttnDrop make_drop(const AttnArgs& a) {
  return AttnDrop{a.drop_key, a.drop_p > 0.f ? drop_threshold(a.drop_p) : 0u, 1.f / (1.f - a.drop_p), a.H};
}
template <typename T>
static void attn_fwd_naive(hipStream_t s, const AttnArgs& a) {
  const float scale = 1.f / sqrtf((float)a.dh);
  dim3 grid(a.max_lq, a.H, a.B), block(AN_THREADS);
  const size_t shm = (size_t)(a.dh + a.max_lk) * sizeof(float);
  hipLaunchKernelGGL((attn_fwd_naive_kernel<T>), grid, block, shm, s, (const T*)a.q, a.ldq, (const T*)a.k, a.ldk, (const T*)a.v,
                     a.ldv, (T*)a.o, a.ldo, a.lse, a.q_off, a.k_off, a.dh, a.total_q, a.causal, scale, make_drop(a));
}
template <typename T>
static void attn_bwd_naive(hipStream_t s, const AttnArgs& a) {
  const float scale = 1.f / sqrtf((float)a.dh);
  {
    dim3 grid(a.max_lq, a.H, a.B), block(AN_THREADS);
    const size_t shm = (size_t)(2 * a.dh + a.max_lk) * sizeof(float);
    hipLaunchKernelGGL((attn_bwd_dq_naive_kernel<T>), grid, block, shm, s, (const T*)a.q, a.ldq, (const T*)a.k, a.ldk,
                       (const T*)a.v, a.ldv, (const T*)a.o, a.ldo, (const T*)a.d_o, a.lddo, a.lse, (T*)a.dq, a.lddq, a.q_off,
                       a.k_off, a.dh, a.total_q, a.causal, scale, make_drop(a));
  }
  {
    dim3 grid(a.max_lk, a.H, a.B), block(AN_THREADS);
    const size_t shm = (size_t)(2 * a.dh + 2 * a.max_lq) * sizeof(float);
    hipLaunchKernelGGL((attn_bwd_dkv_naive_kernel<T>), grid, block, shm, s, (const T*)a.q, a.ldq, (const T*)a.k, a.ldk,
                       (const T*)a.v, a.ldv, (const T*)a.o, a.ldo, (const T*)a.d_o, a.lddo, a.lse, (T*)a.dk, a.lddk, (T*)a.dv,
                       a.lddv, a.q_off, a.k_off, a.dh, a.total_q, a.max_lq, a.causal, scale, make_drop(a));
  }
}

void launch_attention_fwd_naive(hipStream_t s, const AttnArgs& a) {
  if (a.B <= 0 || a.max_lq <= 0) return;
  if (a.dt == F32) attn_fwd_naive<float>(s, a);
  else if (a.dt == F16) attn_fwd_naive<half_t>(s, a);
  else attn_fwd_naive<bf16_t>(s, a);
}
void launch_attention_bwd_naive(hipStream_t s, const AttnArgs& a) {
  if (a.B <= 0 || a.max_lq <= 0) return;
  if (a.dt == F32) attn_bwd_naive<float>(s, a);
  else if (a.dt == F16) attn_bwd_naive<half_t>(s, a);
  else attn_bwd_naive<bf16_t>(s, a);
}

}  // namespace tfm
