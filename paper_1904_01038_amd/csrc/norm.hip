// Residual + dropout + LayerNorm forward and backward, and column sums (bias gradients).  All HBM-bound: one
// wavefront owns one row, each lane moves 8 contiguous elements per access (16 bytes in half precision), the row
// stays in registers between the statistics and the normalisation, statistics are fp32.
#include "common.h"
#include "kernels.h"

namespace tfm {

constexpr int LN_VEC = 8;
constexpr float LN_EPS = 1e-5f;

// s = x + drop(y); n = gamma * (s - mean) * rstd + beta.  NCH = chunks of 8 elements per lane (d <= NCH * 512).
template <typename T, int NCH>
__global__ __launch_bounds__(256) void residual_layernorm_fwd_kernel(
    const T* __restrict__ x, const T* __restrict__ y, const T* __restrict__ gamma, const T* __restrict__ beta,
    T* __restrict__ s_out, T* __restrict__ n_out, float* __restrict__ mean, float* __restrict__ rstd, int rows, int d,
    uint64_t key, uint32_t thr, float inv_keep) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const size_t base = (size_t)row * d;
  float v[NCH][LN_VEC];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) {
      load_f<T, LN_VEC>(x + base + col, v[c]);
      if (y) {
        float t[LN_VEC];
        load_f<T, LN_VEC>(y + base + col, t);
        if (thr) drop_apply<LN_VEC>(t, key, base + col, thr, inv_keep);
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) v[c][i] += t[i];
      }
      if (s_out) {
        store_f<T, LN_VEC>(s_out + base + col, v[c]);
        // the backward pass reads the stored (rounded) sum, so normalise exactly that
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) v[c][i] = to_f<T>(from_f<T>(v[c][i]));
      }
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) sum += v[c][i];
    }
  }
  const float mu = wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) {
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) { const float t = v[c][i] - mu; sq += t * t; }
    }
  }
  const float rs = rsqrtf(wave_sum(sq) / (float)d + LN_EPS);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) {
      float g[LN_VEC], b[LN_VEC], o[LN_VEC];
      load_f<T, LN_VEC>(gamma + col, g);
      load_f<T, LN_VEC>(beta + col, b);
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) o[i] = g[i] * ((v[c][i] - mu) * rs) + b[i];
      store_f<T, LN_VEC>(n_out + base + col, o);
    }
  }
}

// s = x + (bias + sum of the fp32 slices); n = gamma * (s - mean) * rstd + beta.  One wavefront per row as above.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void splitk_layernorm_fwd_kernel(
    const T* __restrict__ x, const float* __restrict__ partial, int splits, const T* __restrict__ bias,
    const T* __restrict__ gamma, const T* __restrict__ beta, T* __restrict__ s_out, T* __restrict__ n_out, int rows, int d) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const size_t base = (size_t)row * d, slice = (size_t)rows * d;
  float v[NCH][LN_VEC];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) {
      load_f<T, LN_VEC>(x + base + col, v[c]);
      // all slices' loads are issued together (at most 8 slices: the split-K launch's own limit), then added in order
      float t[8][LN_VEC], y[LN_VEC];
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k < splits) load_f<float, LN_VEC>(partial + k * slice + base + col, t[k]);
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) y[i] = t[0][i];
#pragma unroll
      for (int k = 1; k < 8; ++k)
        if (k < splits) {
#pragma unroll
          for (int i = 0; i < LN_VEC; ++i) y[i] += t[k][i];
        }
      if (bias) {
        float t[LN_VEC];
        load_f<T, LN_VEC>(bias + col, t);
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) y[i] += t[i];
      }
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) v[c][i] += y[i];
      if (s_out) {
        store_f<T, LN_VEC>(s_out + base + col, v[c]);
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) v[c][i] = to_f<T>(from_f<T>(v[c][i]));     // normalise what was stored, as above
      }
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) sum += v[c][i];
    }
  }
  const float mu = wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) {
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) { const float t = v[c][i] - mu; sq += t * t; }
    }
  }
  const float rs = rsqrtf(wave_sum(sq) / (float)d + LN_EPS);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) {
      float g[LN_VEC], b[LN_VEC], o[LN_VEC];
      load_f<T, LN_VEC>(gamma + col, g);
      load_f<T, LN_VEC>(beta + col, b);
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) o[i] = g[i] * ((v[c][i] - mu) * rs) + b[i];
      store_f<T, LN_VEC>(n_out + base + col, o);
    }
  }
}

template <typename T>
static void splitk_ln_dispatch(hipStream_t s, const void* x, const float* partial, int splits, const void* bias, const void* gamma,
                               const void* beta, void* s_out, void* n_out, int rows, int d) {
  dim3 grid((rows + 3) / 4), block(256);
  const int nch = (d + 511) / 512;
#define SLN(N)                                                                                                             \
  hipLaunchKernelGGL((splitk_layernorm_fwd_kernel<T, N>), grid, block, 0, s, (const T*)x, partial, splits, (const T*)bias, \
                     (const T*)gamma, (const T*)beta, (T*)s_out, (T*)n_out, rows, d)
  if (nch <= 1) SLN(1); else if (nch == 2) SLN(2); else if (nch == 3) SLN(3); else SLN(4);
#undef SLN
}
void launch_splitk_layernorm_fwd(hipStream_t s, int dt, const void* x, const float* partial, int splits, const void* bias,
                                 const void* gamma, const void* beta, void* s_out, void* n_out, int rows, int d) {
  if (rows <= 0) return;
  if (dt == F16) splitk_ln_dispatch<half_t>(s, x, partial, splits, bias, gamma, beta, s_out, n_out, rows, d);
  else if (dt == BF16) splitk_ln_dispatch<bf16_t>(s, x, partial, splits, bias, gamma, beta, s_out, n_out, rows, d);
  // (split-K launches exist for the 2-byte types only)
}

template <typename T>
static void ln_fwd_dispatch(hipStream_t s, const void* x, const void* y, const void* gamma, const void* beta, void* s_out,
                            void* n_out, float* mean, float* rstd, int rows, int d, uint64_t key, float p) {
  const uint32_t thr = (p > 0.f && y) ? drop_threshold(p) : 0u;
  const float inv_keep = 1.f / (1.f - p);
  dim3 grid((rows + 3) / 4), block(256);
  const int nch = (d + 511) / 512;
#define LN_FWD(N)                                                                                                        \
  hipLaunchKernelGGL((residual_layernorm_fwd_kernel<T, N>), grid, block, 0, s, (const T*)x, (const T*)y, (const T*)gamma, \
                     (const T*)beta, (T*)s_out, (T*)n_out, mean, rstd, rows, d, key, thr, inv_keep)
  if (nch <= 1) LN_FWD(1); else if (nch == 2) LN_FWD(2); else if (nch == 3) LN_FWD(3); else LN_FWD(4);
#undef LN_FWD
}

void launch_residual_layernorm_fwd(hipStream_t s, int dt, const void* x, const void* y, const void* gamma,
                                   const void* beta, void* s_out, void* n_out, float* mean, float* rstd, int rows,
                                   int d, uint64_t key, float p) {
  if (rows <= 0) return;
  if (dt == F32) ln_fwd_dispatch<float>(s, x, y, gamma, beta, s_out, n_out, mean, rstd, rows, d, key, p);
  else if (dt == F16) ln_fwd_dispatch<half_t>(s, x, y, gamma, beta, s_out, n_out, mean, rstd, rows, d, key, p);
  else ln_fwd_dispatch<bf16_t>(s, x, y, gamma, beta, s_out, n_out, mean, rstd, rows, d, key, p);
}

// ---- backward -----------------------------------------------------------------------------------------------------------
// Per row: xhat = (s - mean) rstd; dxhat = dn * gamma; ds = rstd (dxhat - mean(dxhat) - xhat mean(dxhat xhat)) + add.
// Column partial sums (dgamma = sum dn xhat, dbeta = sum dn, dbias = sum dropout-backward(ds)) are kept in registers
// while a wavefront walks its rows, combined across the block's 8 wavefronts in LDS (one quantity at a time, so the
// LDS footprint stays at 8 rows), and written once per block to partial[block][3][d]; a second kernel adds the
// partials in a fixed order.  One block per CU, 8 wavefronts each, keeps enough rows in flight to cover HBM latency.
constexpr int LNB_MAX_BLOCKS = 256;
constexpr int LNB_WAVES = 8;

template <typename T, int NCH>
__global__ __launch_bounds__(64 * LNB_WAVES) void layernorm_bwd_kernel(
    const T* __restrict__ dn, const T* __restrict__ add, const T* __restrict__ sres, const float* __restrict__ mean,
    const float* __restrict__ rstd, const T* __restrict__ gamma, T* __restrict__ ds, T* __restrict__ ds_drop,
    float* __restrict__ partial, int rows, int d, uint64_t key, uint32_t thr, float inv_keep, int nk) {
  extern __shared__ float lds[];     // [LNB_WAVES][d]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float g[NCH][LN_VEC], ag[NCH][LN_VEC], ab[NCH][LN_VEC], ac[NCH][LN_VEC];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * LN_VEC;
    if (col < d) load_f<T, LN_VEC>(gamma + col, g[c]);
#pragma unroll
    for (int i = 0; i < LN_VEC; ++i) ag[c][i] = ab[c][i] = ac[c][i] = 0.f;
  }
  // The next row's operands are fetched into registers before the current row's reductions, so a wavefront always has
  // a full row of loads in flight.
  float a[NCH][LN_VEC], b[NCH][LN_VEC], t[NCH][LN_VEC];
  const int rstep = gridDim.x * LNB_WAVES;
  int row = blockIdx.x * LNB_WAVES + w;
  auto fetch = [&](int r, float (&fa)[NCH][LN_VEC], float (&fb)[NCH][LN_VEC], float (&ft)[NCH][LN_VEC]) {
    const size_t base = (size_t)r * d;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
        load_f<T, LN_VEC>(dn + base + col, fa[c]);
        load_f<T, LN_VEC>(sres + base + col, fb[c]);
        if (add) load_f<T, LN_VEC>(add + base + col, ft[c]);
      }
    }
  };
  if (row < rows) fetch(row, a, b, t);
  for (; row < rows; row += rstep) {
    const size_t base = (size_t)row * d;
    const float mu = mean[row], rs = rstd[row];
    float xh[NCH][LN_VEC], dxh[NCH][LN_VEC], tt[NCH][LN_VEC];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) {
          xh[c][i] = (b[c][i] - mu) * rs;
          dxh[c][i] = a[c][i] * g[c][i];
          s1 += dxh[c][i];
          s2 += dxh[c][i] * xh[c][i];
          ag[c][i] += a[c][i] * xh[c][i];
          ab[c][i] += a[c][i];
          tt[c][i] = t[c][i];
        }
      }
    }
    if (row + rstep < rows) fetch(row + rstep, a, b, t);
    const float c1 = wave_sum(s1) / (float)d, c2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
        float o[LN_VEC];
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) o[i] = rs * (dxh[c][i] - c1 - xh[c][i] * c2);
        if (add) {
#pragma unroll
          for (int i = 0; i < LN_VEC; ++i) o[i] += tt[c][i];
        }
        store_f<T, LN_VEC>(ds + base + col, o);
        if (thr) {
          drop_apply<LN_VEC>(o, key, base + col, thr, inv_keep);
          store_f<T, LN_VEC>(ds_drop + base + col, o);
        }
        // the consumers read the rounded value; sum exactly what they will see
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) ac[c][i] += to_f<T>(from_f<T>(o[i]));
      }
    }
  }
  for (int k = 0; k < nk; ++k) {                        // nk = 2: the bias sum is not wanted
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) lds[w * d + col + i] = k == 0 ? ag[c][i] : (k == 1 ? ab[c][i] : ac[c][i]);
      }
    }
    __syncthreads();
    for (int col = threadIdx.x; col < d; col += 64 * LNB_WAVES) {
      float t = 0.f;
#pragma unroll
      for (int ww = 0; ww < LNB_WAVES; ++ww) t += lds[ww * d + col];
      partial[((size_t)blockIdx.x * 3 + k) * d + col] = t;
    }
  }
}

// Column held by slot p of the row kernel's LDS / partial layout: lane l keeps elements i = 0..7 of 8-vector
// l + 64 c in slot c * 512 + i * 64 + l, so that a wavefront's stores of one element hit 64 different banks
// (storing a lane's 8 values side by side would be an 8-way conflict, 16 wavefronts deep).  d must be a multiple of 512.
__host__ __device__ __forceinline__ int ln_slot_column(int p) { return ((p & 63) + 64 * (p >> 9)) * 8 + ((p >> 6) & 7); }

// The same computation when every row can have a wavefront of its own (rows <= LNB_MAX_BLOCKS * LNR_WAVES): 16
// wavefronts per block, one row each, no loop.  Nothing is accumulated across rows, so the three per-column
// quantities go from the row's registers straight into the block's LDS reduction, the register footprint stays below
// 128 and a row's two dependent passes are the whole critical path.
constexpr int LNR_WAVES = 16;

template <typename T, int NCH>
__global__ __launch_bounds__(64 * LNR_WAVES) void layernorm_bwd_row_kernel(
    const T* __restrict__ dn, const T* __restrict__ add, const T* __restrict__ sres, const float* __restrict__ mean,
    const float* __restrict__ rstd, const T* __restrict__ gamma, T* __restrict__ ds, T* __restrict__ ds_drop,
    float* __restrict__ partial, int rows, int d, uint64_t key, uint32_t thr, float inv_keep, int nk) {
  extern __shared__ float lds[];     // [LNR_WAVES][d]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int row = blockIdx.x * LNR_WAVES + w;
  const bool live = row < rows;
  const size_t base = (size_t)(live ? row : 0) * d;
  float a[NCH][LN_VEC], xh[NCH][LN_VEC], o[NCH][LN_VEC];
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int i = 0; i < LN_VEC; ++i) a[c][i] = xh[c][i] = o[c][i] = 0.f;
  if (live) {
    const float mu = mean[row], rs = rstd[row];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
        float b[LN_VEC], g[LN_VEC];
        load_f<T, LN_VEC>(dn + base + col, a[c]);
        load_f<T, LN_VEC>(sres + base + col, b);
        load_f<T, LN_VEC>(gamma + col, g);
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) {
          xh[c][i] = (b[i] - mu) * rs;
          o[c][i] = a[c][i] * g[i];                      // dxhat, turned into ds below
          s1 += o[c][i];
          s2 += o[c][i] * xh[c][i];
        }
      }
    }
    const float c1 = wave_sum(s1) / (float)d, c2 = wave_sum(s2) / (float)d;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) o[c][i] = rs * (o[c][i] - c1 - xh[c][i] * c2);
        if (add) {
          float t[LN_VEC];
          load_f<T, LN_VEC>(add + base + col, t);
#pragma unroll
          for (int i = 0; i < LN_VEC; ++i) o[c][i] += t[i];
        }
        store_f<T, LN_VEC>(ds + base + col, o[c]);
        if (thr) {
          drop_apply<LN_VEC>(o[c], key, base + col, thr, inv_keep);
          store_f<T, LN_VEC>(ds_drop + base + col, o[c]);
        }
        // the consumers read the rounded value; sum exactly what they will see
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i) o[c][i] = to_f<T>(from_f<T>(o[c][i]));
      }
    }
  }
  for (int k = 0; k < nk; ++k) {                        // nk = 2: the bias sum is not wanted
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * LN_VEC;
      if (col < d) {
#pragma unroll
        for (int i = 0; i < LN_VEC; ++i)                  // slot (c, i, lane): consecutive lanes, consecutive banks
          lds[w * d + c * 512 + i * 64 + lane] = k == 0 ? a[c][i] * xh[c][i] : (k == 1 ? a[c][i] : o[c][i]);
      }
    }
    __syncthreads();
    for (int slot = threadIdx.x; slot < d; slot += 64 * LNR_WAVES) {    // partials stay in slot order (see ln_slot_column)
      float t = 0.f;
#pragma unroll
      for (int ww = 0; ww < LNR_WAVES; ++ww) t += lds[ww * d + slot];
      partial[((size_t)blockIdx.x * 3 + k) * d + slot] = t;
    }
  }
}

// out_k[j] = sum_p partial[p][k][j], p in a fixed order; k < nk <= 3.  One block owns 32 columns of one k: 32 row
// lanes stride over the partials (coalesced 128-byte reads, all of a lane's loads in flight at once for up to 256
// partials), then LDS combines the 32 lanes in a fixed order.
constexpr int RP_LANES = 32;
template <typename T>
__device__ __forceinline__ void reduce_partials_body(const float* __restrict__ partial, int np, int nk, int n, T* o0, T* o1, T* o2, int slots) {
  __shared__ float sh[RP_LANES][33];
  const int cx = threadIdx.x & 31, py = threadIdx.x >> 5;
  const int k = blockIdx.y;
  const int j = blockIdx.x * 32 + cx;
  float acc = 0.f;
  if (j < n) {
    int p = py;
    for (; p + 7 * RP_LANES < np; p += 8 * RP_LANES) {  // 8 loads in flight per thread; the order of the adds is fixed
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = partial[((size_t)(p + RP_LANES * u) * nk + k) * n + j];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; p < np; p += RP_LANES) acc += partial[((size_t)p * nk + k) * n + j];
  }
  sh[py][cx] = acc;
  __syncthreads();
  if (py == 0 && j < n) {
    T* o = k == 0 ? o0 : (k == 1 ? o1 : o2);
    if (o) {
      float t = 0.f;
#pragma unroll
      for (int i = 0; i < RP_LANES; ++i) t += sh[i][cx];
      o[slots ? ln_slot_column(j) : j] = from_f<T>(t);    // slots: index j is a slot of the row kernel's layout
    }
  }
}
template <typename T>
__global__ __launch_bounds__(32 * RP_LANES) void reduce_partials_kernel(const float* __restrict__ partial, int np, int nk, int n, T* o0,
                                                                        T* o1, T* o2, int slots) {
  reduce_partials_body<T>(partial, np, nk, n, o0, o1, o2, slots);
}
// The reductions of many LayerNorm backward launches in one: blockIdx.z picks the job (the table travels in the kernel
// arguments).  Every job has the [np][3][d] layout; an output that is null is skipped.
struct LnReduceTable { LnReduceJob job[LN_REDUCE_MAX]; };
template <typename T>
__global__ __launch_bounds__(32 * RP_LANES) void reduce_partials_batched_kernel(LnReduceTable tab, int d) {
  const LnReduceJob& j = tab.job[blockIdx.z];
  reduce_partials_body<T>(j.partial, j.np, 3, d, (T*)j.dgamma, (T*)j.dbeta, (T*)j.dbias, j.slots);
}

static int lnb_blocks(int rows) {
  int b = (rows + LNB_WAVES - 1) / LNB_WAVES;
  return b > LNB_MAX_BLOCKS ? LNB_MAX_BLOCKS : (b < 1 ? 1 : b);
}
size_t layernorm_bwd_scratch_bytes(int rows, int d) { return (size_t)lnb_blocks(rows) * 3 * d * sizeof(float); }

template <typename T>
static void ln_bwd_dispatch(hipStream_t s, const void* dn, const void* add, const void* sres, const float* mean,
                            const float* rstd, const void* gamma, void* ds, void* ds_drop, void* dgamma, void* dbeta,
                            void* dbias, int rows, int d, uint64_t key, float p, void* scratch, LnReduceJob* defer) {
  const int nk = dbias ? 3 : 2;
  const uint32_t thr = (p > 0.f && ds_drop) ? drop_threshold(p) : 0u;
  const float inv_keep = 1.f / (1.f - p);
  const int nch = (d + 511) / 512;
  if (rows <= LNB_MAX_BLOCKS * LNR_WAVES && d % 512 == 0 && nch <= 2) {   // a wavefront per row (its LDS stage stays within 64 KB)
    const int nbr = (rows + LNR_WAVES - 1) / LNR_WAVES;
    const size_t shr = (size_t)LNR_WAVES * d * sizeof(float);
#define LN_BWD_ROW(N)                                                                                                   \
  hipLaunchKernelGGL((layernorm_bwd_row_kernel<T, N>), dim3(nbr), dim3(64 * LNR_WAVES), shr, s, (const T*)dn, (const T*)add,        \
                     (const T*)sres, mean, rstd, (const T*)gamma, (T*)ds, (T*)ds_drop, (float*)scratch, rows, d, key, thr, \
                     inv_keep, nk)
    if (nch <= 1) LN_BWD_ROW(1); else LN_BWD_ROW(2);
#undef LN_BWD_ROW
    if (defer) { *defer = LnReduceJob{(const float*)scratch, nbr, 1, dgamma, dbeta, dbias}; return; }
    hipLaunchKernelGGL((reduce_partials_kernel<T>), dim3((d + 31) / 32, 3), dim3(32 * RP_LANES), 0, s, (const float*)scratch, nbr, 3, d,
                       (T*)dgamma, (T*)dbeta, (T*)dbias, 1);
    return;
  }
  const int nb = lnb_blocks(rows);
  const size_t shm = (size_t)LNB_WAVES * d * sizeof(float);
#define LN_BWD(N)                                                                                                       \
  hipLaunchKernelGGL((layernorm_bwd_kernel<T, N>), dim3(nb), dim3(64 * LNB_WAVES), shm, s, (const T*)dn, (const T*)add,             \
                     (const T*)sres, mean, rstd, (const T*)gamma, (T*)ds, (T*)ds_drop, (float*)scratch, rows, d, key, thr, \
                     inv_keep, nk)
  if (nch <= 1) LN_BWD(1); else if (nch == 2) LN_BWD(2); else if (nch == 3) LN_BWD(3); else LN_BWD(4);
#undef LN_BWD
  if (defer) { *defer = LnReduceJob{(const float*)scratch, nb, 0, dgamma, dbeta, dbias}; return; }
  hipLaunchKernelGGL((reduce_partials_kernel<T>), dim3((d + 31) / 32, 3), dim3(32 * RP_LANES), 0, s, (const float*)scratch, nb, 3, d,
                     (T*)dgamma, (T*)dbeta, (T*)dbias, 0);
}

void launch_layernorm_bwd(hipStream_t s, int dt, const void* dn, const void* add, const void* sres, const float* mean,
                          const float* rstd, const void* gamma, void* ds, void* ds_drop, void* dgamma, void* dbeta,
                          void* dbias, int rows, int d, uint64_t key, float p, void* scratch, LnReduceJob* defer) {
  if (dt == F32) ln_bwd_dispatch<float>(s, dn, add, sres, mean, rstd, gamma, ds, ds_drop, dgamma, dbeta, dbias, rows, d, key, p, scratch, defer);
  else if (dt == F16) ln_bwd_dispatch<half_t>(s, dn, add, sres, mean, rstd, gamma, ds, ds_drop, dgamma, dbeta, dbias, rows, d, key, p, scratch, defer);
  else ln_bwd_dispatch<bf16_t>(s, dn, add, sres, mean, rstd, gamma, ds, ds_drop, dgamma, dbeta, dbias, rows, d, key, p, scratch, defer);
}

void launch_ln_reduce_batched(hipStream_t s, int dt, const LnReduceJob* jobs, int n, int d) {
  for (int i0 = 0; i0 < n; i0 += LN_REDUCE_MAX) {
    const int m = n - i0 < LN_REDUCE_MAX ? n - i0 : LN_REDUCE_MAX;
    LnReduceTable tab;
    for (int i = 0; i < m; ++i) tab.job[i] = jobs[i0 + i];
    const dim3 grid((d + 31) / 32, 3, m), block(32 * RP_LANES);
    if (dt == F32) hipLaunchKernelGGL((reduce_partials_batched_kernel<float>), grid, block, 0, s, tab, d);
    else if (dt == F16) hipLaunchKernelGGL((reduce_partials_batched_kernel<half_t>), grid, block, 0, s, tab, d);
    else hipLaunchKernelGGL((reduce_partials_batched_kernel<bf16_t>), grid, block, 0, s, tab, d);
  }
}

// ---- column sums --------------------------------------------------------------------------------------------------------
// out[j] = sum_r x[r, j].  Block = 64 column chunks (8 columns each) x 4 row lanes; grid.y row slabs write partials.
constexpr int CS_ROWS_PER_BLOCK = 64;

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ x, int ld, int rows, int n, float* __restrict__ partial) {
  __shared__ float lds[4][64 * LN_VEC];
  const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + cx) * LN_VEC;
  float acc[LN_VEC];
#pragma unroll
  for (int i = 0; i < LN_VEC; ++i) acc[i] = 0.f;
  const int r0 = blockIdx.y * CS_ROWS_PER_BLOCK;
  const int r1 = min(rows, r0 + CS_ROWS_PER_BLOCK);
  if (col < n) {
    for (int r = r0 + ry; r < r1; r += 4) {
      float t[LN_VEC];
      load_f<T, LN_VEC>(x + (size_t)r * ld + col, t);
#pragma unroll
      for (int i = 0; i < LN_VEC; ++i) acc[i] += t[i];
    }
  }
#pragma unroll
  for (int i = 0; i < LN_VEC; ++i) lds[ry][cx * LN_VEC + i] = acc[i];
  __syncthreads();
  for (int j = threadIdx.x; j < 64 * LN_VEC; j += 256) {
    const int c = blockIdx.x * 64 * LN_VEC + j;
    if (c < n) partial[(size_t)blockIdx.y * n + c] = (lds[0][j] + lds[1][j]) + (lds[2][j] + lds[3][j]);
  }
}

size_t colsum_scratch_bytes(int rows, int n) {
  return (size_t)((rows + CS_ROWS_PER_BLOCK - 1) / CS_ROWS_PER_BLOCK + 1) * n * sizeof(float);
}

template <typename T>
static void colsum_dispatch(hipStream_t s, const void* x, int ld, int rows, int n, void* out, void* scratch) {
  const int ny = (rows + CS_ROWS_PER_BLOCK - 1) / CS_ROWS_PER_BLOCK;
  dim3 grid((n + 64 * LN_VEC - 1) / (64 * LN_VEC), ny);
  hipLaunchKernelGGL((colsum_kernel<T>), grid, dim3(256), 0, s, (const T*)x, ld, rows, n, (float*)scratch);
  hipLaunchKernelGGL((reduce_partials_kernel<T>), dim3((n + 31) / 32, 1), dim3(32 * RP_LANES), 0, s, (const float*)scratch, ny, 1, n,
                     (T*)out, (T*)nullptr, (T*)nullptr, 0);
}

void launch_colsum(hipStream_t s, int dt, const void* x, int ld, int rows, int n, void* out, void* scratch) {
  if (dt == F32) colsum_dispatch<float>(s, x, ld, rows, n, out, scratch);
  else if (dt == F16) colsum_dispatch<half_t>(s, x, ld, rows, n, out, scratch);
  else colsum_dispatch<bf16_t>(s, x, ld, rows, n, out, scratch);
}

}  // namespace tfm
