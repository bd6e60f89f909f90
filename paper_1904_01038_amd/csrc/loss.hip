// Fused log-softmax + label-smoothed cross-entropy, forward and backward in place over the vocabulary.
// HBM-bound: one block per target token; the row of logits is read once into registers when it fits
// (V <= 1024 threads * 16 chunks * 8), reduced (max, sum exp, sum z) in fp32, and overwritten with
// scale * (softmax(z) - q).  Algorithmic traffic: one read + one write of the logits.
#include "common.h"
#include "kernels.h"

namespace tfm {

constexpr int LV = 8;
constexpr int LOSS_THREADS = 256;
constexpr int LOSS_MAX_CHUNKS = 16;      // register-resident row: up to 1024 threads * 16 chunks * 8 = 131072 logits

struct OnlineLse { float m, s; };
__device__ __forceinline__ void lse_add(OnlineLse& a, float z) {
  if (z > a.m) { a.s = a.s * __expf(a.m - z) + 1.f; a.m = z; } else { a.s += __expf(z - a.m); }
}

// CACHED: the row lives in registers (NCH chunks per thread); otherwise it is read twice.
template <typename T, int VEC, bool CACHED, int NCH, int NT>
__global__ __launch_bounds__(NT) void loss_kernel(T* __restrict__ z, const int* __restrict__ labels,
                                                            float* __restrict__ loss_rows, float* __restrict__ nll_rows, int V,
                                                            float eps, const float* __restrict__ scale_ptr, float mult,
                                                            float* __restrict__ step_scale_out) {
  __shared__ float sh[16];
  const int row = blockIdx.x;
  T* zr = z + (size_t)row * V;
  const int label = labels[row];
  float scale = (scale_ptr ? *scale_ptr : 1.f) * mult;
  if (row == 0 && threadIdx.x == 0 && step_scale_out) *step_scale_out = scale;

  float cache[CACHED ? NCH : 1][VEC];
  float lmax = -INFINITY, zsum = 0.f;
  if (CACHED) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (threadIdx.x + c * NT) * VEC;
      if (col < V) {
        load_f<T, VEC>(zr + col, cache[c]);
#pragma unroll
        for (int i = 0; i < VEC; ++i) { lmax = fmaxf(lmax, cache[c][i]); zsum += cache[c][i]; }
      }
    }
  } else {
    for (int col = threadIdx.x * VEC; col < V; col += NT * VEC) {
      float t[VEC];
      load_f<T, VEC>(zr + col, t);
#pragma unroll
      for (int i = 0; i < VEC; ++i) { lmax = fmaxf(lmax, t[i]); zsum += t[i]; }
    }
  }
  const float m = block_max(lmax, sh);
  float se = 0.f;
  if (CACHED) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (threadIdx.x + c * NT) * VEC;
      if (col < V) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) se += __expf(cache[c][i] - m);
      }
    }
  } else {
    for (int col = threadIdx.x * VEC; col < V; col += NT * VEC) {
      float t[VEC];
      load_f<T, VEC>(zr + col, t);
#pragma unroll
      for (int i = 0; i < VEC; ++i) se += __expf(t[i] - m);
    }
  }
  se = block_sum(se, sh);
  zsum = block_sum(zsum, sh);
  const float lse = m + logf(se);
  const float zy = to_f<T>(zr[label]);       // read before any thread overwrites the row
  __syncthreads();
  if (threadIdx.x == 0) {
    const float nll = lse - zy;
    const float smooth = lse - zsum / (float)V;
    loss_rows[row] = (1.f - eps) * nll + eps * smooth;
    nll_rows[row] = nll;
  }
  const float qs = eps / (float)V;
  if (CACHED) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (threadIdx.x + c * NT) * VEC;
      if (col < V) {
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          const float q = qs + ((col + i) == label ? (1.f - eps) : 0.f);
          o[i] = scale * (__expf(cache[c][i] - lse) - q);
        }
        store_f<T, VEC>(zr + col, o);
      }
    }
  } else {
    for (int col = threadIdx.x * VEC; col < V; col += NT * VEC) {
      float t[VEC], o[VEC];
      load_f<T, VEC>(zr + col, t);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        const float q = qs + ((col + i) == label ? (1.f - eps) : 0.f);
        o[i] = scale * (__expf(t[i] - lse) - q);
      }
      store_f<T, VEC>(zr + col, o);
    }
  }
}

template <typename T>
static void loss_dispatch(hipStream_t s, void* z, const int* labels, float* loss_rows, float* nll_rows, int rows, int V,
                          float eps, const float* scale_ptr, float mult, float* sso) {
  dim3 grid(rows);
#define LOSS(VEC, CACHED, NCH, NT)                                                                                       \
  hipLaunchKernelGGL((loss_kernel<T, VEC, CACHED, NCH, NT>), grid, dim3(NT), 0, s, (T*)z, labels, loss_rows, nll_rows, V, eps, \
                     scale_ptr, mult, sso)
  if (V % LV != 0) { LOSS(1, false, 1, 256); return; }
  const int vecs = V / LV;                               // 8-element vectors in a row
  // the row stays in registers when it fits; long rows get 1024 threads so that few registers hold it and many
  // wavefronts per CU keep loads in flight
  if (sizeof(T) == 2 && vecs <= 4 * 256) LOSS(LV, true, 4, 256);
  else if (sizeof(T) == 2 && vecs <= 4 * 1024) LOSS(LV, true, 4, 1024);
  else if (sizeof(T) == 2 && vecs <= LOSS_MAX_CHUNKS * 1024) LOSS(LV, true, LOSS_MAX_CHUNKS, 1024);
  else LOSS(LV, false, 1, 1024);
#undef LOSS
}

void launch_loss(hipStream_t s, int dt, void* z, const int* labels, float* loss_rows, float* nll_rows, int rows, int V,
                 float eps, const float* scale_ptr, float mult, float* step_scale_out) {
  if (rows <= 0) return;
  if (dt == F32) loss_dispatch<float>(s, z, labels, loss_rows, nll_rows, rows, V, eps, scale_ptr, mult, step_scale_out);
  else if (dt == F16) loss_dispatch<half_t>(s, z, labels, loss_rows, nll_rows, rows, V, eps, scale_ptr, mult, step_scale_out);
  else loss_dispatch<bf16_t>(s, z, labels, loss_rows, nll_rows, rows, V, eps, scale_ptr, mult, step_scale_out);
}

__global__ __launch_bounds__(1024) void sum_rows_kernel(const float* __restrict__ a, const float* __restrict__ b, int rows,
                                                        double* __restrict__ sums) {
  __shared__ double sh[2][1024];
  double sa = 0.0, sb = 0.0;
  for (int r = threadIdx.x; r < rows; r += 1024) { sa += (double)a[r]; sb += (double)b[r]; }
  sh[0][threadIdx.x] = sa;
  sh[1][threadIdx.x] = sb;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (threadIdx.x < o) { sh[0][threadIdx.x] += sh[0][threadIdx.x + o]; sh[1][threadIdx.x] += sh[1][threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { sums[0] = sh[0][0]; sums[1] = sh[1][0]; }
}
void launch_sum_rows(hipStream_t s, const float* loss_rows, const float* nll_rows, int rows, double* sums) {
  hipLaunchKernelGGL(sum_rows_kernel, dim3(1), dim3(1024), 0, s, loss_rows, nll_rows, rows, sums);
}

}  // namespace tfm
