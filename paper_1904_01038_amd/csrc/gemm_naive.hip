// Shape-agnostic GEMM with fp32 accumulation on the vector ALUs.  It serves the fp32 precision mode (the tiny
// parity configuration) and any shape the MFMA kernels do not take (unaligned leading dimensions); it is not on
// the performance path.  64x64 output tile, 16-deep LDS stages, 4x4 outputs per thread.
#include "common.h"
#include "kernels.h"

namespace tfm {

template <typename T, int FORM>
__global__ __launch_bounds__(256) void gemm_naive_kernel(int M, int N, int K, const T* __restrict__ A, int lda,
                                                         const T* __restrict__ B, int ldb, T* __restrict__ C, int ldc,
                                                         const T* __restrict__ bias, int relu, const T* __restrict__ mask,
                                                         const T* __restrict__ residual, uint64_t drop_key, uint32_t drop_thr,
                                                         float inv_keep, float mask_scale) {
  __shared__ float As[16][64 + 1];
  __shared__ float Bs[16][64 + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      int mm, kk;
      if (FORM == 2) { mm = i & 63; kk = i >> 6; } else { kk = i & 15; mm = i >> 4; }     // walk the contiguous dim
      const int gm = m0 + mm, gk = k0 + kk;
      float v = 0.f;
      if (gm < M && gk < K) v = to_f<T>(FORM == 2 ? A[(size_t)gk * lda + gm] : A[(size_t)gm * lda + gk]);
      As[kk][mm] = v;
    }
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      int nn, kk;
      if (FORM == 0) { kk = i & 15; nn = i >> 4; } else { nn = i & 63; kk = i >> 6; }
      const int gn = n0 + nn, gk = k0 + kk;
      float v = 0.f;
      if (gn < N && gk < K) v = to_f<T>(FORM == 0 ? B[(size_t)gn * ldb + gk] : B[(size_t)gk * ldb + gn]);
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      float v = acc[i][j];
      if (bias) v += to_f<T>(bias[gn]);
      if (relu) v = fmaxf(v, 0.f);
      if (drop_thr) {
        const uint64_t e = (uint64_t)gm * N + gn;
        v = drop_keep(drop_word(drop_key, e >> 2), (int)(e & 3), drop_thr) ? v * inv_keep : 0.f;
      }
      const size_t o = (size_t)gm * ldc + gn;
      if (mask) v = to_f<T>(mask[o]) > 0.f ? v * mask_scale : 0.f;
      if (residual) v += to_f<T>(residual[o]);
      C[o] = from_f<T>(v);
    }
  }
}

template <typename T>
static void gemm_naive_dispatch(hipStream_t s, const GemmArgs& a) {
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64), block(256);
  const uint32_t thr = a.drop_p > 0.f ? drop_threshold(a.drop_p) : 0u;
#define GN(F)                                                                                                          \
  hipLaunchKernelGGL((gemm_naive_kernel<T, F>), grid, block, 0, s, a.M, a.N, a.K, (const T*)a.A, a.lda, (const T*)a.B, a.ldb, \
                     (T*)a.C, a.ldc, (const T*)a.bias, a.relu, (const T*)a.mask, (const T*)a.residual, a.drop_key, thr,  \
                     1.f / (1.f - a.drop_p), a.mask_scale)
  if (a.form == 0) GN(0); else if (a.form == 1) GN(1); else GN(2);
#undef GN
}

void launch_gemm_naive(hipStream_t s, const GemmArgs& a) {
  if (a.M <= 0 || a.N <= 0) return;
  if (a.dt == F32) gemm_naive_dispatch<float>(s, a);
  else if (a.dt == F16) gemm_naive_dispatch<half_t>(s, a);
  else gemm_naive_dispatch<bf16_t>(s, a);
}

}  // namespace tfm
