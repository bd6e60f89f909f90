// Row movers for adaptive input embeddings and the adaptive softmax (Applications, language modeling): tokens of a
// tail cluster are gathered into compact matrices, pushed through the cluster's narrow table and projection with the
// ordinary GEMMs, and scattered back.  All index lists come from the host (it has the token ids), so every kernel is
// a plain coalesced copy or add; nothing here uses atomics.
#include "common.h"
#include "kernels.h"

namespace tfm {

// dst[k][j] = src[idx[k]][j], j < width
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T* __restrict__ src, int ld_src, const int* __restrict__ idx,
                                                          T* __restrict__ dst, int width, int n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)n * width) return;
  const int k = (int)(i / width), j = (int)(i - (long long)k * width);
  dst[i] = src[(size_t)idx[k] * ld_src + j];
}
// dst[k][j] = scale * dropout-backward(dx[idx[k]][j]) with the forward's keep bits of element (row, j) of a [rows, d] site
template <typename T>
__global__ __launch_bounds__(256) void gather_dx_kernel(const T* __restrict__ dx, const int* __restrict__ idx, T* __restrict__ dst, int d,
                                                        int n, float scale, uint64_t key, uint32_t thr, float inv_keep) {
  const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;      // 4 elements = one 64-bit word of keep bits
  if (i >= (long long)n * d) return;
  const int k = (int)(i / d), j = (int)(i - (long long)k * d);
  const int row = idx[k];
  float v[4];
  load_f<T, 4>(dx + (size_t)row * d + j, v);
  if (thr) drop_apply<4>(v, key, (uint64_t)row * d + j, thr, inv_keep);
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] *= scale;
  store_f<T, 4>(dst + i, v);
}
// dst[idx[k]][j] += src[k][j]; the idx are distinct
template <typename T>
__global__ __launch_bounds__(256) void scatter_add_rows_kernel(T* __restrict__ dst, int ld_dst, const int* __restrict__ idx,
                                                               const T* __restrict__ src, int width, int n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)n * width) return;
  const int k = (int)(i / width), j = (int)(i - (long long)k * width);
  T* p = dst + (size_t)idx[k] * ld_dst + j;
  *p = from_f<T>(to_f<T>(*p) + to_f<T>(src[i]));
}
__global__ __launch_bounds__(256) void scatter_add_f32_kernel(float* __restrict__ a, float* __restrict__ b, const int* __restrict__ idx,
                                                              const float* __restrict__ sa, const float* __restrict__ sb, int n) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n) return;
  a[idx[k]] += sa[k];
  b[idx[k]] += sb[k];
}
// dst[tok[s]][j] += sum over e in [beg[s], end[s]) of src[entries[e]][j], one block per segment (distinct tokens),
// entries in ascending order: a fixed summation order
template <typename T>
__global__ __launch_bounds__(256) void segsum_add_rows_kernel(T* __restrict__ dst, const T* __restrict__ src, int width,
                                                              const int* __restrict__ tok, const int* __restrict__ beg,
                                                              const int* __restrict__ end, const int* __restrict__ entries) {
  const int s = blockIdx.x, b = beg[s], e = end[s];
  T* row = dst + (size_t)tok[s] * width;
  for (int j = threadIdx.x; j < width; j += 256) {
    float acc = 0.f;
    for (int k = b; k < e; ++k) acc += to_f<T>(src[(size_t)entries[k] * width + j]);
    row[j] = from_f<T>(to_f<T>(row[j]) + acc);
  }
}

// Decoding with an adaptive softmax: the scores of one cluster's tokens join the row of "virtual logits" over the whole
// vocabulary, virt[r][col0 + j] = z[r][j] + offset[r]; for a tail cluster offset = (head score of the cluster's entry) - (the
// cluster's own log-sum-exp), for the head's tokens 0.  The log-sum-exp of a finished row is then the head's, and a row's
// log-softmax gives log p_head(cluster) + log p_cluster(token) for every tail token.
template <typename T>
__global__ __launch_bounds__(256) void adaptive_virtual_kernel(const T* __restrict__ z, int ldz, int width, T* __restrict__ virt, int ldv, int col0,
                                                               const T* __restrict__ head, int ldh, int entry, const float* __restrict__ lse) {
  const int r = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  if (j >= width) return;
  const float off = entry >= 0 ? to_f<T>(head[(size_t)r * ldh + entry]) - lse[r] : 0.f;
  virt[(size_t)r * ldv + col0 + j] = from_f<T>(to_f<T>(z[(size_t)r * ldz + j]) + off);
}

#define BY_DTYPE(CALL)                                  \
  do {                                                  \
    if (dt == F32) { typedef float T; CALL; }           \
    else if (dt == F16) { typedef half_t T; CALL; }     \
    else { typedef bf16_t T; CALL; }                    \
  } while (0)

static inline unsigned blocks_for(long long n) { return (unsigned)((n + 255) / 256); }

void launch_gather_rows(hipStream_t s, int dt, const void* src, int ld_src, const int* idx, void* dst, int width, int n) {
  if (n <= 0) return;
  BY_DTYPE(hipLaunchKernelGGL((gather_rows_kernel<T>), dim3(blocks_for((long long)n * width)), dim3(256), 0, s, (const T*)src, ld_src, idx,
                              (T*)dst, width, n));
}
void launch_gather_dx(hipStream_t s, int dt, const void* dx, const int* idx, void* dst, int d, int n, float scale, uint64_t key, float p) {
  if (n <= 0) return;
  const uint32_t thr = p > 0.f ? drop_threshold(p) : 0u;
  const float inv_keep = 1.f / (1.f - p);
  BY_DTYPE(hipLaunchKernelGGL((gather_dx_kernel<T>), dim3(blocks_for((long long)n * d / 4)), dim3(256), 0, s, (const T*)dx, idx, (T*)dst, d, n,
                              scale, key, thr, inv_keep));
}
void launch_scatter_add_rows(hipStream_t s, int dt, void* dst, int ld_dst, const int* idx, const void* src, int width, int n) {
  if (n <= 0) return;
  BY_DTYPE(hipLaunchKernelGGL((scatter_add_rows_kernel<T>), dim3(blocks_for((long long)n * width)), dim3(256), 0, s, (T*)dst, ld_dst, idx,
                              (const T*)src, width, n));
}
void launch_scatter_add_f32(hipStream_t s, float* a, float* b, const int* idx, const float* sa, const float* sb, int n) {
  if (n <= 0) return;
  hipLaunchKernelGGL(scatter_add_f32_kernel, dim3(blocks_for(n)), dim3(256), 0, s, a, b, idx, sa, sb, n);
}
void launch_adaptive_virtual(hipStream_t s, int dt, const void* z, int ldz, int width, void* virt, int ldv, int col0, const void* head, int ldh,
                             int entry, const float* lse, int rows) {
  if (rows <= 0 || width <= 0) return;
  BY_DTYPE(hipLaunchKernelGGL((adaptive_virtual_kernel<T>), dim3(blocks_for(width), rows), dim3(256), 0, s, (const T*)z, ldz, width, (T*)virt, ldv,
                              col0, (const T*)head, ldh, entry, lse));
}
void launch_segsum_add_rows(hipStream_t s, int dt, void* dst, const void* src, int width, const int* tok, const int* beg, const int* end,
                            const int* entries, int n_seg) {
  if (n_seg <= 0) return;
  BY_DTYPE(hipLaunchKernelGGL((segsum_add_rows_kernel<T>), dim3(n_seg), dim3(256), 0, s, (T*)dst, (const T*)src, width, tok, beg, end, entries));
}

}  // namespace tfm
