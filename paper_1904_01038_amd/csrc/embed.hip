// Embedding forward (gather, scale by sqrt(d), add the sinusoidal position, dropout) and backward (per-token
// segmented sum into the shared embedding gradient).  HBM-bound; one wavefront per row, 16-byte accesses.
#include "common.h"
#include "kernels.h"

namespace tfm {

constexpr int EV = 8;

template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const T* __restrict__ E, const int* __restrict__ ids,
                                                        const int* __restrict__ pos, const float* __restrict__ pe,
                                                        T* __restrict__ out, int rows, int d, float scale, uint64_t key,
                                                        uint32_t thr, float inv_keep) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T* e = E + (size_t)ids[row] * d;
  const float* p = pe + (size_t)pos[row] * d;
  for (int col = lane * EV; col < d; col += 64 * EV) {
    float v[EV];
    load_f<T, EV>(e + col, v);
#pragma unroll
    for (int i = 0; i < EV; ++i) v[i] = scale * v[i] + p[col + i];
    if (thr) drop_apply<EV>(v, key, (uint64_t)row * d + col, thr, inv_keep);
    store_f<T, EV>(out + (size_t)row * d + col, v);
  }
}

void launch_embed_fwd(hipStream_t s, int dt, const void* E, const int* ids, const int* pos, const float* pe, void* out,
                      int rows, int d, uint64_t key, float p) {
  if (rows <= 0) return;
  const uint32_t thr = p > 0.f ? drop_threshold(p) : 0u;
  const float inv_keep = 1.f / (1.f - p), scale = sqrtf((float)d);
  dim3 grid((rows + 3) / 4), block(256);
  if (dt == F32) hipLaunchKernelGGL((embed_fwd_kernel<float>), grid, block, 0, s, (const float*)E, ids, pos, pe, (float*)out, rows, d, scale, key, thr, inv_keep);
  else if (dt == F16) hipLaunchKernelGGL((embed_fwd_kernel<half_t>), grid, block, 0, s, (const half_t*)E, ids, pos, pe, (half_t*)out, rows, d, scale, key, thr, inv_keep);
  else hipLaunchKernelGGL((embed_fwd_kernel<bf16_t>), grid, block, 0, s, (const bf16_t*)E, ids, pos, pe, (bf16_t*)out, rows, d, scale, key, thr, inv_keep);
}

// One block per distinct token.  Its occurrences (host-built list, fixed order) are summed in fp32 registers and
// added to the token's gradient row, which already holds the output-projection contribution.  No atomics: frequent
// tokens under a Zipf law would serialise them, and the result would depend on the order.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(T* __restrict__ gE, const int* __restrict__ uniq,
                                                        const int* __restrict__ start, const int* __restrict__ entries,
                                                        const T* __restrict__ dx0, const T* __restrict__ dx1, int d, float scale,
                                                        uint64_t key0, uint64_t key1, uint32_t thr, float inv_keep) {
  const int u = blockIdx.x;
  const int b = start[u], e = start[u + 1];
  T* grow = gE + (size_t)uniq[u] * d;
  for (int col = threadIdx.x * 4; col < d; col += 256 * 4) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k = b; k < e; ++k) {
      const int ent = entries[k];
      const int stream = ent >> 30, row = ent & 0x3fffffff;
      const T* src = (stream ? dx1 : dx0) + (size_t)row * d + col;
      float v[4];
      load_f<T, 4>(src, v);
      if (thr) drop_apply<4>(v, stream ? key1 : key0, (uint64_t)row * d + col, thr, inv_keep);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] += v[i];
    }
    float g[4];
    load_f<T, 4>(grow + col, g);
#pragma unroll
    for (int i = 0; i < 4; ++i) g[i] += scale * acc[i];
    store_f<T, 4>(grow + col, g);
  }
}

void launch_embed_bwd(hipStream_t s, int dt, void* gE, const int* uniq, const int* start, const int* entries, int n_uniq,
                      const void* dx0, const void* dx1, int d, uint64_t key0, uint64_t key1, float p) {
  if (n_uniq <= 0) return;
  const uint32_t thr = p > 0.f ? drop_threshold(p) : 0u;
  const float inv_keep = 1.f / (1.f - p), scale = sqrtf((float)d);
  dim3 grid(n_uniq), block(256);
  if (dt == F32) hipLaunchKernelGGL((embed_bwd_kernel<float>), grid, block, 0, s, (float*)gE, uniq, start, entries, (const float*)dx0, (const float*)dx1, d, scale, key0, key1, thr, inv_keep);
  else if (dt == F16) hipLaunchKernelGGL((embed_bwd_kernel<half_t>), grid, block, 0, s, (half_t*)gE, uniq, start, entries, (const half_t*)dx0, (const half_t*)dx1, d, scale, key0, key1, thr, inv_keep);
  else hipLaunchKernelGGL((embed_bwd_kernel<bf16_t>), grid, block, 0, s, (bf16_t*)gE, uniq, start, entries, (const bf16_t*)dx0, (const bf16_t*)dx1, d, scale, key0, key1, thr, inv_keep);
}

__global__ void dropout_mask_kernel(uint64_t key, uint32_t thr, uint8_t* out, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  out[e] = drop_keep(drop_word(key, (uint64_t)e >> 2), (int)(e & 3), thr) ? 1 : 0;
}
void launch_dropout_mask(hipStream_t s, uint64_t key, float p, uint8_t* out, int64_t n) {
  if (n <= 0) return;
  hipLaunchKernelGGL(dropout_mask_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, key, drop_threshold(p), out, n);
}

uint64_t dropout_site_key(uint64_t seed, uint64_t step, int stream, int layer, int sub) {
  const uint64_t site = (uint64_t)(1000 * stream + 10 * (layer + 1) + sub);
  uint64_t k = mix64(seed + GOLDEN);
  k = mix64(k ^ (step * 0xD1B54A32D192ED03ull));
  k = mix64(k ^ (site * 0x8CB92BA72F3D8DD7ull));
  return k;
}

}  // namespace tfm
