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
                                                        uint32_t thr, float inv_keep, const T* __restrict__ alt) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  // a negative id -1-k selects row k of `alt` (adaptive inputs: the projected vectors of tail-cluster tokens)
  const int id = ids[row];
  const T* e = id >= 0 ? E + (size_t)id * d : alt + (size_t)(-1 - id) * d;
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
                      int rows, int d, uint64_t key, float p, const void* alt) {
  if (rows <= 0) return;
  const uint32_t thr = p > 0.f ? drop_threshold(p) : 0u;
  const float inv_keep = 1.f / (1.f - p), scale = sqrtf((float)d);
  dim3 grid((rows + 3) / 4), block(256);
  if (dt == F32) hipLaunchKernelGGL((embed_fwd_kernel<float>), grid, block, 0, s, (const float*)E, ids, pos, pe, (float*)out, rows, d, scale, key, thr, inv_keep, (const float*)alt);
  else if (dt == F16) hipLaunchKernelGGL((embed_fwd_kernel<half_t>), grid, block, 0, s, (const half_t*)E, ids, pos, pe, (half_t*)out, rows, d, scale, key, thr, inv_keep, (const half_t*)alt);
  else hipLaunchKernelGGL((embed_fwd_kernel<bf16_t>), grid, block, 0, s, (const bf16_t*)E, ids, pos, pe, (bf16_t*)out, rows, d, scale, key, thr, inv_keep, (const bf16_t*)alt);
}

// Embedding gradient.  The host groups the occurrences of every distinct token (fixed order) and cuts each group into
// segments of at most EMB_SEG occurrences, so that a frequent token under the Zipf law does not serialise one block.
// Kernel 1: one block per segment; its 4 wavefronts take occurrences round-robin, each lane owning 8-column chunks of
// the row, fp32 registers; LDS combines the 4 wavefronts in a fixed order.  A single-segment token adds straight into
// its gradient row (which already holds the output-projection contribution); a multi-segment token writes an fp32
// partial row.  Kernel 2: one block per multi-segment token adds its partial rows in order.  No atomics.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void embed_bwd_kernel(T* __restrict__ gE, float* __restrict__ partial, const int* __restrict__ seg_tok,
                                                        const int* __restrict__ seg_beg, const int* __restrict__ seg_end,
                                                        const int* __restrict__ seg_dst, const int* __restrict__ entries,
                                                        const T* __restrict__ dx0, const T* __restrict__ dx1, int d, float scale,
                                                        uint64_t key0, uint64_t key1, uint32_t thr, float inv_keep) {
  extern __shared__ float lds[];        // [4][d]
  const int sgm = blockIdx.x, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = seg_beg[sgm], e = seg_end[sgm];
  float acc[NCH][EV];
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int i = 0; i < EV; ++i) acc[c][i] = 0.f;
  for (int k = b + w; k < e; k += 4) {
    const int ent = entries[k];
    const int stream = ent >> 30, row = ent & 0x3fffffff;
    const T* src = (stream ? dx1 : dx0) + (size_t)row * d;
    const uint64_t key = stream ? key1 : key0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int col = (lane + 64 * c) * EV;
      if (col < d) {
        float v[EV];
        load_f<T, EV>(src + col, v);
        if (thr) drop_apply<EV>(v, key, (uint64_t)row * d + col, thr, inv_keep);
#pragma unroll
        for (int i = 0; i < EV; ++i) acc[c][i] += v[i];
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int col = (lane + 64 * c) * EV;
    if (col < d) {
#pragma unroll
      for (int i = 0; i < EV; ++i) lds[w * d + col + i] = acc[c][i];
    }
  }
  __syncthreads();
  const int dst = seg_dst[sgm];
  T* grow = gE + (size_t)seg_tok[sgm] * d;
  for (int col = threadIdx.x * 4; col < d; col += 256 * 4) {
    float t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = (lds[col + i] + lds[d + col + i]) + (lds[2 * d + col + i] + lds[3 * d + col + i]);
    if (dst < 0) {
      float g[4];
      load_f<T, 4>(grow + col, g);
#pragma unroll
      for (int i = 0; i < 4; ++i) g[i] += scale * t[i];
      store_f<T, 4>(grow + col, g);
    } else {
      store_f<float, 4>(partial + (size_t)dst * d + col, t);
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_merge_kernel(T* __restrict__ gE, const float* __restrict__ partial,
                                                              const int* __restrict__ mt_tok, const int* __restrict__ mt_row0,
                                                              const int* __restrict__ mt_n, int d, float scale) {
  const int k = blockIdx.x;
  const int r0 = mt_row0[k], n = mt_n[k];
  T* grow = gE + (size_t)mt_tok[k] * d;
  for (int col = threadIdx.x * 4; col < d; col += 256 * 4) {
    float t[4] = {0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < n; ++r) {
      float v[4];
      load_f<float, 4>(partial + (size_t)(r0 + r) * d + col, v);
#pragma unroll
      for (int i = 0; i < 4; ++i) t[i] += v[i];
    }
    float g[4];
    load_f<T, 4>(grow + col, g);
#pragma unroll
    for (int i = 0; i < 4; ++i) g[i] += scale * t[i];
    store_f<T, 4>(grow + col, g);
  }
}

template <typename T>
static void embed_bwd_dispatch(hipStream_t s, const EmbedBwdArgs& a) {
  const uint32_t thr = a.p > 0.f ? drop_threshold(a.p) : 0u;
  const float inv_keep = 1.f / (1.f - a.p), scale = sqrtf((float)a.d);
  const size_t shm = (size_t)4 * a.d * sizeof(float);
#define EMB_BWD(N)                                                                                                             \
  hipLaunchKernelGGL((embed_bwd_kernel<T, N>), dim3(a.n_seg), dim3(256), shm, s, (T*)a.gE, a.partial, a.seg_tok, a.seg_beg, a.seg_end, \
                     a.seg_dst, a.entries, (const T*)a.dx0, (const T*)a.dx1, a.d, scale, a.key0, a.key1, thr, inv_keep)
  if (a.d <= 512) EMB_BWD(1); else if (a.d <= 1024) EMB_BWD(2); else if (a.d <= 1536) EMB_BWD(3); else EMB_BWD(4);   // d <= 2048
#undef EMB_BWD
  if (a.n_multi > 0)
    hipLaunchKernelGGL((embed_bwd_merge_kernel<T>), dim3(a.n_multi), dim3(256), 0, s, (T*)a.gE, (const float*)a.partial, a.mt_tok,
                       a.mt_row0, a.mt_n, a.d, scale);
}

void launch_embed_bwd(hipStream_t s, const EmbedBwdArgs& a) {
  if (a.n_seg <= 0) return;
  if (a.dt == F32) embed_bwd_dispatch<float>(s, a);
  else if (a.dt == F16) embed_bwd_dispatch<half_t>(s, a);
  else embed_bwd_dispatch<bf16_t>(s, a);
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
