// Measurement aids: what this device sustains on the two resources the rooflines are drawn against, so that the
// benchmark can print the measured ceilings beside the published ones.  Not on the training path.
#include "../../include/tfm.h"
#include <algorithm>

#include "common.h"

namespace tfm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// A register-only loop of independent 32x32x16 MFMAs: 8 accumulators per wavefront, 8 wavefronts per block, one block per
// CU slot.  No memory traffic inside the loop: this is the rate the matrix pipes reach at the clock they sustain.
template <bool BF>
__global__ __launch_bounds__(512) void mfma_probe_kernel(float* out, int iters) {
  f32x16 c[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) c[i][e] = 0.f;
  f16x8 ah[2], bh[2];
  bf16x8 ab[2], bb[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v = (float)((threadIdx.x + e + i) & 7) * 0.125f;
      ah[i][e] = (_Float16)v; bh[i][e] = (_Float16)(1.f - v);
      ab[i][e] = (__bf16)v; bb[i][e] = (__bf16)(1.f - v);
    }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (BF) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ab[i & 1], bb[(i >> 1) & 1], c[i], 0, 0, 0);
      else c[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[i & 1], bh[(i >> 1) & 1], c[i], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c[i][e];
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Plain streaming copy: 16 bytes per lane, one access each way per thread, non-temporal (the fastest form of a copy found
// on this device: 6.4-6.5 TB/s read + written over 1 GiB, against 4.8 TB/s for a grid-stride loop over plain accesses).
typedef unsigned int copy_vec __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_probe_kernel(copy_vec* __restrict__ dst, const copy_vec* __restrict__ src, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Re-reads a private region per block with 16-byte loads, 8 in flight per lane: the rate at which a compute unit can pull
// operand tiles in.  Regions of 64 KiB per block stay in the L2 of the block's XCD (16 MiB in all), regions of 512 KiB
// (128 MiB in all) exceed the L2s and are served by the memory side (infinity cache / HBM) through the fabric.
typedef unsigned int fetch_vec __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(1024) void fetch_probe_kernel(const fetch_vec* __restrict__ buf, unsigned region_vecs, int iters, fetch_vec* out) {
  const fetch_vec* base = buf + (size_t)blockIdx.x * region_vecs;
  fetch_vec acc = {0u, 0u, 0u, 0u};
  unsigned idx = threadIdx.x;                              // < 1024 <= region_vecs
  for (int it = 0; it < iters; ++it) {
    fetch_vec v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { v[u] = base[idx]; idx += 1024; if (idx >= region_vecs) idx -= region_vecs; }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) out[threadIdx.x] = acc;   // (keeps the loads; practically never taken)
}

}  // namespace tfm

using namespace tfm;

extern "C" {

int tfm_probe_mfma(int32_t dtype, void* scratch, size_t scratch_bytes, double* tflops, void* stream) {
  if ((dtype != TFM_FP16 && dtype != TFM_BF16) || !scratch || !tflops) return TFM_EINVAL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return TFM_EHIP;
  const int blocks = cus;                                  // one 8-wavefront block per compute unit
  if (scratch_bytes < (size_t)blocks * 512 * sizeof(float)) return TFM_ENOMEM;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return TFM_EHIP;
  const int iters = 20000;
  auto launch = [&](int it) {
    if (dtype == TFM_BF16) hipLaunchKernelGGL((mfma_probe_kernel<true>), dim3(blocks), dim3(512), 0, s, (float*)scratch, it);
    else hipLaunchKernelGGL((mfma_probe_kernel<false>), dim3(blocks), dim3(512), 0, s, (float*)scratch, it);
  };
  launch(100);
  hipEventRecord(e0, s);
  launch(iters);
  hipEventRecord(e1, s);
  float ms = 0.f;
  const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (!ok || hipGetLastError() != hipSuccess) return TFM_EHIP;
  *tflops = (double)blocks * 8.0 * iters * 8.0 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
  return TFM_OK;
}

int tfm_probe_copy(void* dst, const void* src, size_t bytes, double* gbs, void* stream) {
  if (!dst || !src || !gbs || bytes < 16 || bytes % 16 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return TFM_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return TFM_EHIP;
  const size_t n = bytes / 16;
  if ((n + 255) / 256 > 0x7fffffffull) return TFM_EINVAL;
  const unsigned grid = (unsigned)((n + 255) / 256);
  const int reps = 10;
  hipLaunchKernelGGL(copy_probe_kernel, dim3(grid), dim3(256), 0, s, (copy_vec*)dst, (const copy_vec*)src, n);
  hipEventRecord(e0, s);
  for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(copy_probe_kernel, dim3(grid), dim3(256), 0, s, (copy_vec*)dst, (const copy_vec*)src, n);
  hipEventRecord(e1, s);
  float ms = 0.f;
  const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (!ok || hipGetLastError() != hipSuccess) return TFM_EHIP;
  *gbs = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;   // bytes read plus bytes written
  return TFM_OK;
}

int tfm_probe_fetch(const void* buf, size_t bytes, size_t region_bytes, double* gbs_per_cu, double* gbs_total, void* stream) {
  if (!buf || !gbs_per_cu || !gbs_total || ((uintptr_t)buf & 15)) return TFM_EINVAL;
  if (region_bytes < 16384 || region_bytes % 16384 || region_bytes > ((size_t)1 << 30)) return TFM_EINVAL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return TFM_EHIP;
  if (bytes < (size_t)cus * region_bytes + 16384) return TFM_ENOMEM;        // every block's region, plus the result slot
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return TFM_EHIP;
  const fetch_vec* b = (const fetch_vec*)buf;
  fetch_vec* out = (fetch_vec*)((char*)buf + (size_t)cus * region_bytes);
  const unsigned vecs = (unsigned)(region_bytes / 16);
  const int iters = 400;
  hipLaunchKernelGGL(fetch_probe_kernel, dim3(cus), dim3(1024), 0, s, b, vecs, iters, out);
  hipEventRecord(e0, s);
  hipLaunchKernelGGL(fetch_probe_kernel, dim3(cus), dim3(1024), 0, s, b, vecs, iters, out);
  hipEventRecord(e1, s);
  float ms = 0.f;
  const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (!ok || hipGetLastError() != hipSuccess) return TFM_EHIP;
  *gbs_total = (double)cus * 1024.0 * 16.0 * 8.0 * iters / (ms * 1e-3) / 1e9;
  *gbs_per_cu = *gbs_total / cus;
  return TFM_OK;
}

}  // extern "C"
