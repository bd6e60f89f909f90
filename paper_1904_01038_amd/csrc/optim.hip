// Inf/nan scan (+ optional accumulation into the fp32 window buffer), the loss-scale state machine, and the fp32
// master-weight Adam update.  All HBM-bound streaming kernels with 16-byte accesses; reductions use per-block
// partials added in a fixed order (no floating-point atomics), so every result is reproducible.
#include <mutex>

#include "../../include/tfm.h"
#include "common.h"
#include "kernels.h"

namespace tfm {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_VEC = 8;
constexpr int SCAN_MAX_BLOCKS = 2048;

static int scan_blocks(int64_t n) {
  int64_t b = (n + (int64_t)SCAN_THREADS * SCAN_VEC - 1) / ((int64_t)SCAN_THREADS * SCAN_VEC);
  if (b > SCAN_MAX_BLOCKS) b = SCAN_MAX_BLOCKS;
  return b < 1 ? 1 : (int)b;
}
size_t scan_scratch_bytes(int64_t n) { return (size_t)scan_blocks(n) * 2 * sizeof(float); }

// ACC: 0 none, 1 acc = x, 2 acc += x.  n must be a multiple of SCAN_VEC (buffers are padded by the caller).
template <typename T, int ACC>
__global__ __launch_bounds__(SCAN_THREADS) void scan_kernel(const T* __restrict__ x, int64_t n, float* __restrict__ acc,
                                                            float* __restrict__ partial) {
  __shared__ float sh[16];
  float bad = 0.f, sq = 0.f;
  // two vectors in flight per lane, non-temporal: the data is on its way through, nothing here reads it twice
  const int64_t stride = (int64_t)gridDim.x * SCAN_THREADS * SCAN_VEC;
  for (int64_t i = ((int64_t)blockIdx.x * SCAN_THREADS + threadIdx.x) * SCAN_VEC; i < n; i += 2 * stride) {
    const int64_t i1 = i + stride;
    const bool two = i1 < n;
    float v[2][SCAN_VEC];
    load_f_nt<T, SCAN_VEC>(x + i, v[0]);
    if (two) load_f_nt<T, SCAN_VEC>(x + i1, v[1]);
    else {
#pragma unroll
      for (int k = 0; k < SCAN_VEC; ++k) v[1][k] = 0.f;
    }
    float a[2][SCAN_VEC] = {};
    if (ACC == 2) {
      load_f_nt<float, SCAN_VEC>(acc + i, a[0]);
      if (two) load_f_nt<float, SCAN_VEC>(acc + i1, a[1]);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int k = 0; k < SCAN_VEC; ++k) {
        if (!(fabsf(v[u][k]) <= 3.402823466e38f)) bad = 1.f;
        sq += v[u][k] * v[u][k];
      }
    if (ACC == 1) {
      store_f_nt<float, SCAN_VEC>(acc + i, v[0]);
      if (two) store_f_nt<float, SCAN_VEC>(acc + i1, v[1]);
    } else if (ACC == 2) {
#pragma unroll
      for (int k = 0; k < SCAN_VEC; ++k) { a[0][k] += v[0][k]; a[1][k] += v[1][k]; }
      store_f_nt<float, SCAN_VEC>(acc + i, a[0]);
      if (two) store_f_nt<float, SCAN_VEC>(acc + i1, a[1]);
    }
  }
  bad = block_max(bad, sh);
  sq = block_sum(sq, sh);
  if (threadIdx.x == 0) { partial[2 * blockIdx.x] = bad; partial[2 * blockIdx.x + 1] = sq; }
}

__global__ __launch_bounds__(256) void scan_finish_kernel(const float* __restrict__ partial, int nb, float* __restrict__ result,
                                                          DevState* __restrict__ st) {
  __shared__ double shs[256];
  __shared__ float shb[256];
  double sq = 0.0;
  float bad = 0.f;
  for (int i = threadIdx.x; i < nb; i += 256) { bad = fmaxf(bad, partial[2 * i]); sq += (double)partial[2 * i + 1]; }
  shs[threadIdx.x] = sq;
  shb[threadIdx.x] = bad;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) { shs[threadIdx.x] += shs[threadIdx.x + o]; shb[threadIdx.x] = fmaxf(shb[threadIdx.x], shb[threadIdx.x + o]); }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    // a non-finite partial sum also means a non-finite (or overflowing) input
    const float flag = (shb[0] > 0.f || !(fabs(shs[0]) <= 1.7e308)) ? 1.f : 0.f;
    if (result) { result[0] = flag; result[1] = (float)shs[0]; }
    if (st) {
      st->scan_flag = flag;
      st->scan_sumsq = shs[0];
      st->step_overflow = flag > 0.f ? 1 : 0;
      if (flag > 0.f) st->window_overflow = 1;
    }
  }
}

template <typename T>
static void scan_dispatch(hipStream_t s, const void* x, int64_t n, float* result, DevState* st, float* acc, int acc_mode,
                          void* scratch) {
  const int nb = scan_blocks(n);
  dim3 grid(nb), block(SCAN_THREADS);
  if (acc_mode == 1) hipLaunchKernelGGL((scan_kernel<T, 1>), grid, block, 0, s, (const T*)x, n, acc, (float*)scratch);
  else if (acc_mode == 2) hipLaunchKernelGGL((scan_kernel<T, 2>), grid, block, 0, s, (const T*)x, n, acc, (float*)scratch);
  else hipLaunchKernelGGL((scan_kernel<T, 0>), grid, block, 0, s, (const T*)x, n, acc, (float*)scratch);
  hipLaunchKernelGGL(scan_finish_kernel, dim3(1), dim3(256), 0, s, (const float*)scratch, nb, result, st);
}

void launch_scan(hipStream_t s, int dt, const void* x, int64_t n, float* result, DevState* st, float* acc, int acc_mode,
                 void* scratch) {
  if (dt == F32) scan_dispatch<float>(s, x, n, result, st, acc, acc_mode, scratch);
  else if (dt == F16) scan_dispatch<half_t>(s, x, n, result, st, acc, acc_mode, scratch);
  else scan_dispatch<bf16_t>(s, x, n, result, st, acc, acc_mode, scratch);
}

// ---- the scan for callers that cannot allocate ------------------------------------------------------------------------------
// Same kernels as launch_scan; the per-block partials live in a file-scope device array instead of caller memory.  Every
// block writes its own two floats and the finishing kernel reads exactly the blocks of this launch, so nothing has to be
// cleared between calls.  In host code the array's name is only a handle: its device address is looked up once per
// device and kept.
static __device__ __align__(256) float scan_static_scratch[2 * SCAN_MAX_BLOCKS];     // 16 KiB on every device the library runs on
constexpr int SCAN_STATIC_DEVICES = 64;
static float* g_scan_static_ptr[SCAN_STATIC_DEVICES];
static std::mutex g_scan_static_mutex;

// device address of scan_static_scratch on the current device, or null with *err set
static float* scan_static_address(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= SCAN_STATIC_DEVICES) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scan_static_mutex);
  if (!g_scan_static_ptr[dev]) {
    float* p = nullptr;
    *err = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scan_static_scratch));
    if (*err != hipSuccess) return nullptr;
    g_scan_static_ptr[dev] = p;
  }
  return g_scan_static_ptr[dev];
}

// ---- conversion ---------------------------------------------------------------------------------------------------------
// 8 elements per thread in one pass with non-temporal accesses (the whole-buffer conversions move hundreds of megabytes
// that nothing reads again soon); the last n % 8 elements, and buffers that are not 16-byte aligned, go one by one.
template <typename S, typename D>
__global__ __launch_bounds__(256) void convert_vec_kernel(const S* __restrict__ src, D* __restrict__ dst, int64_t n8) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n8) return;
  float v[8];
  load_f_nt<S, 8>(src + i, v);
  store_f_nt<D, 8>(dst + i, v);
}
template <typename S, typename D>
__global__ void convert_kernel(const S* __restrict__ src, D* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = from_f<D>(to_f<S>(src[i]));
}
template <typename S, typename D>
static void convert_typed(hipStream_t s, const S* src, D* dst, int64_t n) {
  int64_t n8 = 0;
  if ((((uintptr_t)src | (uintptr_t)dst) & 31) == 0) {
    n8 = n / 8 * 8;
    if (n8) hipLaunchKernelGGL((convert_vec_kernel<S, D>), dim3((unsigned)((n8 / 8 + 255) / 256)), dim3(256), 0, s, src, dst, n8);
  }
  if (n > n8) {
    int64_t b = (n - n8 + 255) / 256;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL((convert_kernel<S, D>), dim3((unsigned)b), dim3(256), 0, s, src + n8, dst + n8, n - n8);
  }
}
template <typename S>
static void convert_from(hipStream_t s, const void* src, int dst_dt, void* dst, int64_t n) {
  if (dst_dt == F32) convert_typed<S, float>(s, (const S*)src, (float*)dst, n);
  else if (dst_dt == F16) convert_typed<S, half_t>(s, (const S*)src, (half_t*)dst, n);
  else convert_typed<S, bf16_t>(s, (const S*)src, (bf16_t*)dst, n);
}
void launch_convert(hipStream_t s, int src_dt, const void* src, int dst_dt, void* dst, int64_t n) {
  if (n <= 0) return;
  if (src_dt == F32) convert_from<float>(s, src, dst_dt, dst, n);
  else if (src_dt == F16) convert_from<half_t>(s, src, dst_dt, dst, n);
  else convert_from<bf16_t>(s, src, dst_dt, dst, n);
}

// ---- loss-scale state machine + Adam scalars (one thread) -----------------------------------------------------------------
// Overflow anywhere in the window: skip, halve the scale, restart the clean counter.  Otherwise take an optimiser
// step and double the scale after `scale_window` clean updates (Implementation, Mixed precision).
__global__ void scaler_update_kernel(DevState* st, long long ntokens, float clip_norm, float beta1, float beta2,
                                     int scale_window, float min_scale, int dynamic) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  if (st->window_overflow) {
    st->skipped = 1;
    st->grad_norm = __uint_as_float(0x7fc00000u);
    st->grad_mult = 0.f;
    if (dynamic) st->loss_scale *= 0.5f;
    st->clean_steps = 0;
  } else {
    st->skipped = 0;
    const double inv = 1.0 / ((double)st->loss_scale * (double)(ntokens > 0 ? ntokens : 1));
    const double gnorm = sqrt(st->scan_sumsq) * inv;
    double coef = 1.0;
    if (clip_norm > 0.f && gnorm > (double)clip_norm) coef = (double)clip_norm / gnorm;
    st->grad_norm = (float)gnorm;
    st->grad_mult = (float)(inv * coef);
    st->num_updates += 1;
    const double t = (double)st->num_updates;
    st->bc1 = (float)(1.0 - pow((double)beta1, t));
    st->bc2 = (float)(1.0 - pow((double)beta2, t));
    st->clean_steps += 1;
    if (dynamic && st->clean_steps == scale_window) { st->loss_scale *= 2.f; st->clean_steps = 0; }
  }
  st->window_overflow = 0;
  st->scale_too_small = st->loss_scale < min_scale ? 1 : 0;       // (cleared again once the scale is back at or above the minimum)
}
void launch_scaler_update(hipStream_t s, DevState* st, long long ntokens, float clip_norm, float beta1, float beta2,
                          int scale_window, float min_scale, int dynamic) {
  hipLaunchKernelGGL(scaler_update_kernel, dim3(1), dim3(64), 0, s, st, ntokens, clip_norm, beta1, beta2, scale_window, min_scale, dynamic);
}

// ---- Adam -------------------------------------------------------------------------------------------------------------------
// Per parameter: read w, m, v (12 B) and the gradient (2 or 4 B), write w, m, v (12 B) and the half model copy (2 B).
// One pass, no loop: a thread owns ADAM_UN groups of ADAM_VEC consecutive parameters, a block's width apart, issues all their
// loads before the first result is needed, and touches everything with non-temporal accesses (nothing here is read again
// before the next forward pass has gone through hundreds of megabytes).  Measured on the big model's 210 M parameters
// against a grid-stride loop over plain accesses: 1.27 -> 1.01 ms (4.6 -> 5.8 TB/s).
constexpr int ADAM_VEC = 4, ADAM_UN = 4, ADAM_THREADS = 256;
template <typename GT, typename HT>
__global__ __launch_bounds__(ADAM_THREADS) void adam_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                                                            const GT* __restrict__ g, HT* __restrict__ hcopy, int64_t n, float lr,
                                                            float beta1, float beta2, float eps, const DevState* __restrict__ st,
                                                            float grad_mult, float bc1, float bc2, float wd) {
  if (st) {
    if (st->skipped) return;
    grad_mult = st->grad_mult; bc1 = st->bc1; bc2 = st->bc2;
  }
  const float step = lr / bc1, rbc2 = 1.f / bc2;
  const int64_t i0 = ((int64_t)blockIdx.x * ADAM_UN * ADAM_THREADS + threadIdx.x) * ADAM_VEC;
  float wv[ADAM_UN][ADAM_VEC], mv[ADAM_UN][ADAM_VEC], vv[ADAM_UN][ADAM_VEC], gv[ADAM_UN][ADAM_VEC];
#pragma unroll
  for (int u = 0; u < ADAM_UN; ++u) {
    const int64_t i = i0 + (int64_t)u * ADAM_THREADS * ADAM_VEC;
    if (i < n) {
      load_f_nt<float, ADAM_VEC>(w + i, wv[u]);
      load_f_nt<float, ADAM_VEC>(m + i, mv[u]);
      load_f_nt<float, ADAM_VEC>(v + i, vv[u]);
      load_f_nt<GT, ADAM_VEC>(g + i, gv[u]);
    }
  }
#pragma unroll
  for (int u = 0; u < ADAM_UN; ++u) {
    const int64_t i = i0 + (int64_t)u * ADAM_THREADS * ADAM_VEC;
    if (i < n) {
#pragma unroll
      for (int k = 0; k < ADAM_VEC; ++k) {
        const float gg = gv[u][k] * grad_mult + wd * wv[u][k];
        mv[u][k] = beta1 * mv[u][k] + (1.f - beta1) * gg;
        vv[u][k] = beta2 * vv[u][k] + (1.f - beta2) * gg * gg;
        wv[u][k] -= step * mv[u][k] / (sqrtf(vv[u][k] * rbc2) + eps);
      }
      store_f_nt<float, ADAM_VEC>(w + i, wv[u]);
      store_f_nt<float, ADAM_VEC>(m + i, mv[u]);
      store_f_nt<float, ADAM_VEC>(v + i, vv[u]);
      if (hcopy) store_f_nt<HT, ADAM_VEC>(hcopy + i, wv[u]);
    }
  }
}

template <typename GT>
static void adam_dispatch(hipStream_t s, const AdamArgs& a) {
  const int64_t per_block = (int64_t)ADAM_THREADS * ADAM_VEC * ADAM_UN;
  dim3 grid((unsigned)((a.n + per_block - 1) / per_block)), block(ADAM_THREADS);      // n < 2^31 * 4096: the grid fits
#define ADAM(HT)                                                                                                       \
  hipLaunchKernelGGL((adam_kernel<GT, HT>), grid, block, 0, s, a.w, a.m, a.v, (const GT*)a.g, (HT*)a.half_copy, a.n, a.lr, \
                     a.beta1, a.beta2, a.eps, a.st, a.grad_mult, a.bc1, a.bc2, a.weight_decay)
  if (a.hdt == F16) ADAM(half_t); else if (a.hdt == BF16) ADAM(bf16_t); else ADAM(float);
#undef ADAM
}
void launch_adam(hipStream_t s, const AdamArgs& a) {
  if (a.n <= 0) return;
  if (a.gdt == F32) adam_dispatch<float>(s, a);
  else if (a.gdt == F16) adam_dispatch<half_t>(s, a);
  else adam_dispatch<bf16_t>(s, a);
}

}  // namespace tfm

extern "C" int tfm_op_scan_noalloc(int32_t dtype, const void* x, int64_t n, float* result, void* stream) {
  using namespace tfm;
  if (dtype < 0 || dtype > 2 || !x || !result || n < 0 || n % 8) { set_global_error("tfm_op_scan_noalloc: bad argument (dtype, null pointer, or n not a multiple of 8)"); return TFM_EINVAL; }
  if (n > TFM_SCAN_NOALLOC_MAX_N) { set_global_error("tfm_op_scan_noalloc: n exceeds TFM_SCAN_NOALLOC_MAX_N"); return TFM_EINVAL; }
  hipError_t e = hipSuccess;
  float* scratch = scan_static_address(&e);
  if (!scratch) { set_global_error(hipGetErrorString(e)); return TFM_EHIP; }
  launch_scan((hipStream_t)stream, dtype, x, n, result, nullptr, nullptr, 0, scratch);
  e = hipGetLastError();
  if (e != hipSuccess) { set_global_error(hipGetErrorString(e)); return TFM_EHIP; }
  return TFM_OK;
}
