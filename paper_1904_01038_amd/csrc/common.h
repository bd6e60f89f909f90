// Shared device-side helpers for the gfx950 kernels: storage types, conversions, wavefront reductions and the
// counter-based dropout generator.  Wavefronts are 64 lanes wide on CDNA4; every reduction below assumes that.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tfm {

enum DType : int { F32 = 0, F16 = 1, BF16 = 2 };

typedef _Float16 half_t;
struct bf16_t { uint16_t x; };

static inline size_t dtype_size(int dt) { return dt == F32 ? 4 : 2; }

// ---- conversions (round to nearest even; a value beyond the half range becomes inf, which is what the
// overflow detection of the mixed-precision path relies on) -------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<half_t>(half_t v) { return (float)v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf16_bits_to_f(v.x); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ half_t from_f<half_t>(float v) { return (half_t)v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { bf16_t r; r.x = f_to_bf16_bits(v); return r; }

// ---- vectors of VEC elements moved with one memory instruction ------------------------------------------------------
template <typename T, int VEC> struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };

template <typename T, int VEC> __device__ __forceinline__ void load_f(const T* p, float (&out)[VEC]) {
  Pack<T, VEC> k = *reinterpret_cast<const Pack<T, VEC>*>(p);
#pragma unroll
  for (int i = 0; i < VEC; ++i) out[i] = to_f<T>(k.v[i]);
}
template <typename T, int VEC> __device__ __forceinline__ void store_f(T* p, const float (&in)[VEC]) {
  Pack<T, VEC> k;
#pragma unroll
  for (int i = 0; i < VEC; ++i) k.v[i] = from_f<T>(in[i]);
  *reinterpret_cast<Pack<T, VEC>*>(p) = k;
}

// The same for data that is touched once (optimiser state, gradients on their way to the update): non-temporal accesses, which
// leave the caches to the data that is used again.  On this device a streaming kernel built on them moves 15-30 % more bytes
// per second than one built on plain accesses.
template <int BYTES> struct RawVec;
template <> struct RawVec<16> { typedef unsigned int type __attribute__((ext_vector_type(4))); };
template <> struct RawVec<8> { typedef unsigned int type __attribute__((ext_vector_type(2))); };
template <> struct RawVec<4> { typedef unsigned int type; };
template <typename T, int VEC> __device__ __forceinline__ void load_f_nt(const T* p, float (&out)[VEC]) {
  constexpr int B = (int)sizeof(T) * VEC;
  if constexpr (B == 32) {
    float lo[VEC / 2], hi[VEC / 2];
    load_f_nt<T, VEC / 2>(p, lo);
    load_f_nt<T, VEC / 2>(p + VEC / 2, hi);
#pragma unroll
    for (int i = 0; i < VEC / 2; ++i) { out[i] = lo[i]; out[VEC / 2 + i] = hi[i]; }
  } else {
    typedef typename RawVec<B>::type R;
    const R r = __builtin_nontemporal_load(reinterpret_cast<const R*>(p));
    Pack<T, VEC> k;
    __builtin_memcpy(&k, &r, B);
#pragma unroll
    for (int i = 0; i < VEC; ++i) out[i] = to_f<T>(k.v[i]);
  }
}
template <typename T, int VEC> __device__ __forceinline__ void store_f_nt(T* p, const float (&in)[VEC]) {
  constexpr int B = (int)sizeof(T) * VEC;
  if constexpr (B == 32) {
    float lo[VEC / 2], hi[VEC / 2];
#pragma unroll
    for (int i = 0; i < VEC / 2; ++i) { lo[i] = in[i]; hi[i] = in[VEC / 2 + i]; }
    store_f_nt<T, VEC / 2>(p, lo);
    store_f_nt<T, VEC / 2>(p + VEC / 2, hi);
  } else {
    typedef typename RawVec<B>::type R;
    Pack<T, VEC> k;
#pragma unroll
    for (int i = 0; i < VEC; ++i) k.v[i] = from_f<T>(in[i]);
    R r;
    __builtin_memcpy(&r, &k, B);
    __builtin_nontemporal_store(r, reinterpret_cast<R*>(p));
  }
}

// ---- reductions -------------------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Block-wide reductions for blockDim.x a multiple of 64, up to 1024 threads.  `sh` holds >= 16 floats.  Every
// thread receives the result.  The summation order is fixed, so results are reproducible.
__device__ __forceinline__ float block_sum(float v, float* sh) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += sh[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float* sh) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = sh[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, sh[i]);
  return t;
}

// ---- dropout: counter-based keep bits -----------------------------------------------------------------------------------
// Element e of an activation uses the 16-bit field (e & 3) of word mix64(key + (e >> 2) * GOLDEN); it is kept when
// that field is >= floor(p * 65536).  mix64 is the finaliser of the published splitmix64 generator.
constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t drop_word(uint64_t key, uint64_t group) { return mix64(key + group * GOLDEN); }
__host__ __device__ __forceinline__ bool drop_keep(uint64_t word, int field, uint32_t thr) {
  return ((uint32_t)(word >> (16 * field)) & 0xffffu) >= thr;
}
static inline uint32_t drop_threshold(float p) { return (uint32_t)floor((double)p * 65536.0); }

// Applies inverted dropout to VEC (multiple of 4) consecutive elements starting at element index e0 (e0 % 4 == 0).
template <int VEC> __device__ __forceinline__ void drop_apply(float (&v)[VEC], uint64_t key, uint64_t e0, uint32_t thr, float inv_keep) {
#pragma unroll
  for (int g = 0; g < VEC / 4; ++g) {
    const uint64_t w = drop_word(key, (e0 >> 2) + g);
#pragma unroll
    for (int f = 0; f < 4; ++f) v[g * 4 + f] = drop_keep(w, f, thr) ? v[g * 4 + f] * inv_keep : 0.f;
  }
}

}  // namespace tfm
