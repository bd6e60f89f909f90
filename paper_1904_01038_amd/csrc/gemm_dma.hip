// Experimental "NT" MFMA GEMM whose global->LDS traffic uses the CDNA4 direct-to-LDS buffer loads
// (buffer_load_dwordx4 ... lds): no registers and no ds_write instructions on the load path, a 3-stage LDS ring,
// XOR-swizzled unpadded [row][k] tiles.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace tfm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace dma {
constexpr int BN = 128, BK = 32, STAGES = 3;
constexpr uint32_t OOB = 0x80000000u;

template <typename T> struct M;
template <> struct M<half_t> {
  static __device__ __forceinline__ f32x16 run(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct M<bf16_t> {
  static __device__ __forceinline__ f32x16 run(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

struct P {
  int M, N, K;
  const uint16_t* A; int lda;
  const uint16_t* B; int ldb;
  uint16_t* C; int ldc;
  const uint16_t* bias; int relu;
  const uint16_t* mask; const uint16_t* residual;
  int tiles_n, tiles_total;
  uint32_t a_bytes, b_bytes;
};

typedef __attribute__((address_space(3))) void* lds_ptr;

template <typename T, int BM>
__global__ __launch_bounds__(256, 2) void gemm_nt_dma_kernel(P p) {
  constexpr int TM = BM / 64;                            // MFMA tiles per wavefront along M
  constexpr int LA = BM / 64;                            // direct-to-LDS loads per wavefront per stage for A (16 rows each)
  __shared__ __attribute__((aligned(1024))) unsigned char As[STAGES][BM * BK * 2];
  __shared__ __attribute__((aligned(1024))) unsigned char Bs[STAGES][BN * BK * 2];
  int tile;
  {
    const int b = blockIdx.x, nb = p.tiles_total, q = nb >> 3, r = nb & 7, x = b & 7;
    tile = x * q + (x < r ? x : r) + (b >> 3);
  }
  const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
  // raw buffer descriptors: base, stride 0, byte extent, format word
  const u32x4 ra = {(uint32_t)(uintptr_t)p.A, (uint32_t)((uintptr_t)p.A >> 32) & 0xffffu, p.a_bytes, 0x00020000u};
  const u32x4 rb = {(uint32_t)(uintptr_t)p.B, (uint32_t)((uintptr_t)p.B >> 32) & 0xffffu, p.b_bytes, 0x00020000u};

  // direct-to-LDS load geometry: wavefront w issues 2 loads per operand per stage, each covering 16 rows x 64 bytes;
  // lane l lands at (row l/4, 16-byte slot l%4) and therefore fetches logical k-vector slot ^ ((row >> 2) & 3)
  // (a wavefront's 16-row groups are LA (A) and 2 (B) consecutive ones; (row >> 2) & 3 == (lane >> 4) for all of them)
  uint32_t offa[LA], offb[2];
  const int kv = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
#pragma unroll
  for (int i = 0; i < LA; ++i) offa[i] = ((uint32_t)(m0 + (wave * LA + i) * 16 + (lane >> 2)) * (uint32_t)p.lda + (uint32_t)kv) * 2u;
#pragma unroll
  for (int i = 0; i < 2; ++i) offb[i] = ((uint32_t)(n0 + (wave * 2 + i) * 16 + (lane >> 2)) * (uint32_t)p.ldb + (uint32_t)kv) * 2u;
  const int nk = (p.K + BK - 1) / BK;
  // LDS addresses as 32-bit offsets (the ring base of each operand; stage and group offsets are added as scalars)
  const uint32_t lds_a = (uint32_t)(uintptr_t)(lds_ptr)(&As[0][0]), lds_b = (uint32_t)(uintptr_t)(lds_ptr)(&Bs[0][0]);
  auto issue = [&](int kt, int stage) {
    const bool ok = kt * BK + kv < p.K;
    // Issued as assembly on purpose: the compiler would otherwise wait for every outstanding direct-to-LDS load
    // before each LDS read, which serialises the ring.  Completion is tracked by hand with s_waitcnt vmcnt.
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      const uint32_t oa = ok ? offa[i] + (uint32_t)kt * (BK * 2) : OOB;
      const uint32_t la = lds_a + stage * (BM * BK * 2) + (wave * LA + i) * 1024;
      asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(__builtin_amdgcn_readfirstlane(la)), "v"(oa), "s"(ra) : "memory");
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t ob = ok ? offb[i] + (uint32_t)kt * (BK * 2) : OOB;
      const uint32_t lb = lds_b + stage * (BN * BK * 2) + (wave * 2 + i) * 1024;
      asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(__builtin_amdgcn_readfirstlane(lb)), "v"(ob), "s"(rb) : "memory");
    }
  };

  f32x16 acc[TM][2];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  issue(0, 0);
  issue(1, 1);
  // fragment read offsets (bytes) within a stage; every fragment row r has (r >> 2) & 3 == (lane >> 2) & 3
  int fra[TM], frb[2];
  const int swz = (lane >> 2) & 3;
#pragma unroll
  for (int i = 0; i < TM; ++i) fra[i] = (wm * (BM / 2) + i * 32 + (lane & 31)) * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i) frb[i] = (wn * 64 + i * 32 + (lane & 31)) * 64;
  constexpr int WAIT = LA + 2;                           // loads per wavefront per K-step
  auto read_frags = [&](int stage, int kk, u32x4 (&fa)[TM], u32x4 (&fb)[2]) {
    const int ko = ((kk * 2 + (lane >> 5)) ^ swz) << 4;
    const unsigned char* as = As[stage];
    const unsigned char* bs = Bs[stage];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const u32x4*>(as + fra[i] + ko);
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i] = *reinterpret_cast<const u32x4*>(bs + frb[i] + ko);
  };
  auto mfmas = [&](const u32x4 (&fa)[TM], const u32x4 (&fb)[2]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = M<T>::run(fb[j], fa[i], acc[i][j]);
  };
  // Software pipeline across the barrier: the fragments of the first half of a K-step are read right after the
  // barrier while the MFMAs of the previous K-step's second half execute; the second half's fragments are read
  // while the first half's MFMAs execute.  LDS latency is therefore always covered by matrix work.
  u32x4 fa0[TM], fb0[2], fa1[TM], fb1[2];
  __builtin_amdgcn_s_waitcnt(0x0F70 | WAIT);             // K-step 0 has landed (K-step 1 may be in flight)
  __syncthreads();
  issue(2, 2);
  read_frags(0, 0, fa0, fb0);
  read_frags(0, 1, fa1, fb1);
  const int nk3 = (nk + STAGES - 1) / STAGES * STAGES;
  for (int base = 0; base < nk3; base += STAGES) {
#pragma unroll
    for (int u = 0; u < STAGES; ++u) {
      const int kt = base + u;
      // (the scheduling fences keep the compiler from sinking the LDS reads back next to the MFMAs that use them)
      mfmas(fa0, fb0);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(0x0F70 | WAIT);         // K-step kt+1 has landed (kt+2 may be in flight)
      __syncthreads();                                   // ... for every wavefront, and stage u is no longer read
      read_frags((u + 1) % STAGES, 0, fa0, fb0);
      issue(kt + 3, u);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(fa1, fb1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags((u + 1) % STAGES, 1, fa1, fb1);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                   // drain the trailing (zero-fill) loads before the block ends

  const T* bias = reinterpret_cast<const T*>(p.bias);
  const T* mask = reinterpret_cast<const T*>(p.mask);
  const T* res = reinterpret_cast<const T*>(p.residual);
  T* C = reinterpret_cast<T*>(p.C);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * (BM / 2) + i * 32 + (lane & 31);
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int n = n0 + wn * 64 + j * 32 + rg * 8 + (lane >> 5) * 4;
        if (n >= p.N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][rg * 4 + e];
        if (bias) {
          float b[4];
          load_f<T, 4>(bias + n, b);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += b[e];
        }
        if (p.relu) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
        }
        const size_t o = (size_t)m * p.ldc + n;
        if (mask) {
          float k[4];
          load_f<T, 4>(mask + o, k);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = k[e] > 0.f ? v[e] : 0.f;
        }
        if (res) {
          float k[4];
          load_f<T, 4>(res + o, k);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += k[e];
        }
        store_f<T, 4>(C + o, v);
      }
    }
  }
}
}  // namespace dma

void launch_gemm_nt_dma(hipStream_t s, const GemmArgs& a) {
  dma::P p;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.A = (const uint16_t*)a.A; p.lda = a.lda; p.B = (const uint16_t*)a.B; p.ldb = a.ldb; p.C = (uint16_t*)a.C; p.ldc = a.ldc;
  p.bias = (const uint16_t*)a.bias; p.relu = a.relu; p.mask = (const uint16_t*)a.mask; p.residual = (const uint16_t*)a.residual;
  static int force = -1;
  if (force < 0) { const char* e = getenv("TFM_GEMM_BM"); force = e ? atoi(e) : 0; }
  int bm = ((long)((a.M + 255) / 256) * ((a.N + 127) / 128) >= 300) ? 256 : 128;
  if (force == 128 || force == 256) bm = force;
  p.tiles_n = (a.N + 127) / 128;
  p.tiles_total = p.tiles_n * ((a.M + bm - 1) / bm);
  p.a_bytes = (uint32_t)(((uint64_t)(a.M - 1) * a.lda + a.K) * 2ull);
  p.b_bytes = (uint32_t)(((uint64_t)(a.N - 1) * a.ldb + a.K) * 2ull);
  dim3 grid(p.tiles_total), block(256);
  if (a.dt == F16) {
    if (bm == 256) hipLaunchKernelGGL((dma::gemm_nt_dma_kernel<half_t, 256>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((dma::gemm_nt_dma_kernel<half_t, 128>), grid, block, 0, s, p);
  } else {
    if (bm == 256) hipLaunchKernelGGL((dma::gemm_nt_dma_kernel<bf16_t, 256>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((dma::gemm_nt_dma_kernel<bf16_t, 128>), grid, block, 0, s, p);
  }
}

}  // namespace tfm
