// MFMA GEMM for gfx950: C[M,N] = epilogue(op(A) op(B)), fp16 or bf16 operands, fp32 accumulation in the matrix
// cores (v_mfma_f32_32x32x16_{f16,bf16}).
//
// Tiling: one 256-thread block (4 wavefronts of 64 lanes, 2x2) owns a 128x128 output tile and walks K in steps of
// 64; each wavefront owns 64x64 = 2x2 MFMA tiles (64 fp32 accumulators per lane).  Global memory is read with
// 16-byte loads into registers one K-step ahead of the math and staged through LDS.
//
// Operand layouts.  The MFMA wants, per lane, 8 consecutive k of one row.  An operand whose contraction index is
// contiguous in memory (A of "NT"/"NN", B of "NT") is staged as [row][k] with a padded pitch and read back with
// one ds_read_b128 per fragment.  An operand whose contraction index is the slow one (B of "NN", both of "TN")
// is staged as it lies in memory, [k][row], and read back with the CDNA4 LDS transpose read ds_read_b64_tr_b16:
// a 16-lane group reads a 4(k) x 16(row) patch and each lane receives the 4 k-values of one row.
//
// The accumulators are produced transposed (the B fragment is fed as the MFMA's first operand), so that a lane
// holds 4 consecutive columns of one output row and the epilogue (bias, ReLU, ReLU-mask, residual) moves 8 bytes
// per access.
//
// Block ids are re-mapped so that each XCD (blocks are dealt round-robin to the 8 XCDs, each with its own L2)
// works on a contiguous run of tiles and re-uses the A/B panels it has pulled into its L2.
#include "common.h"
#include "kernels.h"

namespace tfm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int PITCH_D = BK + 8;        // [row][k] staging: 144-byte rows, conflict-free 16-byte reads
constexpr int PITCH_T = 128 + 16;      // [k][row] staging: 288-byte rows, 4 consecutive k-rows hit distinct banks
constexpr int TILE_HALFS = 128 * PITCH_D;   // == 64 * PITCH_T == 9216
static_assert(128 * PITCH_D == 64 * PITCH_T, "both stagings use the same LDS footprint");

template <typename T> struct Mfma;
template <> struct Mfma<half_t> {
  static __device__ __forceinline__ f32x16 run(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mfma<bf16_t> {
  static __device__ __forceinline__ f32x16 run(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

struct MfmaGemmParams {
  int M, N, K;
  const uint16_t* A; int lda;
  const uint16_t* B; int ldb;
  uint16_t* C; int ldc;
  const uint16_t* bias;
  int relu;
  const uint16_t* mask;
  const uint16_t* residual;
  int tiles_n, tiles_total;
};

// Loads the 4 16-byte vectors a thread contributes to one operand tile (zero outside the matrix).
// TR == false: memory is [rows, K] (k contiguous);  TR == true: memory is [K, rows] (row index contiguous).
template <bool TR>
__device__ __forceinline__ void load_tile(const uint16_t* __restrict__ P, int ld, int row0, int nrows, int k0, int K, u32x4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + 256 * i;
    int row, k;
    if (!TR) { row = row0 + (v >> 3); k = k0 + (v & 7) * 8; } else { k = k0 + (v >> 4); row = row0 + (v & 15) * 8; }
    const bool ok = row < nrows && k < K;
    const size_t off = TR ? (size_t)k * ld + row : (size_t)row * ld + k;
    r[i] = ok ? *reinterpret_cast<const u32x4*>(P + off) : u32x4{0u, 0u, 0u, 0u};
  }
}
template <bool TR>
__device__ __forceinline__ void store_tile(uint16_t* __restrict__ S, const u32x4 (&r)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + 256 * i;
    const int off = TR ? (v >> 4) * PITCH_T + (v & 15) * 8 : (v >> 3) * PITCH_D + (v & 7) * 8;
    *reinterpret_cast<u32x4*>(S + off) = r[i];
  }
}
// Fragment of rows r0..r0+31, k = kk*16 .. kk*16+15 of the staged tile: lane l gets row r0 + l%32, k-group l/32.
template <bool TR>
__device__ __forceinline__ u32x4 read_frag(const uint16_t* S, int r0, int kk, int lane) {
  if (!TR) {
    return *reinterpret_cast<const u32x4*>(S + (r0 + (lane & 31)) * PITCH_D + kk * 16 + (lane >> 5) * 8);
  } else {
    const int s = lane & 15, ibase = lane & 16, kb = kk * 16 + (lane >> 5) * 8;
    const uint16_t* p = S + (kb + (s >> 2)) * PITCH_T + r0 + ibase + 4 * (s & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * PITCH_T));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    return u32x4{l2[0], l2[1], h2[0], h2[1]};
  }
}

template <typename T, bool ATR, bool BTR>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(MfmaGemmParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t As[TILE_HALFS];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[TILE_HALFS];
  // XCD-aware tile order: hardware deals block b to XCD b % 8; give each XCD a contiguous run of tile ids
  int tile;
  {
    const int b = blockIdx.x, nb = p.tiles_total, q = nb >> 3, r = nb & 7, x = b & 7;
    tile = x * q + (x < r ? x : r) + (b >> 3);
  }
  const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 ra[4], rb[4];
  load_tile<ATR>(p.A, p.lda, m0, p.M, 0, p.K, ra);
  load_tile<BTR>(p.B, p.ldb, n0, p.N, 0, p.K, rb);
  const int nk = (p.K + BK - 1) / BK;
  for (int kt = 0; kt < nk; ++kt) {
    store_tile<ATR>(As, ra);
    store_tile<BTR>(Bs, rb);
    __syncthreads();
    if (kt + 1 < nk) {
      load_tile<ATR>(p.A, p.lda, m0, p.M, (kt + 1) * BK, p.K, ra);
      load_tile<BTR>(p.B, p.ldb, n0, p.N, (kt + 1) * BK, p.K, rb);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      u32x4 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = read_frag<ATR>(As, wm * 64 + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = read_frag<BTR>(Bs, wn * 64 + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = Mfma<T>::run(fb[j], fa[i], acc[i][j]);   // transposed product: D'[n][m]
    }
    __syncthreads();
  }

  // epilogue: lane owns row m, and for each (j, rg) 4 consecutive columns
  const T* bias = reinterpret_cast<const T*>(p.bias);
  const T* mask = reinterpret_cast<const T*>(p.mask);
  const T* res = reinterpret_cast<const T*>(p.residual);
  T* C = reinterpret_cast<T*>(p.C);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = m0 + wm * 64 + i * 32 + (lane & 31);
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

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

bool gemm_mfma_supported(const GemmArgs& a) {
  if (a.dt != F16 && a.dt != BF16) return false;
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
  // every 16-byte vector must lie entirely inside or outside the matrix and be aligned
  const bool a_tr = a.form == 2, b_tr = a.form != 0;
  if ((a_tr ? a.M : a.K) % 8 || (b_tr ? a.N : a.K) % 8 || a.N % 8) return false;
  if (a.lda % 8 || a.ldb % 8 || a.ldc % 8) return false;
  if (!aligned16(a.A) || !aligned16(a.B) || !aligned16(a.C)) return false;
  if (a.bias && !aligned16(a.bias)) return false;
  if (a.mask && !aligned16(a.mask)) return false;
  if (a.residual && !aligned16(a.residual)) return false;
  return true;
}

template <typename T>
static void gemm_mfma_dispatch(hipStream_t s, const GemmArgs& a) {
  MfmaGemmParams p;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.A = (const uint16_t*)a.A; p.lda = a.lda; p.B = (const uint16_t*)a.B; p.ldb = a.ldb; p.C = (uint16_t*)a.C; p.ldc = a.ldc;
  p.bias = (const uint16_t*)a.bias; p.relu = a.relu; p.mask = (const uint16_t*)a.mask; p.residual = (const uint16_t*)a.residual;
  p.tiles_n = (a.N + BN - 1) / BN;
  p.tiles_total = p.tiles_n * ((a.M + BM - 1) / BM);
  dim3 grid(p.tiles_total), block(256);
  if (a.form == 0) hipLaunchKernelGGL((gemm_mfma_kernel<T, false, false>), grid, block, 0, s, p);
  else if (a.form == 1) hipLaunchKernelGGL((gemm_mfma_kernel<T, false, true>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((gemm_mfma_kernel<T, true, true>), grid, block, 0, s, p);
}

void launch_gemm_mfma(hipStream_t s, const GemmArgs& a) {
  if (a.dt == F16) gemm_mfma_dispatch<half_t>(s, a);
  else gemm_mfma_dispatch<bf16_t>(s, a);
}

}  // namespace tfm
