// MFMA GEMM for gfx950: C[M,N] = epilogue(op(A) op(B)), fp16 or bf16 operands, fp32 accumulation in the matrix
// cores (v_mfma_f32_32x32x16_{f16,bf16}).
//
// Tiling: one 256-thread block (4 wavefronts of 64 lanes, 2x2) owns a BM x 128 output tile (BM = 128 or 256) and
// walks K in steps of 32; each wavefront owns (BM/2) x 64 = (BM/64) x 2 MFMA tiles.
//
// Pipeline: global memory is read with 16-byte range-checked buffer loads (out-of-range rows read as zero, so
// ragged M, N and K need no branches) into registers three K-steps ahead of the math; LDS is double buffered, so
// one barrier per K-step separates the write of step k+1 from the MFMAs of step k.
//
// Operand layouts.  The MFMA wants, per lane, 8 consecutive k of one row.  An operand whose contraction index is
// contiguous in memory (A of "NT"/"NN", B of "NT") is staged as [row][k] with a padded pitch and read back with
// one ds_read_b128 per fragment.  An operand whose contraction index is the slow one (B of "NN", both of "TN")
// is staged as it lies in memory, [k][row], and read back with the CDNA4 LDS transpose read ds_read_b64_tr_b16:
// a 16-lane group reads a 4(k) x 16(row) patch and each lane receives the 4 k-values of one row.  Both pitches
// are chosen so that the 16 lanes served together hit 16 distinct 16-byte bank groups.
//
// The accumulators are produced transposed (the B fragment is fed as the MFMA's first operand), so that a lane
// holds 4 consecutive columns of one output row and the epilogue (bias, ReLU, ReLU-mask, residual) moves 8 bytes
// per access.
//
// Block ids are re-mapped so that each XCD (blocks are dealt round-robin to the 8 XCDs, each with its own L2)
// works on a contiguous run of tiles and re-uses the A/B panels it has pulled into its L2.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace tfm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int BN = 128;
constexpr uint32_t OOB = 0x80000000u;                   // beyond any buffer this kernel accepts: reads as zero

template <int ROWS, int BK> struct Geom {
  static constexpr int NV = ROWS * BK / 8 / 256;        // 16-byte vectors per thread per K-step
  static constexpr int PITCH_D = BK + 8;                // [row][k] staging: 80- or 144-byte rows
  static constexpr int PITCH_T = ROWS + 32;             // [k][row] staging: row bytes = 64 (mod 256)
  static constexpr int HALFS = (ROWS * PITCH_D > BK * PITCH_T) ? ROWS * PITCH_D : BK * PITCH_T;
};

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
  int ksteps_per_split;                                  // split-K: K-steps per blockIdx.y slice
  float* partial;                                        // split-K: fp32 partial tiles [split][M][N], else null
  uint32_t a_bytes, b_bytes;                             // extents for the range-checked loads
};

// Per-thread byte offsets of its vectors in K-step 0, and the K-step stride.
// TR == false: memory [rows, K] (k contiguous);  TR == true: memory [K, rows] (row index contiguous).
template <int ROWS, int BK, bool TR>
struct Loader {
  typedef Geom<ROWS, BK> G;
  static constexpr int VPR = BK / 8;                     // vectors per row in the [row][k] layout
  uint32_t off[G::NV];
  int kvec[G::NV];        // direct layout: first k of the vector (for the K-tail test)
  uint32_t step;
  int K;
  __device__ __forceinline__ void init(int ld, int row0, int K_) {
    K = K_;
#pragma unroll
    for (int i = 0; i < G::NV; ++i) {
      const int v = threadIdx.x + 256 * i;
      if (!TR) {
        const int row = row0 + v / VPR;
        kvec[i] = (v % VPR) * 8;
        off[i] = ((uint32_t)row * (uint32_t)ld + (uint32_t)kvec[i]) * 2u;
      } else {
        const int k = v / (ROWS / 8), row = row0 + (v % (ROWS / 8)) * 8;
        kvec[i] = 0;
        off[i] = ((uint32_t)k * (uint32_t)ld + (uint32_t)row) * 2u;
      }
    }
    step = TR ? (uint32_t)BK * (uint32_t)ld * 2u : (uint32_t)BK * 2u;
  }
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, int kt, u32x4 (&r)[G::NV]) const {
#pragma unroll
    for (int i = 0; i < G::NV; ++i) {
      uint32_t o = off[i] + (uint32_t)kt * step;
      if (!TR) { if (kt * BK + kvec[i] >= K) o = OOB; }                // k-tail inside a row is not caught by the range check
      else { if (kt * BK + (int)((threadIdx.x + 256 * i) / (ROWS / 8)) >= K) o = OOB; }
      r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)o, 0, 0);
    }
  }
  static __device__ __forceinline__ void store(uint16_t* S, const u32x4 (&r)[G::NV]) {
#pragma unroll
    for (int i = 0; i < G::NV; ++i) {
      const int v = threadIdx.x + 256 * i;
      const int o = TR ? (v / (ROWS / 8)) * G::PITCH_T + (v % (ROWS / 8)) * 8 : (v / VPR) * G::PITCH_D + (v % VPR) * 8;
      *reinterpret_cast<u32x4*>(S + o) = r[i];
    }
  }
  // Fragment of rows r0..r0+31, k = kk*16 .. kk*16+15 of the staged tile: lane l gets row r0 + l%32, k-group l/32.
  static __device__ __forceinline__ u32x4 frag(const uint16_t* S, int r0, int kk, int lane) {
    if (!TR) {
      return *reinterpret_cast<const u32x4*>(S + (r0 + (lane & 31)) * G::PITCH_D + kk * 16 + (lane >> 5) * 8);
    } else {
      const int s = lane & 15, ibase = lane & 16, kb = kk * 16 + (lane >> 5) * 8;
      const uint16_t* p = S + (kb + (s >> 2)) * G::PITCH_T + r0 + ibase + 4 * (s & 3);
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * G::PITCH_T));
      const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
      return u32x4{l2[0], l2[1], h2[0], h2[1]};
    }
  }
};

template <typename T, int BM, int BK, int PF, bool ATR, bool BTR>
__global__ __launch_bounds__(256, 2) void gemm_mfma_kernel(MfmaGemmParams p) {
  // BK: K-step; PF: K-steps held in registers ahead of the math
  constexpr int TM = BM / 64;                            // MFMA tiles per wavefront along M
  typedef Loader<BM, BK, ATR> LA;
  typedef Loader<BN, BK, BTR> LB;
  __shared__ __attribute__((aligned(16))) uint16_t As[2][Geom<BM, BK>::HALFS];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][Geom<BN, BK>::HALFS];
  // XCD-aware tile order: hardware deals block b to XCD b % 8; give each XCD a contiguous run of tile ids
  int tile;
  {
    const int b = blockIdx.x, nb = p.tiles_total, q = nb >> 3, r = nb & 7, x = b & 7;
    tile = x * q + (x < r ? x : r) + (b >> 3);
  }
  const int m0 = (tile / p.tiles_n) * BM, n0 = (tile % p.tiles_n) * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;

  f32x16 acc[TM][2];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const __amdgpu_buffer_rsrc_t ra_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)p.A, 0, p.a_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rb_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)p.B, 0, p.b_bytes, 0x00020000);
  LA la;
  LB lb;
  // split-K: this block covers K-steps [kt0, kt0 + nk); everything beyond its slice reads as zero
  const int kt0 = blockIdx.y * p.ksteps_per_split;
  const int kend = min(p.K, (kt0 + p.ksteps_per_split) * BK);
  la.init(p.lda, m0, kend);
  lb.init(p.ldb, n0, kend);
  const int nk = max(0, (kend - kt0 * BK + BK - 1) / BK);

  u32x4 ra[PF][Geom<BM, BK>::NV], rb[PF][Geom<BN, BK>::NV];
#pragma unroll
  for (int u = 0; u < PF; ++u) { la.load(ra_rsrc, kt0 + u, ra[u]); lb.load(rb_rsrc, kt0 + u, rb[u]); }
  LA::store(As[0], ra[0]);
  LB::store(Bs[0], rb[0]);
  la.load(ra_rsrc, kt0 + PF, ra[0]);
  lb.load(rb_rsrc, kt0 + PF, rb[0]);
  __syncthreads();

  // The trip count is rounded up to a multiple of the prefetch depth: K-steps beyond K read zeros (range check), so
  // the extra MFMAs add nothing and the loop body stays branch-free.
  const int nk_pad = (nk + PF - 1) / PF * PF;
  for (int base = 0; base < nk_pad; base += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int kt = base + u;
      const int slot = (u + 1) % PF;                     // registers holding K-step kt+1
      const int cur = kt & 1;
      LA::store(As[cur ^ 1], ra[slot]);
      LB::store(Bs[cur ^ 1], rb[slot]);
      la.load(ra_rsrc, kt0 + kt + 1 + PF, ra[slot]);
      lb.load(rb_rsrc, kt0 + kt + 1 + PF, rb[slot]);
      const uint16_t* as = As[cur];
      const uint16_t* bs = Bs[cur];
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        u32x4 fa[TM], fb[2];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = LA::frag(as, wm * (BM / 2) + i * 32, kk, lane);
#pragma unroll
        for (int j = 0; j < 2; ++j) fb[j] = LB::frag(bs, wn * 64 + j * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = Mfma<T>::run(fb[j], fa[i], acc[i][j]);   // transposed product: D'[n][m]
      }
      __syncthreads();
    }
  }

  if (p.partial) {                                        // split-K: raw fp32 tile, summed by splitk_reduce_kernel
    float* P = p.partial + (size_t)blockIdx.y * p.M * p.N;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * (BM / 2) + i * 32 + (lane & 31);
      if (m >= p.M) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int n = n0 + wn * 64 + j * 32 + rg * 8 + (lane >> 5) * 4;
          if (n >= p.N) continue;
          float4 v = {acc[i][j][rg * 4], acc[i][j][rg * 4 + 1], acc[i][j][rg * 4 + 2], acc[i][j][rg * 4 + 3]};
          *reinterpret_cast<float4*>(P + (size_t)m * p.N + n) = v;
        }
    }
    return;
  }
  // epilogue: lane owns row m, and for each (j, rg) 4 consecutive columns
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

// C[m, n] = sum over splits (fixed order) of partial[s][m][n]
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int M, int N, T* __restrict__ C, int ldc) {
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const size_t total = (size_t)M * N;
  if (idx >= total) return;
  float4 a = *reinterpret_cast<const float4*>(partial + idx);
  for (int s = 1; s < splits; ++s) {
    const float4 b = *reinterpret_cast<const float4*>(partial + (size_t)s * total + idx);
    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
  }
  const int m = (int)(idx / N), n = (int)(idx % N);
  const float v[4] = {a.x, a.y, a.z, a.w};
  store_f<T, 4>(C + (size_t)m * ldc + n, v);
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// bytes spanned by a [rows, width] view with row stride ld (elements of 2 bytes)
static uint64_t extent_bytes(int rows, int width, int ld) { return ((uint64_t)(rows - 1) * ld + width) * 2ull; }

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
  // 32-bit byte offsets in the range-checked loads, including the rows of a ragged last tile
  const uint64_t lim = 0x7f000000ull;
  const uint64_t ea = a_tr ? extent_bytes(a.K + 256, a.M + 256, a.lda) : extent_bytes(a.M + 256, a.K + 256, a.lda);
  const uint64_t eb = b_tr ? extent_bytes(a.K + 256, a.N + 256, a.ldb) : extent_bytes(a.N + 256, a.K + 256, a.ldb);
  if (ea >= lim || eb >= lim) return false;
  return true;
}

template <typename T, int BM, int BK, int PF>
static void gemm_mfma_launch(hipStream_t s, const GemmArgs& a) {
  MfmaGemmParams p;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.A = (const uint16_t*)a.A; p.lda = a.lda; p.B = (const uint16_t*)a.B; p.ldb = a.ldb; p.C = (uint16_t*)a.C; p.ldc = a.ldc;
  p.bias = (const uint16_t*)a.bias; p.relu = a.relu; p.mask = (const uint16_t*)a.mask; p.residual = (const uint16_t*)a.residual;
  p.tiles_n = (a.N + BN - 1) / BN;
  p.tiles_total = p.tiles_n * ((a.M + BM - 1) / BM);
  p.a_bytes = (uint32_t)(a.form == 2 ? extent_bytes(a.K, a.M, a.lda) : extent_bytes(a.M, a.K, a.lda));
  p.b_bytes = (uint32_t)(a.form == 0 ? extent_bytes(a.N, a.K, a.ldb) : extent_bytes(a.K, a.N, a.ldb));
  // Split-K for weight-gradient shapes whose output has too few tiles to fill the chip: slices of K go to
  // blockIdx.y, fp32 partial tiles go to the caller's workspace and are added in a fixed order.
  const int nk = (a.K + BK - 1) / BK;
  int splits = 1;
  if (a.form == 2 && a.splitk_ws && !a.bias && !a.relu && !a.mask && !a.residual && p.tiles_total <= 128 && nk >= 32) {
    splits = 256 / p.tiles_total;
    if (splits > 8) splits = 8;
    while (splits > 1 && (size_t)splits * a.M * a.N * sizeof(float) > a.splitk_ws_bytes) --splits;
  }
  p.ksteps_per_split = (nk + splits - 1) / splits;
  p.partial = splits > 1 ? (float*)a.splitk_ws : nullptr;
  dim3 grid(p.tiles_total, splits), block(256);
  if (a.form == 0) hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BK, PF, false, false>), grid, block, 0, s, p);
  else if (a.form == 1) hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BK, PF, false, true>), grid, block, 0, s, p);
  else hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BK, PF, true, true>), grid, block, 0, s, p);
  if (splits > 1) {
    const size_t quads = ((size_t)a.M * a.N + 3) / 4;
    hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, (const float*)a.splitk_ws, splits,
                       a.M, a.N, (T*)a.C, a.ldc);
  }
}

// 256-row tiles halve the B-panel traffic per flop; they pay off once there are enough of them to fill the chip.
static int forced_bm() {                                 // tuning aid: TFM_GEMM_BM=128|256 overrides the choice
  static int v = -1;
  if (v < 0) { const char* e = getenv("TFM_GEMM_BM"); v = e ? atoi(e) : 0; }
  return v;
}

void launch_gemm_mfma(hipStream_t s, const GemmArgs& a) {
  int bm = 128;
  const long tiles256 = (long)((a.M + 255) / 256) * ((a.N + BN - 1) / BN);
  if (tiles256 >= 400) bm = 256;
  if (forced_bm() == 128 || forced_bm() == 256) bm = forced_bm();
  static int bk64 = -1;
  if (bk64 < 0) { const char* e = getenv("TFM_GEMM_BK"); bk64 = (e && atoi(e) == 64) ? 1 : 0; }
  if (a.dt == F16) {
    if (bm == 256) gemm_mfma_launch<half_t, 256, 32, 2>(s, a);
    else if (bk64) gemm_mfma_launch<half_t, 128, 64, 2>(s, a);
    else gemm_mfma_launch<half_t, 128, 32, 3>(s, a);
  } else {
    if (bm == 256) gemm_mfma_launch<bf16_t, 256, 32, 2>(s, a);
    else if (bk64) gemm_mfma_launch<bf16_t, 128, 64, 2>(s, a);
    else gemm_mfma_launch<bf16_t, 128, 32, 3>(s, a);
  }
}

}  // namespace tfm
