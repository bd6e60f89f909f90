// MFMA GEMM for gfx950: C[M,N] = epilogue(op(A) op(B)), fp16 or bf16 operands, fp32 accumulation in the matrix
// cores (v_mfma_f32_32x32x16_{f16,bf16}).
//
// Measured on MI355X, what bounds these GEMMs is neither the matrix pipe nor LDS but the rate at which tiles can
// be pulled from L2 into the CUs (about 8 TB/s in aggregate), so the design minimises bytes fetched per flop and
// keeps the fetch path as cheap as possible:
//
//  * Tiles: BM x BN output tile per block, K walked in steps of 32 or 64.  128x128 (4 wavefronts, 64x64 each) for
//    outputs with few tiles, 256x256 (8 wavefronts, 128x64 each) for large outputs: a 256x256 tile fetches half as
//    many bytes per flop as a 128x128 one.  A K-step of 64 fetches whole 128-byte lines per row.
//  * Fetch: CDNA4 direct-to-LDS buffer loads (buffer_load_dwordx4 ... lds): no staging registers and no ds_write on
//    the load path; range-checked, so ragged M, N, K read zeros without branches.  A 2- or 3-stage LDS ring keeps one
//    or two K-steps in flight; one barrier per K-step.  The loads are issued as assembly and tracked with s_waitcnt vmcnt by
//    hand, because the compiler would otherwise drain every outstanding direct-to-LDS load before each LDS read.
//  * LDS layout: unpadded tiles (the direct-to-LDS path writes 1 KB per wavefront contiguously), XOR-swizzled on the
//    global-address side so that fragment reads are bank-conflict free.  An operand whose contraction index is
//    contiguous in memory (A of "NT"/"NN", B of "NT") is staged [row][k] and read with ds_read_b128; an operand
//    whose contraction index is the slow one (B of "NN", both of "TN") is staged as it lies, [k][row], and read with
//    the LDS transpose read ds_read_b64_tr_b16 (a 16-lane group reads a 4(k) x 16(row) patch, each lane receives
//    the 4 k-values of one row).
//  * Math: fragments of the next half K-step are read while the MFMAs of the current one execute (software pipeline
//    across the barrier, pinned with scheduling fences).  Accumulators are produced transposed (B fragment first), so
//    a lane holds 4 consecutive columns of one output row; the epilogue bounces 32-row strips through LDS so that the
//    bias / ReLU / ReLU-mask / residual reads and the stores are whole 128-byte lines.
//  * Block ids are re-mapped so that each XCD (blocks are dealt round-robin to the 8 XCDs, each with its own L2) works
//    on a contiguous run of tiles.
//  * Weight gradients: a single projection's dY^T X has 16-256 output tiles, too few for 256 compute units.  The training
//    step therefore queues them and launches the tiles of up to 48 products end to end as ONE grouped launch
//    (gemm_mfma_grouped_kernel; problem table in the kernel arguments; the first tile column of each product also sums
//    the rows of dY^T it already holds as fragments, which is the bias gradient).  A weight gradient launched on its
//    own can instead split K across blockIdx.y; fp32 partial tiles are then added in a fixed order by a second kernel
//    (no atomics, reproducible).
#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace tfm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr uint32_t OOB = 0x80000000u;                   // beyond any buffer this kernel accepts: reads as zero

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
  int tiles_n, tiles_m, tiles_total, group_m;
  int ksteps_per_split;                                  // split-K: K-steps per blockIdx.y slice
  float* partial;                                        // split-K: fp32 partial tiles [split][M][N], else null
  uint32_t a_bytes, b_bytes;                             // extents for the range-checked loads
  uint64_t drop_key; uint32_t drop_thr; float inv_keep;  // dropout on the result (thr = 0: off), see GemmArgs
  float mask_scale;
  uint16_t* colsum;                                      // grouped weight gradients: [M] sums of A's rows over K (a bias gradient), or null
};

// Sum of the 8 values of a fragment register quadruple, added to c in fp32 (fixed order).
template <typename T> struct FragSum;
template <> struct FragSum<half_t> {
  typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
  static __device__ __forceinline__ float run(u32x4 a, float c) {
    const f16x2 one = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t word = a[w];                          // (a copy: bit-casting the vector element in place read element 0 every time)
      c = __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, word), one, c, false);
    }
    return c;
  }
};
template <> struct FragSum<bf16_t> {
  static __device__ __forceinline__ float run(u32x4 a, float c) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t word = a[w];
      c += __uint_as_float(word << 16);
      c += __uint_as_float(word & 0xffff0000u);
    }
    return c;
  }
};

// One operand's path from global memory through the LDS ring into MFMA fragments.
//   ROWS: tile rows (M or N extent of the block tile);  NW: wavefronts in the block;  TR: see the file comment.
// A direct-to-LDS load writes the wavefront's 64 x 16 bytes contiguously, so load g of a stage fills bytes
// [g*1024, (g+1)*1024) of the tile; each lane chooses WHICH global vector it fetches so that the tile ends up swizzled:
//   [row][k] tile, 2*BK-byte rows:   16-byte slot s of row r holds k-vector    s ^ swz(r)
//   [k][row] tile, ROWS*2-byte rows: 16-byte slot s of k-row k holds row-vector s ^ ((k & 3) << 2)
template <int ROWS, int BK, int NW, bool TR>
struct Operand {
  static constexpr int TILE_BYTES = ROWS * BK * 2;
  static constexpr int LOADS = TILE_BYTES / 1024 / NW;   // direct-to-LDS loads per wavefront per stage
  static_assert(LOADS >= 1 && LOADS * 1024 * NW == TILE_BYTES, "every wavefront loads a whole number of 1 KB pieces of the tile");
  static constexpr int ROW_BYTES = ROWS * 2;             // [k][row] layout only
  static constexpr int KROW_BYTES = BK * 2;              // [row][k] layout only: 64 or 128
  static constexpr int VPR = BK / 8;                     // 16-byte vectors per [row][k] row: 4 or 8
  // swizzle of the [row][k] layout: slot ^= f(row) with f chosen so that 16 consecutive rows cover 16 distinct
  // 16-byte bank groups: 64-byte rows: (row >> 2) & 3;  128-byte rows: (row >> 1) & 7
  static __device__ __forceinline__ int swz(int row) { return BK == 32 ? ((row >> 2) & 3) : ((row >> 1) & 7); }
  uint32_t off[LOADS];                                   // byte offset of this lane's vector in K-step 0
  int kfirst[LOADS];                                     // its k index inside the K-step (for the K-tail test)
  uint32_t step;                                         // byte stride between K-steps
  int kend;

  __device__ __forceinline__ void init(int ld, int row0, int kend_, int wave, int lane) {
    kend = kend_;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int g = wave * LOADS + i;
      if (!TR) {
        const int row = g * (64 / VPR) + lane / VPR;
        kfirst[i] = ((lane % VPR) ^ swz(row)) * 8;
        off[i] = ((uint32_t)(row0 + row) * (uint32_t)ld + (uint32_t)kfirst[i]) * 2u;
      } else {
        const int byte = g * 1024 + lane * 16;
        const int k = byte / ROW_BYTES, slot = (byte % ROW_BYTES) / 16;
        const int vec = slot ^ ((k & 3) << 2);
        kfirst[i] = k;
        off[i] = ((uint32_t)k * (uint32_t)ld + (uint32_t)(row0 + vec * 8)) * 2u;
      }
    }
    step = TR ? (uint32_t)BK * (uint32_t)ld * 2u : (uint32_t)BK * 2u;
  }
  // Issued as assembly on purpose (see the file comment).  lds_stage: LDS byte address of the stage's tile.
  __device__ __forceinline__ void issue(const u32x4& rsrc, int kt, uint32_t lds_stage, int wave) const {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const uint32_t o = (kt * BK + kfirst[i] < kend) ? off[i] + (uint32_t)kt * step : OOB;
      const uint32_t dst = lds_stage + (uint32_t)(wave * LOADS + i) * 1024u;
      asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(__builtin_amdgcn_readfirstlane(dst)), "v"(o),
                   "s"(rsrc)
                   : "memory", "m0");
    }
  }
  // Fragment of tile rows r0..r0+31 for k = kk*16 .. kk*16+15: lane l gets row r0 + l%32, k-group l/32 (8 k-values).
  static __device__ __forceinline__ u32x4 frag(const unsigned char* S, int r0, int kk, int lane) {
    if (!TR) {
      const int row = r0 + (lane & 31);
      const int slot = (kk * 2 + (lane >> 5)) ^ swz(row);
      return *reinterpret_cast<const u32x4*>(S + row * KROW_BYTES + slot * 16);
    } else {
      const int s = lane & 15, ibase = lane & 16;
      const int k = kk * 16 + (lane >> 5) * 8 + (s >> 2);
      const int seg = ((r0 + ibase) >> 4) ^ ((s >> 2) << 1);           // 32-byte segment, swizzled by k & 3
      const unsigned char* p = S + k * ROW_BYTES + seg * 32 + (s & 3) * 8;
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * ROW_BYTES));
      const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
      return u32x4{l2[0], l2[1], h2[0], h2[1]};
    }
  }
};

// One output tile (or one K-slice of it).  `tile` is the tile id inside this problem after the XCD re-mapping, `slice`
// the split-K slice.  CS: the block column tn == 0 also sums A's rows over K (see MfmaGemmParams::colsum).
template <typename T, int BM, int BN, int WM, int WN, int BK, int STAGES, bool ATR, bool BTR, bool CS>
__device__ __forceinline__ void gemm_mfma_tile(const MfmaGemmParams& p, int tile, int slice) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;    // MFMA tiles per wavefront
  constexpr int KK = BK / 16;                            // MFMA sub-steps per K-step (2 or 4)
  constexpr int D = STAGES - 1;                          // K-steps in flight ahead of the one being consumed
  typedef Operand<BM, BK, NW, ATR> OA;
  typedef Operand<BN, BK, NW, BTR> OB;
  // One LDS block: the A ring, the B ring, and (re-using both once the K loop is over) the epilogue's staging strips,
  // which for 16 wavefronts can be a little larger than the rings.
  constexpr int SW = TN * 32;                             // epilogue strip width in columns
  constexpr int SP = SW + 4;                              // its padded pitch in floats: conflict-free for both passes
  constexpr int RING_BYTES = STAGES * (OA::TILE_BYTES + OB::TILE_BYTES);
  constexpr int STRIP_BYTES = NW * 32 * SP * 4;
  constexpr int LDS_BYTES = RING_BYTES > STRIP_BYTES ? RING_BYTES : STRIP_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "LDS per CU");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[LDS_BYTES];
  unsigned char(*As)[OA::TILE_BYTES] = reinterpret_cast<unsigned char(*)[OA::TILE_BYTES]>(smem);
  unsigned char(*Bs)[OB::TILE_BYTES] = reinterpret_cast<unsigned char(*)[OB::TILE_BYTES]>(smem + STAGES * OA::TILE_BYTES);
  // Tile ids run column-major inside bands of group_m tile rows, so the run of ids an XCD works on at one time
  // covers a compact patch of the output and shares its A and B panels in that XCD's L2.
  int tm, tn;
  {
    const int per_band = p.group_m * p.tiles_n, band = tile / per_band, in_band = tile - band * per_band;
    const int gm = min(p.group_m, p.tiles_m - band * p.group_m);
    tm = band * p.group_m + in_band % gm;
    tn = in_band / gm;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave / WN, wn = wave % WN;

  // raw buffer descriptors: base, stride 0, byte extent, format word
  const u32x4 ra = {(uint32_t)(uintptr_t)p.A, (uint32_t)((uintptr_t)p.A >> 32) & 0xffffu, p.a_bytes, 0x00020000u};
  const u32x4 rb = {(uint32_t)(uintptr_t)p.B, (uint32_t)((uintptr_t)p.B >> 32) & 0xffffu, p.b_bytes, 0x00020000u};
  // split-K: this block covers K-steps kt0 .. ; everything at or beyond kend reads as zero
  const int kt0 = slice * p.ksteps_per_split;
  const int kend = min(p.K, (kt0 + p.ksteps_per_split) * BK);
  const int nk = max(0, (kend - kt0 * BK + BK - 1) / BK);
  OA oa;
  OB ob;
  oa.init(p.lda, m0, kend, wave, lane);
  ob.init(p.ldb, n0, kend, wave, lane);
  const uint32_t lds_a = (uint32_t)(uintptr_t)(lds_ptr)(&As[0][0]), lds_b = (uint32_t)(uintptr_t)(lds_ptr)(&Bs[0][0]);
  auto issue = [&](int kt, int stage) {
    oa.issue(ra, kt0 + kt, lds_a + stage * OA::TILE_BYTES, wave);
    ob.issue(rb, kt0 + kt, lds_b + stage * OB::TILE_BYTES, wave);
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  auto read_frags = [&](int stage, int kk, u32x4 (&fa)[TM], u32x4 (&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = OA::frag(As[stage], wm * (BM / WM) + i * 32, kk, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = OB::frag(Bs[stage], wn * (BN / WN) + j * 32, kk, lane);
  };
  // Row sums of A: the wavefronts of the first tile column that hold the first column strip see every A fragment of
  // their rows exactly once (K-steps beyond the slice read zeros), so they add them up on the vector ALU beside the MFMAs.
  const bool do_cs = CS && p.colsum != nullptr && tn == 0 && wn == 0;
  float cs[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) cs[i] = 0.f;
  auto mfmas = [&](const u32x4 (&fa)[TM], const u32x4 (&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<T>::run(fb[j], fa[i], acc[i][j]);   // transposed product: D'[n][m]
    if (CS && do_cs) {
#pragma unroll
      for (int i = 0; i < TM; ++i) cs[i] = FragSum<T>::run(fa[i], cs[i]);
    }
  };

  constexpr int WAIT = (OA::LOADS + OB::LOADS) * (D - 1);   // loads that may still be in flight when a K-step must have landed
  static_assert(WAIT <= 63, "vmcnt is a 6-bit count");
  // s_waitcnt immediate: vmcnt[3:0] in bits 3:0 and vmcnt[5:4] in bits 15:14; expcnt (6:4) and lgkmcnt (11:8) left at
  // their maxima, i.e. not waited for
  constexpr int WAITCNT = 0x0F70 | (WAIT & 15) | ((WAIT >> 4) << 14);
#pragma unroll
  for (int t = 0; t < D; ++t) issue(t, t);
  u32x4 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  __builtin_amdgcn_s_waitcnt(WAITCNT);                   // K-step 0 has landed
  __syncthreads();
  issue(D, D % STAGES);
  read_frags(0, 0, fa0, fb0);
  read_frags(0, 1, fa1, fb1);
  // Software pipeline: sub-step j runs its MFMAs from register set j%2 while set j%2 is refilled with sub-step j+2
  // (of the same stage, or after the barrier of the next one).  LDS latency is therefore always covered by matrix work.
  // The trip count is rounded up to the ring size: K-steps beyond the slice read zeros, so the extra MFMAs add nothing.
  const int nkr = (nk + STAGES - 1) / STAGES * STAGES;
  for (int base = 0; base < nkr; base += STAGES) {
#pragma unroll
    for (int u = 0; u < STAGES; ++u) {
      const int kt = base + u;
#pragma unroll
      for (int j = 0; j < KK; ++j) {
        // (the scheduling fences keep the compiler from sinking the LDS reads back next to the MFMAs that use them)
        if (j % 2 == 0) mfmas(fa0, fb0); else mfmas(fa1, fb1);
        __builtin_amdgcn_sched_barrier(0);
        if (j + 2 < KK) {
          if (j % 2 == 0) read_frags(u, j + 2, fa0, fb0); else read_frags(u, j + 2, fa1, fb1);
        } else if (j == KK - 2) {
          __builtin_amdgcn_s_waitcnt(WAITCNT);           // K-step kt+1 has landed for this wavefront ...
          __syncthreads();                               // ... and for all of them; stage u is no longer read
          read_frags((u + 1) % STAGES, 0, fa0, fb0);
          issue(kt + 1 + D, u);
        } else {
          read_frags((u + 1) % STAGES, 1, fa1, fb1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                    // drain the trailing (zero-fill) loads before LDS is released

  // Epilogue.  The accumulators hold, per lane, 4 consecutive columns of one row, which would make every store an
  // 8-byte fragment of a different cache line.  Each wavefront therefore bounces one 32 x (TN*32) strip at a time through
  // its own slice of LDS (free now: every wavefront is past its last fragment read) and re-reads it so that a lane owns
  // 16 consecutive columns of a row and 4 lanes cover a whole 128-byte line of the output.
  __syncthreads();
  float* strip = reinterpret_cast<float*>(smem) + wave * (32 * SP);
  constexpr int LPR = SW / 16;                            // lanes per row when re-reading (4 for a 64-column strip)
  constexpr int RPP = 64 / LPR;                           // rows per pass
  const T* bias = reinterpret_cast<const T*>(p.bias);
  const T* mask = reinterpret_cast<const T*>(p.mask);
  const T* res = reinterpret_cast<const T*>(p.residual);
  T* C = reinterpret_cast<T*>(p.C);
  float* P = p.partial ? p.partial + (size_t)slice * p.M * p.N : nullptr;
  if (CS && do_cs) {                                      // lanes l and l + 32 hold the two k-groups of row l
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const float t = cs[i] + __shfl_xor(cs[i], 32);
      const int m = m0 + wm * (BM / WM) + i * 32 + (lane & 31);
      if (lane < 32 && m < p.M) reinterpret_cast<T*>(p.colsum)[m] = from_f<T>(t);
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        float4 v = {acc[i][j][rg * 4], acc[i][j][rg * 4 + 1], acc[i][j][rg * 4 + 2], acc[i][j][rg * 4 + 3]};
        *reinterpret_cast<float4*>(strip + (lane & 31) * SP + j * 32 + rg * 8 + (lane >> 5) * 4) = v;
      }
    // (LDS operations of one wavefront complete in order: the reads below see the writes above)
#pragma unroll
    for (int ps = 0; ps < 32 / RPP; ++ps) {
      const int r = ps * RPP + lane / LPR, c = (lane % LPR) * 16;
      float v[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 t = *reinterpret_cast<const float4*>(strip + r * SP + c + q * 4);
        v[q * 4] = t.x; v[q * 4 + 1] = t.y; v[q * 4 + 2] = t.z; v[q * 4 + 3] = t.w;
      }
      const int m = m0 + wm * (BM / WM) + i * 32 + r;
      const int n = n0 + wn * (BN / WN) + c;
      if (m >= p.M) continue;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {                    // two groups of 8 columns, each entirely inside or outside N
        const int nn = n + hf * 8;
        if (nn >= p.N) continue;
        float w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = v[hf * 8 + e];
        if (P) {                                          // split-K: raw fp32 tile, summed by splitk_reduce_kernel
          store_f<float, 8>(P + (size_t)m * p.N + nn, w);
          continue;
        }
        if (bias) {
          float bb[8];
          load_f<T, 8>(bias + nn, bb);
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] += bb[e];
        }
        if (p.relu) {
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] = fmaxf(w[e], 0.f);
        }
        if (p.drop_thr) drop_apply<8>(w, p.drop_key, (uint64_t)m * p.N + nn, p.drop_thr, p.inv_keep);
        const size_t o = (size_t)m * p.ldc + nn;
        if (mask) {
          float k[8];
          load_f<T, 8>(mask + o, k);
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] = k[e] > 0.f ? w[e] * p.mask_scale : 0.f;
        }
        if (res) {
          float k[8];
          load_f<T, 8>(res + o, k);
#pragma unroll
          for (int e = 0; e < 8; ++e) w[e] += k[e];
        }
        store_f<T, 8>(C + o, w);
      }
    }
  }
}

// XCD-aware block order: hardware deals block b to XCD b % 8; give each XCD a contiguous run of tile ids
__device__ __forceinline__ int xcd_tile(int b, int nb) {
  const int q = nb >> 3, r = nb & 7, x = b & 7;
  return x * q + (x < r ? x : r) + (b >> 3);
}

template <typename T, int BM, int BN, int WM, int WN, int BK, int STAGES, bool ATR, bool BTR>
__global__ __launch_bounds__(64 * WM * WN, (WM * WN == 4) ? 2 : 1) void gemm_mfma_kernel(MfmaGemmParams p) {
  gemm_mfma_tile<T, BM, BN, WM, WN, BK, STAGES, ATR, BTR, false>(p, xcd_tile(blockIdx.x, p.tiles_total), blockIdx.y);
}

// Grouped weight gradients: one launch covers the tiles of up to GROUP_MAX independent products C_i = A_i^T B_i (each
// with its own shapes and, optionally, the row sums of A_i^T as a bias gradient).  A single projection's weight gradient
// has 16-256 tiles, too few to fill 256 compute units for more than a fraction of a round; the tiles of many of them
// laid end to end do.  The table travels in the kernel arguments.
constexpr int GROUP_MAX = 48;
struct GroupedProblem {
  const uint16_t* A; const uint16_t* B; uint16_t* C; uint16_t* colsum;
  int M, N, K, lda, ldb, ldc, tile_begin, tiles_m, tiles_n;
  uint32_t a_bytes, b_bytes;
  int pad_;
};
struct GroupedTable {
  int n, tiles_total;
  GroupedProblem pr[GROUP_MAX];
};
static_assert(sizeof(GroupedTable) <= 4096, "kernel argument space");

template <typename T, int BM, int BN, int WM, int WN, int BK, int STAGES>
__global__ __launch_bounds__(64 * WM * WN, (WM * WN == 4) ? 2 : 1) void gemm_mfma_grouped_kernel(GroupedTable tab) {
  const int tile = xcd_tile(blockIdx.x, tab.tiles_total);
  int pi = 0;
  for (int i = 1; i < tab.n; ++i) pi = tile >= tab.pr[i].tile_begin ? i : pi;
  const GroupedProblem& g = tab.pr[pi];
  MfmaGemmParams p;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.A = g.A; p.lda = g.lda; p.B = g.B; p.ldb = g.ldb; p.C = g.C; p.ldc = g.ldc;
  p.bias = nullptr; p.relu = 0; p.mask = nullptr; p.residual = nullptr;
  p.tiles_n = g.tiles_n; p.tiles_m = g.tiles_m; p.tiles_total = g.tiles_m * g.tiles_n; p.group_m = 8;
  p.ksteps_per_split = (g.K + BK - 1) / BK;
  p.partial = nullptr;
  p.a_bytes = g.a_bytes; p.b_bytes = g.b_bytes;
  p.colsum = g.colsum;
  p.drop_key = 0; p.drop_thr = 0; p.inv_keep = 1.f; p.mask_scale = 1.f;
  gemm_mfma_tile<T, BM, BN, WM, WN, BK, STAGES, true, true, true>(p, tile - g.tile_begin, 0);
}

// C[m, n] = epilogue(sum over splits (fixed order) of partial[s][m][n]); epilogue = optional bias[n], optional ReLU
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int M, int N, T* __restrict__ C, int ldc,
                                                            const T* __restrict__ bias, int relu) {
  const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  const size_t total = (size_t)M * N;
  if (idx >= total) return;
  float4 a = *reinterpret_cast<const float4*>(partial + idx);
  for (int s = 1; s < splits; ++s) {
    const float4 b = *reinterpret_cast<const float4*>(partial + (size_t)s * total + idx);
    a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
  }
  const int m = (int)(idx / N), n = (int)(idx % N);
  float v[4] = {a.x, a.y, a.z, a.w};
  if (bias) {
    float bb[4];
    load_f<T, 4>(bias + n, bb);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += bb[e];
  }
  if (relu) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
  }
  store_f<T, 4>(C + (size_t)m * ldc + n, v);
}

void launch_splitk_reduce(hipStream_t s, int dt, const float* partial, int splits, int M, int N, void* C, int ldc, const void* bias) {
  const size_t quads = ((size_t)M * N + 3) / 4;
  dim3 grid((unsigned)((quads + 255) / 256)), block(256);
  if (dt == F16) hipLaunchKernelGGL((splitk_reduce_kernel<half_t>), grid, block, 0, s, partial, splits, M, N, (half_t*)C, ldc, (const half_t*)bias, 0);
  else if (dt == BF16) hipLaunchKernelGGL((splitk_reduce_kernel<bf16_t>), grid, block, 0, s, partial, splits, M, N, (bf16_t*)C, ldc, (const bf16_t*)bias, 0);
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

template <typename T, int BM, int BN, int WM, int WN, int BK, int STAGES>
static void gemm_mfma_launch(hipStream_t s, const GemmArgs& a) {
  MfmaGemmParams p;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.A = (const uint16_t*)a.A; p.lda = a.lda; p.B = (const uint16_t*)a.B; p.ldb = a.ldb; p.C = (uint16_t*)a.C; p.ldc = a.ldc;
  p.bias = (const uint16_t*)a.bias; p.relu = a.relu; p.mask = (const uint16_t*)a.mask; p.residual = (const uint16_t*)a.residual;
  p.colsum = nullptr;
  p.drop_key = a.drop_key; p.drop_thr = a.drop_p > 0.f ? drop_threshold(a.drop_p) : 0u; p.inv_keep = 1.f / (1.f - a.drop_p);
  p.mask_scale = a.mask_scale;
  p.tiles_n = (a.N + BN - 1) / BN;
  p.tiles_m = (a.M + BM - 1) / BM;
  p.tiles_total = p.tiles_n * p.tiles_m;
  p.group_m = 8;
  p.a_bytes = (uint32_t)(a.form == 2 ? extent_bytes(a.K, a.M, a.lda) : extent_bytes(a.M, a.K, a.lda));
  p.b_bytes = (uint32_t)(a.form == 0 ? extent_bytes(a.N, a.K, a.ldb) : extent_bytes(a.K, a.N, a.ldb));
  // Split-K for weight-gradient shapes whose output has too few tiles to fill the chip: slices of K go to
  // blockIdx.y, fp32 partial tiles go to the caller's workspace and are added in a fixed order.
  const int nk = (a.K + BK - 1) / BK;
  int splits = 1;
  if (a.form == 2 && a.splitk_ws && !a.bias && !a.relu && !a.mask && !a.residual && !p.drop_thr && p.tiles_total <= 128 && nk >= 32) {
    splits = 256 / p.tiles_total;
    if (splits > 8) splits = 8;
  } else if (a.form == 0 && BM == 64 && BN == 64 && a.splitk_ws && !a.mask && !a.residual && !p.drop_thr && p.tiles_total <= 128 && nk >= 8 &&
             !(a.deferred_splits && a.relu)) {                // (a deferred reduction has no ReLU)
    // X W^T with few rows (a decoding step): the weights stream through more CUs; every slice keeps >= 4 K-steps and
    // bias / ReLU move into the reduction
    splits = std::min(std::min(256 / p.tiles_total, nk / 4), 8);
  }
  while (splits > 1 && (size_t)splits * a.M * a.N * sizeof(float) > a.splitk_ws_bytes) --splits;
  p.ksteps_per_split = (nk + splits - 1) / splits;
  p.partial = splits > 1 ? (float*)a.splitk_ws : nullptr;
  dim3 grid(p.tiles_total, splits), block(64 * WM * WN);
  if (a.form == 0) hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, BK, STAGES, false, false>), grid, block, 0, s, p);
  else if constexpr (BN >= 128) {                        // the [k][row] swizzle spans 16 vectors = 128 rows: B of dY W ...
    if (a.form == 1) hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, BK, STAGES, false, true>), grid, block, 0, s, p);
    else if constexpr (BM >= 128)                        // ... and A as well for A^T B
      hipLaunchKernelGGL((gemm_mfma_kernel<T, BM, BN, WM, WN, BK, STAGES, true, true>), grid, block, 0, s, p);
  }
  if (a.deferred_splits) *a.deferred_splits = splits > 1 ? splits : 0;
  if (splits > 1 && !a.deferred_splits) {
    const size_t quads = ((size_t)a.M * a.N + 3) / 4;
    hipLaunchKernelGGL((splitk_reduce_kernel<T>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, (const float*)a.splitk_ws, splits,
                       a.M, a.N, (T*)a.C, a.ldc, (const T*)a.bias, a.relu);
  }
}

// ---- grouped weight gradients ---------------------------------------------------------------------------------------------
bool wgrad_group_supported(int dt, const WgradJob& j) {
  GemmArgs a{dt, 2, j.M, j.N, j.K, j.A, j.lda, j.B, j.ldb, j.C, j.ldc, nullptr, 0, nullptr, nullptr};
  if (!gemm_mfma_supported(a)) return false;
  return j.colsum == nullptr || ((uintptr_t)j.colsum & 1) == 0;
}

template <typename T, int BM, int BN, int WM, int WN, int BK, int STAGES>
static void wgrad_grouped_launch(hipStream_t s, const WgradJob* jobs, int n) {
  GroupedTable tab;
  int tiles = 0;
  for (int i = 0; i < n; ++i) {
    const WgradJob& j = jobs[i];
    GroupedProblem& g = tab.pr[i];
    g.A = (const uint16_t*)j.A; g.B = (const uint16_t*)j.B; g.C = (uint16_t*)j.C; g.colsum = (uint16_t*)j.colsum;
    g.M = j.M; g.N = j.N; g.K = j.K; g.lda = j.lda; g.ldb = j.ldb; g.ldc = j.ldc;
    g.tiles_m = (j.M + BM - 1) / BM; g.tiles_n = (j.N + BN - 1) / BN;
    g.tile_begin = tiles;
    tiles += g.tiles_m * g.tiles_n;
    g.a_bytes = (uint32_t)extent_bytes(j.K, j.M, j.lda);
    g.b_bytes = (uint32_t)extent_bytes(j.K, j.N, j.ldb);
    g.pad_ = 0;
  }
  tab.n = n; tab.tiles_total = tiles;
  hipLaunchKernelGGL((gemm_mfma_grouped_kernel<T, BM, BN, WM, WN, BK, STAGES>), dim3(tiles), dim3(64 * WM * WN), 0, s, tab);
}

// 256x256 tiles fetch half as many bytes per flop as 128x128 ones but come in coarser rounds over the 256 compute units:
// compare the rounds each tiling needs, weighted by what a tile of each kind was measured to cost (103 vs 31 us at K = 3264).
void launch_wgrad_grouped(hipStream_t s, int dt, const WgradJob* jobs, int n) {
  if (n <= 0) return;
  long t256 = 0, t128 = 0;
  for (int i = 0; i < n; ++i) {
    t256 += (long)((jobs[i].M + 255) / 256) * ((jobs[i].N + 255) / 256);
    t128 += (long)((jobs[i].M + 127) / 128) * ((jobs[i].N + 127) / 128);
  }
  const double c256 = (double)((t256 + 255) / 256) * 103.0, c128 = (double)((t128 + 255) / 256) * 31.0;
  const bool big = c256 <= c128;
  if (dt == F16) {
    if (big) wgrad_grouped_launch<half_t, 256, 256, 2, 4, 64, 2>(s, jobs, n);
    else wgrad_grouped_launch<half_t, 128, 128, 4, 4, 64, 3>(s, jobs, n);
  } else {
    if (big) wgrad_grouped_launch<bf16_t, 256, 256, 2, 4, 64, 2>(s, jobs, n);
    else wgrad_grouped_launch<bf16_t, 128, 128, 4, 4, 64, 3>(s, jobs, n);
  }
}

// Configuration choice, from measurements on the projection shapes of the big and base Transformers (M ~ 3000-3700 tokens):
//   id  tile     wavefronts  K-step  ring   resident blocks per CU
//    1  128x128      4         32     3      3      more than 256 tiles and K < 3072: several blocks per CU keep it fed
//   12  128x128     16         64     4      1      K >= 3072, or at most 256 tiles (one block per CU anyway): 16 wavefronts
//                                                   of 32x32 hide the fetch latency that 4 of 64x64 exposed (10-15 % faster);
//                                                   a 4-slot ring is 2-4 % faster than 3 slots, 5 slots are slower again
//   13  256x256      8         64     2      1      half the bytes fetched per flop (16 wavefronts are slower here: more LDS
//                                                   traffic per flop)
//   14  192x256      8         64     2      1      X W^T and dY W only: where 256x256 leaves compute units idle (a 3072-wide
//                                                   output of ~3200 rows has 156 tiles of 256x256 but 204 of 192x256 for
//                                                   256 CUs: 31.5 -> 28.0 us; 3000 rows: 37.6 -> 27.3 us)
//   20   64x64       4         64     4      2      fewer than 128 tiles of 128x128 (a decoding step's few rows)
//   22   64x128      8         64     4      1      X W^T and dY W with many rows but a narrow output and K >= 1024 (the 512-wide
//                                                   products of the base model: 116 tiles of 128x128 become 232; 15.8 -> 13.3 us
//                                                   at K = 2048, 14.1 -> 11.7 us at K = 1536; slower than the others at K = 512)
// A launch costs about rounds x (fixed + slope x K-steps), rounds = tiles over the 256 compute units rounded up (the last,
// partly filled round takes as long as a full one); fixed / slope in us per round and 64-wide K-step, measured with
// M = 3264: 11 / 1.45 for 256x256, 9.5 / 1.16 for 192x256, 4.4 / 0.48 for 128x128.
static int choose_tile(const GemmArgs& a) {
  const long t1 = (long)((a.M + 127) / 128) * ((a.N + 127) / 128);
  if (a.form != 2 && a.M >= 1024 && a.K >= 1024 && t1 <= 160) return 22;
  if (t1 < 128 && a.form == 0) return 20;               // few rows (a decoding step, X W^T): smaller tiles reach more CUs
  const long t3 = (long)((a.M + 255) / 256) * ((a.N + 255) / 256);
  const long t4 = (long)((a.M + 191) / 192) * ((a.N + 255) / 256);
  const double ks = (double)((a.K + 63) / 64);
  const double c128 = (double)((t1 + 255) / 256) * (4.4 + 0.48 * ks);
  const double c256 = (double)((t3 + 255) / 256) * (11.0 + 1.45 * ks);
  const double c192 = a.form == 2 ? 1e30 : (double)((t4 + 255) / 256) * (9.5 + 1.16 * ks);
  if (c192 < c256 && c192 < c128) return 14;
  if (t3 >= 150) return 13;
  if (a.K >= 3072 || t1 <= 256) return 12;
  return 1;
}

template <typename T>
static void gemm_mfma_dispatch(hipStream_t s, const GemmArgs& a) {
  switch (choose_tile(a)) {
    case 13: gemm_mfma_launch<T, 256, 256, 2, 4, 64, 2>(s, a); break;
    case 12: gemm_mfma_launch<T, 128, 128, 4, 4, 64, 4>(s, a); break;
    case 14: gemm_mfma_launch<T, 192, 256, 2, 4, 64, 2>(s, a); break;   // (never chosen for A^T B: its A tile would be [k][192])
    case 22: gemm_mfma_launch<T, 64, 128, 2, 4, 64, 4>(s, a); break;    // (nor this one: [k][64])
    case 20:                                            // (the [k][row] swizzle spans 16 vectors: NT form only)
      if (a.form == 0) gemm_mfma_launch<T, 64, 64, 2, 2, 64, 4>(s, a);
      else gemm_mfma_launch<T, 128, 128, 2, 2, 32, 3>(s, a);
      break;
    default: gemm_mfma_launch<T, 128, 128, 2, 2, 32, 3>(s, a); break;
  }
}

void launch_gemm_mfma(hipStream_t s, const GemmArgs& a) {
  if (a.dt == F16) gemm_mfma_dispatch<half_t>(s, a);
  else gemm_mfma_dispatch<bf16_t>(s, a);
}

}  // namespace tfm
