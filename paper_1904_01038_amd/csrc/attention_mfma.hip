// Fused multi-head attention on the matrix cores for head width 64, fp16/bf16 operands, fp32 softmax.
//
// Every product is formed transposed so that one lane owns one softmax row: for scores S^T[key][query] the MFMA
// accumulator layout puts a query in lane%32 and 16 keys in the lane's registers, so row max / row sum are
// in-register reductions plus one exchange between lane halves, and the exponentiated tile is already in the
// operand layout of the second product (O^T = V^T P^T) - no LDS round trip for P.
//
// K and V tiles are staged in LDS once per 64-key chunk and shared by the block's wavefronts.  Operands whose
// contraction index is the slow one in memory (V for O^T = V^T P^T, K for dQ^T = K^T dS^T, Q and dO for
// dK^T/dV^T) are staged as they lie and fetched with the CDNA4 LDS transpose read (ds_read_b64_tr_b16).
//
// Forward: grid (query chunks of 64, heads, sentences), 2 wavefronts x 32 queries, online softmax over key chunks,
//          stores the row log-sum-exp.
// Backward (one launch): blocks [0, nq) along x compute dQ with the forward's decomposition, recomputing P from the
//           saved log-sum-exp; blocks [nq, nq+nk) own 64-key chunks and loop over query chunks for dK/dV.  No atomics.
//           Launches whose sentences all fit one chunk use a kernel that forms all three gradients in one block.
#include "common.h"
#include "kernels.h"

// Minimum wavefronts per SIMD the register allocation must leave room for.  Left to itself the compiler gives the
// backward kernel more than 256 registers (one wavefront per SIMD, two blocks per CU), and the kernel is bound by the
// latency of its dependent load -> product -> softmax chains, which only more resident wavefronts hide.
#ifndef ATT_FWD_MIN_WAVES
#define ATT_FWD_MIN_WAVES 3
#endif
#ifndef ATT_BWD_MIN_WAVES
#define ATT_BWD_MIN_WAVES 2
#endif
namespace tfm {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int DH = 64;
constexpr int PT = 80;                 // LDS pitch (halfs) of a [rows][64] tile: 160-byte rows
constexpr int CH = 64;                 // rows per staged chunk
constexpr int ATT_THREADS = 128;

template <typename T> struct AMfma;
template <> struct AMfma<half_t> {
  static __device__ __forceinline__ f32x16 run(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, v);
  }
};
template <> struct AMfma<bf16_t> {
  static __device__ __forceinline__ f32x16 run(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    return (uint32_t)f_to_bf16_bits(a) | ((uint32_t)f_to_bf16_bits(b) << 16);
  }
};

struct AttnP {
  const uint16_t *q, *k, *v, *o, *d_o;
  uint16_t *out, *dq, *dk, *dv;
  int ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv;
  float* lse;
  const int *q_off, *k_off;
  int total_q, causal;
  float scale;
  // dropout on the attention weights (drop_thr = 0: off): weight (packed query row i, head h, key j) uses element
  // ((i * H + h) << 16) + j of the counter-based generator; one 64-bit word serves four consecutive keys
  uint64_t drop_key;
  uint32_t drop_thr;
  float inv_keep;
  int H;
  // Launches whose sentences all fit one 64-row chunk: consecutive sentences packed into one block.  Entry g of the
  // table is {first sentence, first query row, first key row, 0}; block g serves the sentences from its entry up to the
  // next entry's (at most 16 of them, at most 64 query rows and 64 key rows in total); null: one sentence per block
  const int4* groups;
};
__device__ __forceinline__ uint64_t attn_drop_word(const AttnP& p, int qrow, int h, int j) {
  return drop_word(p.drop_key, ((((uint64_t)qrow * (uint64_t)p.H + (uint64_t)h) << 16) + (uint64_t)j) >> 2);
}

// rows r0..r0+31 of a staged tile as an MFMA operand: lane -> row r0 + lane%32, columns kk*16 + (lane/32)*8 .. +8
template <int P = PT>
__device__ __forceinline__ u32x4 frag_direct(const uint16_t* S, int r0, int kk, int lane) {
  return *reinterpret_cast<const u32x4*>(S + (r0 + (lane & 31)) * P + kk * 16 + (lane >> 5) * 8);
}
// columns c0..c0+31 of a staged tile as an MFMA operand whose contraction runs over 16 tile rows from kbase:
// lane -> column c0 + lane%32; k-slot (half = lane/32, e) -> tile row kbase + 4*half + e (e < 4), kbase + 8 + 4*half + e-4.
// This is the row order in which a 32x32 accumulator holds its rows, so an accumulator converts in place into the
// other operand of the same product.
template <int P = PT>
__device__ __forceinline__ u32x4 frag_tr(const uint16_t* S, int c0, int kbase, int lane) {
  const int s = lane & 15, ibase = lane & 16, half = lane >> 5;
  const uint16_t* p = S + (kbase + 4 * half + (s >> 2)) * P + c0 + ibase + 4 * (s & 3);
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 8 * P));
  const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
  return u32x4{l2[0], l2[1], h2[0], h2[1]};
}
// 64 rows x 64 columns from global (row stride ld) into LDS, zero beyond nvalid rows.  128 threads, 4 vectors each.
template <int P = PT>
__device__ __forceinline__ void stage_tile(uint16_t* S, const uint16_t* __restrict__ G, int ld, int row0, int nvalid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + ATT_THREADS * i;
    const int r = v >> 3, c = (v & 7) * 8;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (row0 + r < nvalid) x = *reinterpret_cast<const u32x4*>(G + (size_t)(row0 + r) * ld + c);
    *reinterpret_cast<u32x4*>(S + r * P + c) = x;
  }
}
// The same in two halves, so that the next chunk's rows travel from memory while the current chunk is being used.
__device__ __forceinline__ void fetch_tile(u32x4 (&x)[4], const uint16_t* __restrict__ G, int ld, int row0, int nvalid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + ATT_THREADS * i;
    const int r = v >> 3, c = (v & 7) * 8;
    x[i] = u32x4{0u, 0u, 0u, 0u};
    if (row0 + r < nvalid) x[i] = *reinterpret_cast<const u32x4*>(G + (size_t)(row0 + r) * ld + c);
  }
}
__device__ __forceinline__ void put_tile(uint16_t* S, const u32x4 (&x)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + ATT_THREADS * i;
    *reinterpret_cast<u32x4*>(S + (v >> 3) * PT + (v & 7) * 8) = x[i];
  }
}
// operand fragments of 32 rows straight from global memory (rows beyond nvalid are zero)
__device__ __forceinline__ void load_frags(u32x4 (&f)[4], const uint16_t* __restrict__ G, int ld, int row, int nvalid, int lane) {
  const int r = row + (lane & 31);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    f[kk] = u32x4{0u, 0u, 0u, 0u};
    if (r < nvalid) f[kk] = *reinterpret_cast<const u32x4*>(G + (size_t)r * ld + kk * 16 + (lane >> 5) * 8);
  }
}
template <typename T>
__device__ __forceinline__ float dot8(u32x4 a, u32x4 b) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t x = a[i], y = b[i];
    float x0, x1, y0, y1;
    if (sizeof(T) == 2 && __is_same(T, half_t)) {
      typedef _Float16 h2 __attribute__((ext_vector_type(2)));
      const h2 xv = __builtin_bit_cast(h2, x), yv = __builtin_bit_cast(h2, y);
      x0 = (float)xv[0]; x1 = (float)xv[1]; y0 = (float)yv[0]; y1 = (float)yv[1];
    } else {
      x0 = bf16_bits_to_f((uint16_t)(x & 0xffff)); x1 = bf16_bits_to_f((uint16_t)(x >> 16));
      y0 = bf16_bits_to_f((uint16_t)(y & 0xffff)); y1 = bf16_bits_to_f((uint16_t)(y >> 16));
    }
    s += x0 * y0 + x1 * y1;
  }
  return s;
}
template <typename T>
__device__ __forceinline__ void store4(uint16_t* p, float a, float b, float c, float d) {
  u32x2 v = {AMfma<T>::pack2(a, b), AMfma<T>::pack2(c, d)};
  *reinterpret_cast<u32x2*>(p) = v;
}

// Results leave the matrix cores with 4 consecutive columns of a row per register quadruple; stored directly, every
// 128-byte row of a result would be written in eight 16-byte pieces.  A block instead parks its 64 x 64 result in an
// LDS tile it no longer needs (pitch P halfs) and then stores whole rows, 8 threads x 16 bytes each.
template <typename T, int P>
__device__ __forceinline__ void park_rows(uint16_t* S, int r, int half, const f32x16 (&acc)[2], float mul) {
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg)
      store4<T>(S + r * P + db * 32 + rg * 8 + half * 4, acc[db][rg * 4] * mul, acc[db][rg * 4 + 1] * mul, acc[db][rg * 4 + 2] * mul,
                acc[db][rg * 4 + 3] * mul);
}
// rows [row0, row0 + 64) of the parked tile to G (row stride ld), rows at or beyond nvalid left out
template <int P>
__device__ __forceinline__ void store_rows(uint16_t* __restrict__ G, int ld, int row0, int nvalid, const uint16_t* S) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + ATT_THREADS * i;
    const int r = v >> 3, c = (v & 7) * 8;
    if (row0 + r < nvalid) *reinterpret_cast<u32x4*>(G + (size_t)(row0 + r) * ld + c) = *reinterpret_cast<const u32x4*>(S + r * P + c);
  }
}

// ---- forward ------------------------------------------------------------------------------------------------------------
template <typename T, bool DROP, bool PACK>
__global__ __launch_bounds__(ATT_THREADS, ATT_FWD_MIN_WAVES) void attn_fwd_mfma_kernel(AttnP p, int H) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[CH * PT];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[CH * PT];
  // Blocks are dispatched x fastest: x walks the (sentence, head) pairs and y the query chunks from the last one down, so
  // under a causal mask (chunk c loops over c + 1 key chunks) the longest blocks of the whole launch start first.
  // With a group table (one-chunk launches only) a block serves a run of consecutive sentences packed into one 64-row tile;
  // a query then admits the keys klo .. khi-1 of the tile, those of its own sentence.
  const int bi = blockIdx.x / H, h = blockIdx.x - bi * H;
  int b0, b1, q0, lq, k0, lk;
  if (PACK) {                                        // (two independent 16-byte loads: no deeper than the offsets' own)
    const int4 g0 = p.groups[bi], g1 = p.groups[bi + 1];
    b0 = g0.x; b1 = g1.x; q0 = g0.y; lq = g1.y - q0; k0 = g0.z; lk = g1.z - k0;
  } else {
    b0 = bi; b1 = bi + 1;
    q0 = p.q_off[b0]; lq = p.q_off[b1] - q0; k0 = p.k_off[b0]; lk = p.k_off[b1] - k0;
  }
  const int qstart = ((int)gridDim.y - 1 - (int)blockIdx.y) * 64;
  if (qstart >= lq) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int qi0 = qstart + wave * 32;
  const bool active = qi0 < lq;
  const int qi = qi0 + (lane & 31);
  int klo = 0, khi = lk, qpos = qi;                  // admissible keys of the tile; the query's position inside its sentence
  if (PACK) {
    // lanes 0 .. 16 fetch the tile-relative offsets of the group's sentences (one load each, in flight together with the
    // Q, K and V rows); every lane then finds its own sentence among them by exchange, without touching memory again
    const int bb = min(b0 + (lane & 31), b1);
    const int qo = p.q_off[bb] - q0, ko = p.k_off[bb] - k0;
    khi = 0;
    for (int j = 0; j < b1 - b0; ++j) {
      const int qs = __shfl(qo, j, 64), qe = __shfl(qo, j + 1, 64), ks = __shfl(ko, j, 64), ke = __shfl(ko, j + 1, 64);
      if (qi >= qs && qi < qe) { klo = ks; khi = ke; qpos = qi - qs; }
    }
  }
  const uint16_t* Q = p.q + (size_t)q0 * p.ldq + h * DH;
  const uint16_t* K = p.k + (size_t)k0 * p.ldk + h * DH;
  const uint16_t* V = p.v + (size_t)k0 * p.ldv + h * DH;
  u32x4 qf[4];
  load_frags(qf, Q, p.ldq, qi0, lq, lane);
  float m = -INFINITY, lsum = 0.f;
  f32x16 acc[2];
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc[0][e] = 0.f; acc[1][e] = 0.f; }
  const int kend = p.causal ? min(lk, qstart + 64) : lk;
  u32x4 kx[4], vx[4];                               // the next chunk's K and V rows, in flight
  fetch_tile(kx, K, p.ldk, 0, lk);
  fetch_tile(vx, V, p.ldv, 0, lk);
  for (int kc = 0; kc < kend; kc += CH) {
    __syncthreads();
    put_tile(Ks, kx);
    put_tile(Vs, vx);
    __syncthreads();
    if (kc + CH < kend) {
      fetch_tile(kx, K, p.ldk, kc + CH, lk);
      fetch_tile(vx, V, p.ldv, kc + CH, lk);
    }
    if (!active) continue;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int j0 = kc + kb * 32;
      if (j0 >= kend) break;
      f32x16 s;
#pragma unroll
      for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) s = AMfma<T>::run(frag_direct(Ks, kb * 32, kk, lane), qf[kk], s);
      float bm = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
        const bool ok = PACK ? (j >= klo && j < khi && (!p.causal || j - klo <= qpos)) : (j < lk && (!p.causal || j <= qi));
        s[r] = ok ? s[r] * p.scale : -INFINITY;
        bm = fmaxf(bm, s[r]);
      }
      bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
      // One sentence per tile: mn is finite from the first block on (key 0 is valid for every query).  A query of a packed
      // tile may admit no key of the first 32-key block: the running maximum is kept out of exp then.
      const float mn = PACK ? fmaxf(fmaxf(m, bm), -3.0e38f) : fmaxf(m, bm);
      const float alpha = __expf(m - mn);
      float ps = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = __expf(s[r] - mn); ps += s[r]; }
      if (DROP) {                                    // the row sum keeps every weight; only the weights that average V are dropped
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint64_t w = attn_drop_word(p, q0 + qi, h, j0 + 8 * g + 4 * half);
#pragma unroll
          for (int f = 0; f < 4; ++f) s[g * 4 + f] = drop_keep(w, f, p.drop_thr) ? s[g * 4 + f] * p.inv_keep : 0.f;
        }
      }
      lsum = lsum * alpha + ps;
      m = mn;
#pragma unroll
      for (int e = 0; e < 16; ++e) { acc[0][e] *= alpha; acc[1][e] *= alpha; }
      u32x4 pf[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int w = 0; w < 4; ++w) pf[ks][w] = AMfma<T>::pack2(s[ks * 8 + 2 * w], s[ks * 8 + 2 * w + 1]);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) acc[db] = AMfma<T>::run(frag_tr(Vs, db * 32, kb * 32 + ks * 16, lane), pf[ks], acc[db]);
    }
  }
  lsum += __shfl_xor(lsum, 32, 64);
  __syncthreads();                                   // every wavefront is done with the K tile
  park_rows<T, PT>(Ks, wave * 32 + (lane & 31), half, acc, active && qi < lq ? 1.f / lsum : 0.f);
  if (active && qi < lq && half == 0) p.lse[(size_t)h * p.total_q + q0 + qi] = m + logf(lsum);
  __syncthreads();
  store_rows<PT>(p.out + (size_t)q0 * p.ldo + h * DH, p.ldo, qstart, lq, Ks);
}

// ---- backward: dQ ---------------------------------------------------------------------------------------------------------
template <typename T, bool DROP>
__device__ __forceinline__ void attn_bwd_dq_body(const AttnP& p, int b, int h, int chunk, uint16_t* Ks, uint16_t* Vs) {
  const int q0 = p.q_off[b], lq = p.q_off[b + 1] - q0, k0 = p.k_off[b], lk = p.k_off[b + 1] - k0;
  const int qstart = chunk * 64;
  if (qstart >= lq) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int qi0 = qstart + wave * 32;
  const bool active = qi0 < lq;
  const int qi = qi0 + (lane & 31);
  const uint16_t* K = p.k + (size_t)k0 * p.ldk + h * DH;
  const uint16_t* V = p.v + (size_t)k0 * p.ldv + h * DH;
  u32x4 qf[4], gf[4], of[4];
  load_frags(qf, p.q + (size_t)q0 * p.ldq + h * DH, p.ldq, qi0, lq, lane);
  load_frags(gf, p.d_o + (size_t)q0 * p.lddo + h * DH, p.lddo, qi0, lq, lane);
  load_frags(of, p.o + (size_t)q0 * p.ldo + h * DH, p.ldo, qi0, lq, lane);
  float delta = 0.f;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) delta += dot8<T>(gf[kk], of[kk]);
  delta += __shfl_xor(delta, 32, 64);
  const float L = qi < lq ? p.lse[(size_t)h * p.total_q + q0 + qi] : 0.f;
  f32x16 acc[2];
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc[0][e] = 0.f; acc[1][e] = 0.f; }
  const int kend = p.causal ? min(lk, qstart + 64) : lk;
  u32x4 kx[4], vx[4];
  fetch_tile(kx, K, p.ldk, 0, lk);
  fetch_tile(vx, V, p.ldv, 0, lk);
  for (int kc = 0; kc < kend; kc += CH) {
    __syncthreads();
    put_tile(Ks, kx);
    put_tile(Vs, vx);
    __syncthreads();
    if (kc + CH < kend) {
      fetch_tile(kx, K, p.ldk, kc + CH, lk);
      fetch_tile(vx, V, p.ldv, kc + CH, lk);
    }
    if (!active) continue;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int j0 = kc + kb * 32;
      if (j0 >= kend) break;
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = AMfma<T>::run(frag_direct(Ks, kb * 32, kk, lane), qf[kk], s);
        dp = AMfma<T>::run(frag_direct(Vs, kb * 32, kk, lane), gf[kk], dp);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint64_t w = DROP ? attn_drop_word(p, q0 + qi, h, j0 + 8 * g + 4 * half) : 0;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          const int r = g * 4 + f;
          const int j = j0 + 8 * g + 4 * half + f;
          const bool ok = j < lk && qi < lq && (!p.causal || j <= qi);
          const float pr = ok ? __expf(s[r] * p.scale - L) : 0.f;
          const float dpd = !DROP ? dp[r] : (drop_keep(w, f, p.drop_thr) ? dp[r] * p.inv_keep : 0.f);   // d/d(softmax output)
          s[r] = pr * (dpd - delta);
        }
      }
      u32x4 df[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int w = 0; w < 4; ++w) df[ks][w] = AMfma<T>::pack2(s[ks * 8 + 2 * w], s[ks * 8 + 2 * w + 1]);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) acc[db] = AMfma<T>::run(frag_tr(Ks, db * 32, kb * 32 + ks * 16, lane), df[ks], acc[db]);
    }
  }
  __syncthreads();
  park_rows<T, PT>(Ks, wave * 32 + (lane & 31), half, acc, p.scale);
  __syncthreads();
  store_rows<PT>(p.dq + (size_t)q0 * p.lddq + h * DH, p.lddq, qstart, lq, Ks);
}

// ---- backward: dK, dV -------------------------------------------------------------------------------------------------------
template <typename T, bool DROP>
__device__ __forceinline__ void attn_bwd_dkv_body(const AttnP& p, int b, int h, int chunk, uint16_t* Qs, uint16_t* Gs, float* Ls, float* Ds) {
  const int q0 = p.q_off[b], lq = p.q_off[b + 1] - q0, k0 = p.k_off[b], lk = p.k_off[b + 1] - k0;
  const int kstart = chunk * 64;
  if (kstart >= lk) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int kj0 = kstart + wave * 32;
  const bool active = kj0 < lk;
  const int kj = kj0 + (lane & 31);
  const uint16_t* Q = p.q + (size_t)q0 * p.ldq + h * DH;
  const uint16_t* G = p.d_o + (size_t)q0 * p.lddo + h * DH;
  const uint16_t* O = p.o + (size_t)q0 * p.ldo + h * DH;
  u32x4 kf[4], vf[4];
  load_frags(kf, p.k + (size_t)k0 * p.ldk + h * DH, p.ldk, kj0, lk, lane);
  load_frags(vf, p.v + (size_t)k0 * p.ldv + h * DH, p.ldv, kj0, lk, lane);
  f32x16 ak[2], av[2];
#pragma unroll
  for (int e = 0; e < 16; ++e) { ak[0][e] = ak[1][e] = av[0][e] = av[1][e] = 0.f; }
  const int qbeg = p.causal ? kstart : 0;     // queries before the chunk's first key see none of its keys
  for (int qc = qbeg; qc < lq; qc += CH) {
    __syncthreads();
    // stage Q and dO; the 8 threads that share a row also form delta = dO . O for it
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = threadIdx.x + ATT_THREADS * i;
      const int r = v >> 3, c = (v & 7) * 8;
      u32x4 xq = {0u, 0u, 0u, 0u}, xg = xq, xo = xq;
      if (qc + r < lq) {
        xq = *reinterpret_cast<const u32x4*>(Q + (size_t)(qc + r) * p.ldq + c);
        xg = *reinterpret_cast<const u32x4*>(G + (size_t)(qc + r) * p.lddo + c);
        xo = *reinterpret_cast<const u32x4*>(O + (size_t)(qc + r) * p.ldo + c);
      }
      *reinterpret_cast<u32x4*>(Qs + r * PT + c) = xq;
      *reinterpret_cast<u32x4*>(Gs + r * PT + c) = xg;
      float dl = dot8<T>(xg, xo);
      dl += __shfl_xor(dl, 1, 64);
      dl += __shfl_xor(dl, 2, 64);
      dl += __shfl_xor(dl, 4, 64);
      if ((v & 7) == 0) {
        Ds[r] = dl;
        Ls[r] = qc + r < lq ? p.lse[(size_t)h * p.total_q + q0 + qc + r] : 0.f;
      }
    }
    __syncthreads();
    if (!active) continue;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int i0 = qc + qb * 32;
      if (i0 >= lq) break;
      if (p.causal && i0 + 31 < kj0) continue;       // every query of this block precedes every key of this wavefront
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = AMfma<T>::run(frag_direct(Qs, qb * 32, kk, lane), kf[kk], s);
        dp = AMfma<T>::run(frag_direct(Gs, qb * 32, kk, lane), vf[kk], dp);
      }
      u32x4 pf[2], df[2];
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int il = qb * 32 + rg * 8 + half * 4;
        const float4 l4 = *reinterpret_cast<const float4*>(Ls + il);
        const float4 d4 = *reinterpret_cast<const float4*>(Ds + il);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
        float pr[4], dsv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = qc + il + e;
          const bool ok = i < lq && kj < lk && (!p.causal || kj <= i);
          pr[e] = ok ? __expf(s[rg * 4 + e] * p.scale - lv[e]) : 0.f;
          float dpd = dp[rg * 4 + e];
          if (DROP) {                                  // this lane's key, one query per register: a word per element
            const bool keep = drop_keep(attn_drop_word(p, q0 + i, h, kj), kj & 3, p.drop_thr);
            dpd = keep ? dpd * p.inv_keep : 0.f;
            dsv[e] = pr[e] * (dpd - dv[e]);
            pr[e] = keep ? pr[e] * p.inv_keep : 0.f;  // dV averages dO with the dropped weights
          } else {
            dsv[e] = pr[e] * (dpd - dv[e]);
          }
        }
        pf[rg >> 1][(rg & 1) * 2] = AMfma<T>::pack2(pr[0], pr[1]);
        pf[rg >> 1][(rg & 1) * 2 + 1] = AMfma<T>::pack2(pr[2], pr[3]);
        df[rg >> 1][(rg & 1) * 2] = AMfma<T>::pack2(dsv[0], dsv[1]);
        df[rg >> 1][(rg & 1) * 2 + 1] = AMfma<T>::pack2(dsv[2], dsv[3]);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          av[db] = AMfma<T>::run(frag_tr(Gs, db * 32, qb * 32 + ks * 16, lane), pf[ks], av[db]);
          ak[db] = AMfma<T>::run(frag_tr(Qs, db * 32, qb * 32 + ks * 16, lane), df[ks], ak[db]);
        }
    }
  }
  __syncthreads();
  park_rows<T, PT>(Qs, wave * 32 + (lane & 31), half, ak, p.scale);
  park_rows<T, PT>(Gs, wave * 32 + (lane & 31), half, av, 1.f);
  __syncthreads();
  store_rows<PT>(p.dk + (size_t)k0 * p.lddk + h * DH, p.lddk, kstart, lk, Qs);
  store_rows<PT>(p.dv + (size_t)k0 * p.lddv + h * DH, p.lddv, kstart, lk, Gs);
}

// One launch for the whole backward: nq_chunks blocks per (sentence, head) compute dQ, nk_chunks dK/dV; the two halves are
// independent, so they run side by side instead of one after the other.  Blocks are dispatched x fastest: x walks the
// (sentence, head) pairs and y the chunks in the order of decreasing work under a causal mask (dK/dV of key chunk c loops
// over n - c query chunks, dQ of query chunk c over c + 1 key chunks), so the longest blocks of the whole launch start
// first and the short ones fill the tail.
template <typename T, bool DROP>
__global__ __launch_bounds__(ATT_THREADS, ATT_BWD_MIN_WAVES) void attn_bwd_mfma_kernel(AttnP p, int nq_chunks, int nk_chunks, int H) {
  __shared__ __attribute__((aligned(16))) uint16_t S0[CH * PT];
  __shared__ __attribute__((aligned(16))) uint16_t S1[CH * PT];
  __shared__ __attribute__((aligned(16))) float Ls[CH];
  __shared__ __attribute__((aligned(16))) float Ds[CH];
  const int b = blockIdx.x / H, h = blockIdx.x - b * H;
  // y = 0, 1, 2, 3, ... -> dK/dV chunk 0, dQ chunk nq-1, dK/dV chunk 1, dQ chunk nq-2, ... while both kinds last
  const int r = blockIdx.y, pairs = min(nq_chunks, nk_chunks);
  bool is_dq;
  int chunk;
  if (r < 2 * pairs) { is_dq = r & 1; chunk = is_dq ? nq_chunks - 1 - (r >> 1) : (r >> 1); }
  else if (nq_chunks > nk_chunks) { is_dq = true; chunk = nq_chunks - 1 - (r - pairs); }
  else { is_dq = false; chunk = r - pairs; }
  if (is_dq) attn_bwd_dq_body<T, DROP>(p, b, h, chunk, S0, S1);
  else attn_bwd_dkv_body<T, DROP>(p, b, h, chunk, S0, S1, Ls, Ds);
}

// ---- backward, sentences of at most 64 tokens: dQ, dK and dV of a (sentence, head) in one block --------------------------
// When every sentence of the launch fits one chunk (most batches of the translation workloads: sentences of similar
// length share a batch), the two halves above would each fetch the five tiles Q, K, V, O, dO of the same (sentence,
// head).  Here one block stages them once and uses them for both: its wavefronts' queries against K, V (dQ) and their
// keys against Q, dO (dK, dV).  The scores are formed in both orientations by the matrix cores, which are nearly idle in
// this kernel anyway, so nothing is transposed through LDS; the operand fragments of the block's own rows also come from
// the staged tiles, so every input is read from memory exactly once.  Four tiles at a 144-byte pitch (16 rows x 16
// bytes cover the 64 banks once) keep four blocks resident per CU.
constexpr int PF = 72;

// Short sentences are packed: a block serves a run of consecutive sentences whose query rows and key rows (contiguous in the
// packed token layout) fill at most one 64-row tile each.  The products are formed over the whole tile; a weight counts
// only where query and key belong to the same sentence, which each row looks up as the range of admissible partners
// (QR: keys of a query's sentence, KR: queries of a key's sentence, both relative to the tile).
template <typename T, bool DROP, bool PACK>
__global__ __launch_bounds__(ATT_THREADS, 2) void attn_bwd_single_kernel(AttnP p) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[CH * PF];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[CH * PF];
  __shared__ __attribute__((aligned(16))) uint16_t Qs[CH * PF];
  __shared__ __attribute__((aligned(16))) uint16_t Gs[CH * PF];
  __shared__ __attribute__((aligned(16))) float Ls[CH];
  __shared__ __attribute__((aligned(16))) float Ds[CH];
  __shared__ int QR[CH], KR[CH];                     // partner range lo | hi << 8, own sentence's first row << 16
  const int h = blockIdx.y;
  int b0, b1, q0, lq, k0, lk;                        // lq, lk in [1, 64]
  if (PACK) {
    const int4 g0 = p.groups[blockIdx.z], g1 = p.groups[blockIdx.z + 1];
    b0 = g0.x; b1 = g1.x; q0 = g0.y; lq = g1.y - q0; k0 = g0.z; lk = g1.z - k0;
  } else {
    b0 = blockIdx.z; b1 = b0 + 1;
    q0 = p.q_off[b0]; lq = p.q_off[b1] - q0; k0 = p.k_off[b0]; lk = p.k_off[b1] - k0;
  }
  if (threadIdx.x < CH) {                            // (the first wavefront: one lane per tile row)
    const int r = threadIdx.x;
    int qr = 0, kr = 0;                              // empty ranges for rows beyond the tile's sentences
    if (PACK) {
      const int bb = min(b0 + (r & 31), b1);         // lanes 0 .. 16 hold the sentences' tile-relative offsets
      const int qo = p.q_off[bb] - q0, ko = p.k_off[bb] - k0;
      for (int j = 0; j < b1 - b0; ++j) {
        const int qs = __shfl(qo, j, 64), qe = __shfl(qo, j + 1, 64), ks = __shfl(ko, j, 64), ke = __shfl(ko, j + 1, 64);
        if (r >= qs && r < qe) qr = ks | (ke << 8) | (qs << 16);
        if (r >= ks && r < ke) kr = qs | (qe << 8) | (ks << 16);
      }
    } else {
      if (r < lq) qr = lk << 8;
      if (r < lk) kr = lq << 8;
    }
    QR[r] = qr;
    KR[r] = kr;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int own0 = wave * 32;                        // first own row of this wavefront (a query for dQ, a key for dK/dV)
  const int own = own0 + (lane & 31);
  const uint16_t* Q = p.q + (size_t)q0 * p.ldq + h * DH;
  const uint16_t* G = p.d_o + (size_t)q0 * p.lddo + h * DH;
  const uint16_t* O = p.o + (size_t)q0 * p.ldo + h * DH;
  stage_tile<PF>(Ks, p.k + (size_t)k0 * p.ldk + h * DH, p.ldk, 0, lk);
  stage_tile<PF>(Vs, p.v + (size_t)k0 * p.ldv + h * DH, p.ldv, 0, lk);
  // stage Q and dO; the 8 threads that share a row also form delta = dO . O for it
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int v = threadIdx.x + ATT_THREADS * i;
    const int r = v >> 3, cc = (v & 7) * 8;
    u32x4 xq = {0u, 0u, 0u, 0u}, xg = xq, xo = xq;
    if (r < lq) {
      xq = *reinterpret_cast<const u32x4*>(Q + (size_t)r * p.ldq + cc);
      xg = *reinterpret_cast<const u32x4*>(G + (size_t)r * p.lddo + cc);
      xo = *reinterpret_cast<const u32x4*>(O + (size_t)r * p.ldo + cc);
    }
    *reinterpret_cast<u32x4*>(Qs + r * PF + cc) = xq;
    *reinterpret_cast<u32x4*>(Gs + r * PF + cc) = xg;
    float dl = dot8<T>(xg, xo);
    dl += __shfl_xor(dl, 1, 64);
    dl += __shfl_xor(dl, 2, 64);
    dl += __shfl_xor(dl, 4, 64);
    if ((v & 7) == 0) {
      Ds[r] = dl;
      Ls[r] = r < lq ? p.lse[(size_t)h * p.total_q + q0 + r] : 0.f;
    }
  }
  __syncthreads();
  f32x16 aq[2], ak[2], av[2];
#pragma unroll
  for (int e = 0; e < 16; ++e) { aq[0][e] = aq[1][e] = ak[0][e] = ak[1][e] = av[0][e] = av[1][e] = 0.f; }
  if (own0 < lq) {
    // dQ^T[d][query] = K^T dS^T with S^T[key][query]: a lane owns one query, 16 keys in registers
    const float delta = Ds[own], L = Ls[own];
    const int klo = QR[own] & 0xff, khi = (QR[own] >> 8) & 0xff, qpos = own - (QR[own] >> 16);   // position inside the sentence
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int j0 = kb * 32;
      if (j0 >= lk) break;
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = AMfma<T>::run(frag_direct<PF>(Ks, j0, kk, lane), frag_direct<PF>(Qs, own0, kk, lane), s);
        dp = AMfma<T>::run(frag_direct<PF>(Vs, j0, kk, lane), frag_direct<PF>(Gs, own0, kk, lane), dp);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // (with dropout a block serves one sentence, so tile keys are sentence keys and a word covers 4 of them)
        const uint64_t w = DROP ? attn_drop_word(p, q0 + own, h, j0 + 8 * g + 4 * half) : 0;
#pragma unroll
        for (int f = 0; f < 4; ++f) {
          const int r = g * 4 + f;
          const int jj = j0 + 8 * g + 4 * half + f;
          const bool ok = jj >= klo && jj < khi && (!p.causal || jj - klo <= qpos);
          const float pr = ok ? __expf(s[r] * p.scale - L) : 0.f;
          const float dpd = !DROP ? dp[r] : (drop_keep(w, f, p.drop_thr) ? dp[r] * p.inv_keep : 0.f);
          s[r] = pr * (dpd - delta);
        }
      }
      u32x4 df[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int w = 0; w < 4; ++w) df[ks][w] = AMfma<T>::pack2(s[ks * 8 + 2 * w], s[ks * 8 + 2 * w + 1]);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) aq[db] = AMfma<T>::run(frag_tr<PF>(Ks, db * 32, j0 + ks * 16, lane), df[ks], aq[db]);
    }
  }
  if (own0 < lk) {
    // dK^T[d][key] = Q^T dS, dV^T[d][key] = dO^T P with S[query][key]: a lane owns one key, 16 queries in registers
    const int qlo = KR[own] & 0xff, qhi = (KR[own] >> 8) & 0xff, kpos = own - (KR[own] >> 16);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int i0 = qb * 32;
      if (i0 >= lq) break;
      if (p.causal && !PACK && i0 + 31 < own0) continue;      // (one sentence) every query of this block precedes every key of this wavefront
      f32x16 s, dp;
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = AMfma<T>::run(frag_direct<PF>(Qs, i0, kk, lane), frag_direct<PF>(Ks, own0, kk, lane), s);
        dp = AMfma<T>::run(frag_direct<PF>(Gs, i0, kk, lane), frag_direct<PF>(Vs, own0, kk, lane), dp);
      }
      u32x4 pf[2], df[2];
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int il = i0 + rg * 8 + half * 4;
        const float4 l4 = *reinterpret_cast<const float4*>(Ls + il);
        const float4 d4 = *reinterpret_cast<const float4*>(Ds + il);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
        float pr[4], dsv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = il + e;
          const bool ok = i >= qlo && i < qhi && (!p.causal || kpos <= i - qlo);
          pr[e] = ok ? __expf(s[rg * 4 + e] * p.scale - lv[e]) : 0.f;
          float dpd = dp[rg * 4 + e];
          if (DROP) {
            const bool keep = drop_keep(attn_drop_word(p, q0 + i, h, own), own & 3, p.drop_thr);
            dpd = keep ? dpd * p.inv_keep : 0.f;
            dsv[e] = pr[e] * (dpd - dv[e]);
            pr[e] = keep ? pr[e] * p.inv_keep : 0.f;
          } else {
            dsv[e] = pr[e] * (dpd - dv[e]);
          }
        }
        pf[rg >> 1][(rg & 1) * 2] = AMfma<T>::pack2(pr[0], pr[1]);
        pf[rg >> 1][(rg & 1) * 2 + 1] = AMfma<T>::pack2(pr[2], pr[3]);
        df[rg >> 1][(rg & 1) * 2] = AMfma<T>::pack2(dsv[0], dsv[1]);
        df[rg >> 1][(rg & 1) * 2 + 1] = AMfma<T>::pack2(dsv[2], dsv[3]);
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          av[db] = AMfma<T>::run(frag_tr<PF>(Gs, db * 32, i0 + ks * 16, lane), pf[ks], av[db]);
          ak[db] = AMfma<T>::run(frag_tr<PF>(Qs, db * 32, i0 + ks * 16, lane), df[ks], ak[db]);
        }
    }
  }
  __syncthreads();                                   // the tiles are no longer needed: park the three results in them
  park_rows<T, PF>(Qs, own, half, aq, p.scale);
  park_rows<T, PF>(Ks, own, half, ak, p.scale);
  park_rows<T, PF>(Vs, own, half, av, 1.f);
  __syncthreads();
  store_rows<PF>(p.dq + (size_t)q0 * p.lddq + h * DH, p.lddq, 0, lq, Qs);
  store_rows<PF>(p.dk + (size_t)k0 * p.lddk + h * DH, p.lddk, 0, lk, Ks);
  store_rows<PF>(p.dv + (size_t)k0 * p.lddv + h * DH, p.lddv, 0, lk, Vs);
}

static bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

bool attention_mfma_supported(const AttnArgs& a, bool bwd) {
  if (a.dt != F16 && a.dt != BF16) return false;
  if (a.dh != DH) return false;
  if (a.ldq % 8 || a.ldk % 8 || a.ldv % 8 || a.ldo % 8) return false;
  if (!al16(a.q) || !al16(a.k) || !al16(a.v) || !al16(a.o)) return false;
  if (bwd) {
    if (a.lddo % 8 || a.lddq % 8 || a.lddk % 8 || a.lddv % 8) return false;
    if (!al16(a.d_o) || !al16(a.dq) || !al16(a.dk) || !al16(a.dv)) return false;
  }
  return true;
}

static AttnP make_params(const AttnArgs& a) {
  AttnP p;
  p.q = (const uint16_t*)a.q; p.k = (const uint16_t*)a.k; p.v = (const uint16_t*)a.v; p.o = (const uint16_t*)a.o;
  p.d_o = (const uint16_t*)a.d_o; p.out = (uint16_t*)a.o; p.dq = (uint16_t*)a.dq; p.dk = (uint16_t*)a.dk; p.dv = (uint16_t*)a.dv;
  p.ldq = a.ldq; p.ldk = a.ldk; p.ldv = a.ldv; p.ldo = a.ldo; p.lddo = a.lddo; p.lddq = a.lddq; p.lddk = a.lddk; p.lddv = a.lddv;
  p.lse = a.lse; p.q_off = a.q_off; p.k_off = a.k_off; p.total_q = a.total_q; p.causal = a.causal;
  p.scale = 1.f / sqrtf((float)a.dh);
  p.drop_key = a.drop_key;
  p.drop_thr = a.drop_p > 0.f ? drop_threshold(a.drop_p) : 0u;
  p.inv_keep = 1.f / (1.f - a.drop_p);
  p.H = a.H;
  p.groups = nullptr;
  return p;
}

void launch_attention_fwd_mfma(hipStream_t s, const AttnArgs& a) {
  AttnP p = make_params(a);
  const bool drop = p.drop_thr != 0;
  // (measured over sentence lengths 11 .. 64 at ~3500 tokens: the forward kernel gains from sharing tiles only from about
  // three sentences per tile on; below that the group lookup costs what the saved blocks bring)
  const bool packed = a.groups != nullptr && a.n_groups > 0 && !drop && a.max_lq <= 64 && a.max_lk <= 64 && 3 * a.n_groups <= a.B;
  p.groups = packed ? (const int4*)a.groups : nullptr;
  dim3 grid(a.H * (packed ? a.n_groups : a.B), (a.max_lq + 63) / 64), block(ATT_THREADS);
  if (a.dt == F16) {
    if (drop) hipLaunchKernelGGL((attn_fwd_mfma_kernel<half_t, true, false>), grid, block, 0, s, p, a.H);
    else if (packed) hipLaunchKernelGGL((attn_fwd_mfma_kernel<half_t, false, true>), grid, block, 0, s, p, a.H);
    else hipLaunchKernelGGL((attn_fwd_mfma_kernel<half_t, false, false>), grid, block, 0, s, p, a.H);
  } else {
    if (drop) hipLaunchKernelGGL((attn_fwd_mfma_kernel<bf16_t, true, false>), grid, block, 0, s, p, a.H);
    else if (packed) hipLaunchKernelGGL((attn_fwd_mfma_kernel<bf16_t, false, true>), grid, block, 0, s, p, a.H);
    else hipLaunchKernelGGL((attn_fwd_mfma_kernel<bf16_t, false, false>), grid, block, 0, s, p, a.H);
  }
}

void launch_attention_bwd_mfma(hipStream_t s, const AttnArgs& a) {
  AttnP p = make_params(a);
  const int nq = (a.max_lq + 63) / 64, nk = (a.max_lk + 63) / 64;
  const bool drop = p.drop_thr != 0;
  if (nq == 1 && nk == 1) {                              // every sentence fits one chunk: one block per (group of sentences, head)
    // (the backward kernel gains from 1.5 sentences per tile on: 41 -> 20 us at 11-token sentences, 27 -> 19 us at 21 tokens)
    const bool packed = a.groups != nullptr && a.n_groups > 0 && !drop && 3 * a.n_groups <= 2 * a.B;
    p.groups = packed ? (const int4*)a.groups : nullptr;
    dim3 grid(1, a.H, packed ? a.n_groups : a.B), block(ATT_THREADS);
    if (a.dt == F16) {
      if (drop) hipLaunchKernelGGL((attn_bwd_single_kernel<half_t, true, false>), grid, block, 0, s, p);
      else if (packed) hipLaunchKernelGGL((attn_bwd_single_kernel<half_t, false, true>), grid, block, 0, s, p);
      else hipLaunchKernelGGL((attn_bwd_single_kernel<half_t, false, false>), grid, block, 0, s, p);
    } else {
      if (drop) hipLaunchKernelGGL((attn_bwd_single_kernel<bf16_t, true, false>), grid, block, 0, s, p);
      else if (packed) hipLaunchKernelGGL((attn_bwd_single_kernel<bf16_t, false, true>), grid, block, 0, s, p);
      else hipLaunchKernelGGL((attn_bwd_single_kernel<bf16_t, false, false>), grid, block, 0, s, p);
    }
    return;
  }
  dim3 grid(a.H * a.B, nq + nk), block(ATT_THREADS);
  if (a.dt == F16) {
    if (drop) hipLaunchKernelGGL((attn_bwd_mfma_kernel<half_t, true>), grid, block, 0, s, p, nq, nk, a.H);
    else hipLaunchKernelGGL((attn_bwd_mfma_kernel<half_t, false>), grid, block, 0, s, p, nq, nk, a.H);
  } else {
    if (drop) hipLaunchKernelGGL((attn_bwd_mfma_kernel<bf16_t, true>), grid, block, 0, s, p, nq, nk, a.H);
    else hipLaunchKernelGGL((attn_bwd_mfma_kernel<bf16_t, false>), grid, block, 0, s, p, nq, nk, a.H);
  }
}

}  // namespace tfm
