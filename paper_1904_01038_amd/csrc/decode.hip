// Kernels of the incremental decoding step (Implementation, Inference): a per-row key/value cache indexed through an
// ancestry table, so a step computes exactly one new position per row.
//
// Cache layout.  Self-attention keys and values of decoder layer l live in K_l, V_l [rows][max_steps][d]: row r writes
// position t of ITS OWN row at step t and never moves anything.  When the search re-orders the beams, only an
// ancestry table changes: anc[r][s] is the physical row that holds position s of the hypothesis now living in row r
// (anc_new[r][s] = anc_old[parent[r]][s] for s < t, anc_new[r][t] = r).  Beams that share a prefix therefore read the
// same cache lines (L2 hits) and a re-ordering costs rows * t integers instead of a copy of every layer's cache.
// Cross-attention keys and values are projected once per source sentence and shared by its beams.
#include "common.h"
#include "kernels.h"

namespace tfm {

__global__ __launch_bounds__(256) void ancestry_kernel(const int* __restrict__ anc_old, int* __restrict__ anc_new,
                                                       const int* __restrict__ parent, int rows, int max_steps, int t) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * (t + 1)) return;
  const int r = i / (t + 1), s = i - r * (t + 1);
  anc_new[(size_t)r * max_steps + s] = s < t ? anc_old[(size_t)parent[r] * max_steps + s] : r;
}
void launch_ancestry(hipStream_t s, const int* anc_old, int* anc_new, const int* parent, int rows, int max_steps, int t) {
  const int n = rows * (t + 1);
  hipLaunchKernelGGL(ancestry_kernel, dim3((n + 255) / 256), dim3(256), 0, s, anc_old, anc_new, parent, rows, max_steps, t);
}

// K[r][t][:] = qkv[r][d .. 2d), V[r][t][:] = qkv[r][2d .. 3d)
template <typename T>
__global__ __launch_bounds__(256) void cache_append_kernel(const T* __restrict__ qkv, T* __restrict__ Kc, T* __restrict__ Vc,
                                                           int rows, int d, int max_steps, int t) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * d) return;
  const int r = i / d, e = i - r * d;
  const size_t dst = ((size_t)r * max_steps + t) * d + e;
  Kc[dst] = qkv[(size_t)r * 3 * d + d + e];
  Vc[dst] = qkv[(size_t)r * 3 * d + 2 * d + e];
}
void launch_cache_append(hipStream_t s, int dt, const void* qkv, void* Kc, void* Vc, int rows, int d, int max_steps, int t) {
  const int n = rows * d;
  dim3 grid((n + 255) / 256), block(256);
  if (dt == F32) hipLaunchKernelGGL(cache_append_kernel<float>, grid, block, 0, s, (const float*)qkv, (float*)Kc, (float*)Vc, rows, d, max_steps, t);
  else if (dt == F16) hipLaunchKernelGGL(cache_append_kernel<half_t>, grid, block, 0, s, (const half_t*)qkv, (half_t*)Kc, (half_t*)Vc, rows, d, max_steps, t);
  else hipLaunchKernelGGL(cache_append_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)qkv, (bf16_t*)Kc, (bf16_t*)Vc, rows, d, max_steps, t);
}

// One wavefront per (row, head): a single query against n positions.
//   phase 1  lane = position: score = q . K[pos] / sqrt(dh), kept in LDS together with the row's address
//   phase 2  softmax over the positions (fp32)
//   phase 3  lane = feature: out[e] = sum_pos p[pos] V[pos][e]; a V row of one head is one 128-byte line at dh = 64
template <typename T, int VEC>
__global__ __launch_bounds__(64) void decode_attention_kernel(DecodeAttnArgs p) {
  extern __shared__ float smem[];
  const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x, dh = p.dh;
  int n, base = 0;
  if (p.anc) n = p.t + 1;
  else { const int s = r / p.beam; base = p.src_off[s]; n = p.src_off[s + 1] - base; }
  float* sc = smem;                                    // [n_max] scores, then probabilities
  int* rowi = reinterpret_cast<int*>(smem + p.n_max);  // [n_max] element offset of the position's K row / V row
  float* qs = smem + 2 * p.n_max;                      // [dh]
  const T* q = reinterpret_cast<const T*>(p.q) + (size_t)r * p.ldq + h * dh;
  for (int e = lane; e < dh; e += 64) qs[e] = to_f<T>(q[e]);
  const T* K = reinterpret_cast<const T*>(p.k);
  const T* V = reinterpret_cast<const T*>(p.v);
  __syncthreads();
  const float scale = rsqrtf((float)dh);
  float lmax = -INFINITY;
  for (int s = lane; s < n; s += 64) {
    // element offset of (position s, head h) from the K and V bases (both have the same strides)
    const long long off = p.anc ? ((long long)p.anc[(size_t)r * p.max_steps + s] * p.max_steps + s) * p.row_stride + h * dh
                                : (long long)(base + s) * p.row_stride + h * dh;
    const T* kr = K + off;
    float acc = 0.f;
    for (int e = 0; e < dh; e += VEC) {
      float kv[VEC];
      load_f<T, VEC>(kr + e, kv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc += qs[e + i] * kv[i];
    }
    acc *= scale;
    sc[s] = acc;
    // offsets fit in 32 bits: the host checks that every cache and projection holds fewer than 2^31 elements
    rowi[s] = (int)off;
    lmax = fmaxf(lmax, acc);
  }
  const float m = wave_max(lmax);
  float lsum = 0.f;
  for (int s = lane; s < n; s += 64) {
    const float e = __expf(sc[s] - m);
    sc[s] = e;
    lsum += e;
  }
  const float inv = 1.f / wave_sum(lsum);
  __syncthreads();
  T* out = reinterpret_cast<T*>(p.o) + (size_t)r * p.ldo + h * dh;
  for (int e = lane; e < dh; e += 64) {
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int s = 0;
    for (; s + 4 <= n; s += 4) {
      a0 += sc[s] * to_f<T>(V[rowi[s] + e]);
      a1 += sc[s + 1] * to_f<T>(V[rowi[s + 1] + e]);
      a2 += sc[s + 2] * to_f<T>(V[rowi[s + 2] + e]);
      a3 += sc[s + 3] * to_f<T>(V[rowi[s + 3] + e]);
    }
    for (; s < n; ++s) a0 += sc[s] * to_f<T>(V[rowi[s] + e]);
    out[e] = from_f<T>((a0 + a1 + a2 + a3) * inv);
  }
}

// The same for head width 64 and 2-byte elements, arranged so that no phase waits for more than one round trip to memory:
//   phase 1  lane = position: the 8 loads of a key row are issued together
//   phase 3  lane = (position group g = lane / 8, feature vector f = lane % 8): a lane reads 16 bytes of V for the positions
//            s = g, g + 8, ... (four of them in flight), and the eight groups are added up with three lane exchanges
template <typename T>
__global__ __launch_bounds__(64) void decode_attention64_kernel(DecodeAttnArgs p) {
  extern __shared__ float smem[];
  constexpr int dh = 64;
  const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  int n, base = 0;
  if (p.anc) n = p.t + 1;
  else { const int s = r / p.beam; base = p.src_off[s]; n = p.src_off[s + 1] - base; }
  float* sc = smem;
  int* rowi = reinterpret_cast<int*>(smem + p.n_max);
  float* qs = smem + 2 * p.n_max;
  if (p.q_partial) {                                   // the query arrives as the slices of a split-K product (at most 8)
    const size_t at = (size_t)r * p.H * dh + h * dh + lane, slice = (size_t)p.rows * p.H * dh;
    float part[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) part[k] = k < p.q_splits ? p.q_partial[k * slice + at] : 0.f;
    float qv = part[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) qv += part[k];
    if (p.q_bias) qv += to_f<T>(reinterpret_cast<const T*>(p.q_bias)[h * dh + lane]);
    qs[lane] = to_f<T>(from_f<T>(qv));                 // rounded as the stored projection would be
  } else {
    const T* q = reinterpret_cast<const T*>(p.q) + (size_t)r * p.ldq + h * dh;
    qs[lane] = to_f<T>(q[lane]);
  }
  const T* K = reinterpret_cast<const T*>(p.k);
  const T* V = reinterpret_cast<const T*>(p.v);
  // position t of a self-attention step may still be outside the caches: it is read from the new rows, and 16 lanes copy
  // this head's 128 + 128 bytes into the row's own cache lines for the steps to come (nobody reads them during this launch)
  const T* knew = nullptr;
  const T* vnew = nullptr;
  if (p.anc && p.k_new) {
    knew = reinterpret_cast<const T*>(p.k_new) + (size_t)r * p.ld_new + h * dh;
    vnew = reinterpret_cast<const T*>(p.v_new) + (size_t)r * p.ld_new + h * dh;
    if (lane < 16) {
      const size_t dst = ((size_t)r * p.max_steps + p.t) * p.row_stride + h * dh + (lane & 7) * 8;
      typedef unsigned int u4 __attribute__((ext_vector_type(4)));
      const T* src = (lane < 8 ? knew : vnew) + (lane & 7) * 8;
      T* cache = const_cast<T*>(lane < 8 ? K : V);
      *reinterpret_cast<u4*>(cache + dst) = *reinterpret_cast<const u4*>(src);
    }
  }
  __syncthreads();
  const float scale = 0.125f;
  float lmax = -INFINITY;
  for (int s = lane; s < n; s += 64) {
    const long long off = p.anc ? ((long long)p.anc[(size_t)r * p.max_steps + s] * p.max_steps + s) * p.row_stride + h * dh
                                : (long long)(base + s) * p.row_stride + h * dh;
    const T* kr = (knew && s == p.t) ? knew : K + off;
    float kv[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) load_f<T, 8>(kr + j * 8, kv[j]);
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += qs[j * 8 + i] * kv[j][i];
    acc *= scale;
    sc[s] = acc;
    rowi[s] = (int)off;
    lmax = fmaxf(lmax, acc);
  }
  const float m = wave_max(lmax);
  float lsum = 0.f;
  for (int s = lane; s < n; s += 64) {
    const float e = __expf(sc[s] - m);
    sc[s] = e;
    lsum += e;
  }
  const float inv = 1.f / wave_sum(lsum);
  __syncthreads();
  const int g = lane >> 3, f = lane & 7;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s0 = g; s0 < n; s0 += 32) {
    float v[4][8], w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int s = s0 + 8 * u;
      w[u] = s < n ? sc[s] : 0.f;
      const int sv = s < n ? s : s0;                                // (a position past the end re-reads a valid row, weight 0)
      load_f<T, 8>(((vnew && sv == p.t) ? vnew : V + rowi[sv]) + f * 8, v[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += w[u] * v[u][i];
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    acc[i] += __shfl_xor(acc[i], 8, 64);
    acc[i] += __shfl_xor(acc[i], 16, 64);
    acc[i] += __shfl_xor(acc[i], 32, 64);
    acc[i] *= inv;
  }
  if (g == 0) store_f<T, 8>(reinterpret_cast<T*>(p.o) + (size_t)r * p.ldo + h * dh + f * 8, acc);
}

// (16-byte accesses: the host side lays q, the caches and the output out with head slices at multiples of 128 bytes)
static bool decode_attention_fast(const DecodeAttnArgs& a) {
  return a.dh == 64 && a.dt != F32 && a.ldq % 8 == 0 && a.row_stride % 8 == 0 && a.ldo % 8 == 0 && (!a.k_new || a.ld_new % 8 == 0);
}
bool decode_attention_appends(const DecodeAttnArgs& a) { return a.anc && a.k_new && a.v_new && decode_attention_fast(a); }

void launch_decode_attention(hipStream_t s, const DecodeAttnArgs& a) {
  if (a.rows <= 0) return;
  dim3 grid(a.rows, a.H), block(64);
  const size_t smem = (size_t)(2 * a.n_max + a.dh) * sizeof(float);
  if (decode_attention_fast(a) && a.q_splits <= 8) {
    if (a.dt == F16) hipLaunchKernelGGL((decode_attention64_kernel<half_t>), grid, block, smem, s, a);
    else hipLaunchKernelGGL((decode_attention64_kernel<bf16_t>), grid, block, smem, s, a);
    return;
  }
  if (a.q_partial)                                     // the general kernel reads a finished query: finish it into q first
    launch_splitk_reduce(s, a.dt, a.q_partial, a.q_splits, a.rows, a.H * a.dh, const_cast<void*>(a.q), a.ldq, a.q_bias);
  const bool vec = a.dh % 8 == 0;
#define DA(T, VEC) hipLaunchKernelGGL((decode_attention_kernel<T, VEC>), grid, block, smem, s, a)
  if (a.dt == F32) { if (vec) DA(float, 8); else DA(float, 1); }
  else if (a.dt == F16) { if (vec) DA(half_t, 8); else DA(half_t, 1); }
  else { if (vec) DA(bf16_t, 8); else DA(bf16_t, 1); }
#undef DA
}

// Per row: log-sum-exp of the logits and the K best tokens.  Order: larger value first, equal values by ascending id.
__device__ __forceinline__ bool better(float v, int i, float w, int j) { return v > w || (v == w && i < j); }

template <typename T, int K>
__global__ __launch_bounds__(256) void row_topk_kernel(const T* __restrict__ z, int ldz, int V, float* __restrict__ top_logp,
                                                       int* __restrict__ top_id, float* __restrict__ lse_out, int k_out) {
  __shared__ float sh[16];
  __shared__ float cand_v[4];
  __shared__ int cand_i[4], cand_owner[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const T* zr = z + (size_t)row * ldz;
  float bv[K];
  int bi[K];
#pragma unroll
  for (int i = 0; i < K; ++i) { bv[i] = -INFINITY; bi[i] = 0x7fffffff; }
  float m = -INFINITY, ssum = 0.f;
  for (int col = tid; col < V; col += 256) {
    const float v = to_f<T>(zr[col]);
    if (v > m) { ssum = ssum * __expf(m - v) + 1.f; m = v; } else { ssum += __expf(v - m); }
    if (better(v, col, bv[K - 1], bi[K - 1])) {
      float cv = v;
      int ci = col;
#pragma unroll
      for (int i = 0; i < K; ++i) {                      // insertion into the sorted list, static indices only
        if (better(cv, ci, bv[i], bi[i])) {
          const float tv = bv[i]; const int ti = bi[i];
          bv[i] = cv; bi[i] = ci; cv = tv; ci = ti;
        }
      }
    }
  }
  const float gm = block_max(m, sh);
  const float gs = block_sum(ssum * __expf(m - gm), sh);   // (a thread that saw nothing has ssum = 0)
  const float lse = gm + logf(gs);
  if (tid == 0 && lse_out) lse_out[row] = lse;
  // K rounds: the best head among the threads' lists wins and its owner moves on to its next entry
  const int lane = tid & 63, wave = tid >> 6;
  for (int round = 0; round < k_out; ++round) {
    float v = bv[0];
    int id = bi[0], owner = tid;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(v, o);
      const int oi = __shfl_xor(id, o), oo = __shfl_xor(owner, o);
      if (better(ov, oi, v, id)) { v = ov; id = oi; owner = oo; }
    }
    if (lane == 0) { cand_v[wave] = v; cand_i[wave] = id; cand_owner[wave] = owner; }
    __syncthreads();
    float wv = cand_v[0];
    int wi = cand_i[0], wo = cand_owner[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
      if (better(cand_v[w], cand_i[w], wv, wi)) { wv = cand_v[w]; wi = cand_i[w]; wo = cand_owner[w]; }
    if (tid == 0) {
      top_logp[(size_t)row * k_out + round] = wv - lse;
      top_id[(size_t)row * k_out + round] = wi;
    }
    if (tid == wo) {
#pragma unroll
      for (int i = 0; i + 1 < K; ++i) { bv[i] = bv[i + 1]; bi[i] = bi[i + 1]; }
      bv[K - 1] = -INFINITY; bi[K - 1] = 0x7fffffff;
    }
    __syncthreads();
  }
}

// The same result with the row held in registers (NCH values per thread, V <= NT * NCH): every thread knows its own
// best value; a round picks the best of those, and only the thread that owned it looks for its next best.
template <typename T, int NCH, int NT>
__global__ __launch_bounds__(NT) void row_topk_cached_kernel(const T* __restrict__ z, int ldz, int V, float* __restrict__ top_logp,
                                                              int* __restrict__ top_id, float* __restrict__ lse_out, int k_out) {
  __shared__ float sh[16];
  __shared__ float cand_v[NT / 64];
  __shared__ int cand_i[NT / 64];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* zr = z + (size_t)row * ldz;
  float c[NCH];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int col = tid + i * NT;
    c[i] = col < V ? to_f<T>(zr[col]) : -INFINITY;
    m = fmaxf(m, c[i]);
  }
  const float gm = block_max(m, sh);
  float se = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) se += __expf(c[i] - gm);                 // exp(-inf) = 0 for the padding
  const float lse = gm + logf(block_sum(se, sh));
  if (tid == 0 && lse_out) lse_out[row] = lse;
  // this thread's best remaining (value, id): columns ascend with i, so the first maximum has the smallest id
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  auto rescan = [&]() {
    bv = -INFINITY; bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < NCH; ++i)
      if (c[i] > bv) { bv = c[i]; bi = tid + i * NT; }
  };
  rescan();
  for (int round = 0; round < k_out; ++round) {
    float v = bv;
    int id = bi;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(v, o);
      const int oi = __shfl_xor(id, o);
      if (better(ov, oi, v, id)) { v = ov; id = oi; }
    }
    if (lane == 0) { cand_v[wave] = v; cand_i[wave] = id; }
    __syncthreads();
    float wv = cand_v[0];
    int wi = cand_i[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w)
      if (better(cand_v[w], cand_i[w], wv, wi)) { wv = cand_v[w]; wi = cand_i[w]; }
    if (tid == 0) {
      top_logp[(size_t)row * k_out + round] = wv - lse;
      top_id[(size_t)row * k_out + round] = wi;
    }
    if (wi % NT == tid) {                                              // the owner drops it and looks again
#pragma unroll
      for (int i = 0; i < NCH; ++i)
        if (tid + i * NT == wi) c[i] = -INFINITY;
      rescan();
    }
    __syncthreads();
  }
}

// The same result again, for rows of whole 8-element vectors: 16-byte loads, and the k rounds run inside each wavefront (lane
// exchanges only, no block barrier); the wavefronts' k candidates each meet in LDS once and one wavefront merges them.
template <typename T, int NV, int NT>
__global__ __launch_bounds__(NT) void row_topk_vec_kernel(const T* __restrict__ z, int ldz, int V, float* __restrict__ top_logp,
                                                           int* __restrict__ top_id, float* __restrict__ lse_out, int k_out) {
  constexpr int NWV = NT / 64;
  __shared__ float sh[16];
  __shared__ float cand_v[NWV * 16];
  __shared__ int cand_i[NWV * 16];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T* zr = z + (size_t)row * ldz;
  float c[NV][8];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int col = (tid + i * NT) * 8;
    if (col < V) load_f<T, 8>(zr + col, c[i]);
    else {
#pragma unroll
      for (int j = 0; j < 8; ++j) c[i][j] = -INFINITY;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) m = fmaxf(m, c[i][j]);
  }
  const float gm = block_max(m, sh);
  float se = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) se += __expf(c[i][j] - gm);              // exp(-inf) = 0 for the padding
  const float lse = gm + logf(block_sum(se, sh));
  if (tid == 0 && lse_out) lse_out[row] = lse;
  // this thread's best remaining (value, id): ids ascend with (i, j), so the first maximum has the smallest id
  float bv;
  int bi;
  auto rescan = [&]() {
    bv = -INFINITY; bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (c[i][j] > bv) { bv = c[i][j]; bi = (tid + i * NT) * 8 + j; }
  };
  rescan();
  for (int round = 0; round < k_out; ++round) {                          // this wavefront's k best, best first
    float v = bv;
    int id = bi;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(v, o);
      const int oi = __shfl_xor(id, o);
      if (better(ov, oi, v, id)) { v = ov; id = oi; }
    }
    if (lane == 0) { cand_v[wave * 16 + round] = v; cand_i[wave * 16 + round] = id; }
    if (id == bi && id != 0x7fffffff) {                                  // the owner drops it and looks again
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if ((tid + i * NT) * 8 + j == id) c[i][j] = -INFINITY;
      rescan();
    }
  }
  __syncthreads();
  if (wave != 0) return;
  // merge: NWV * k_out <= 256 candidates, up to four per lane; a wavefront's list is sorted, but nothing relies on that here
  const int total = NWV * k_out;
  float mv[4];
  int mi[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int idx = lane + 64 * q;
    const bool ok = idx < total;
    const int w = ok ? idx / k_out : 0, r = ok ? idx - w * k_out : 0;
    mv[q] = ok ? cand_v[w * 16 + r] : -INFINITY;
    mi[q] = ok ? cand_i[w * 16 + r] : 0x7fffffff;
  }
  for (int round = 0; round < k_out; ++round) {
    float v = mv[0];
    int id = mi[0];
#pragma unroll
    for (int q = 1; q < 4; ++q)
      if (better(mv[q], mi[q], v, id)) { v = mv[q]; id = mi[q]; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(v, o);
      const int oi = __shfl_xor(id, o);
      if (better(ov, oi, v, id)) { v = ov; id = oi; }
    }
    if (lane == 0) {
      top_logp[(size_t)row * k_out + round] = v - lse;
      top_id[(size_t)row * k_out + round] = id;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (mi[q] == id && id != 0x7fffffff) { mv[q] = -INFINITY; mi[q] = 0x7fffffff; }
  }
}

void launch_row_topk(hipStream_t s, int dt, const void* z, int ldz, int rows, int V, int k, float* top_logp, int* top_id,
                     float* lse) {
  if (rows <= 0) return;
  dim3 grid(rows), block(256);
  if (V % 8 == 0 && ldz % 8 == 0 && ((uintptr_t)z & 15) == 0 && V <= 1024 * 4 * 8 && k <= 16) {
#define TKV(T, NV, NT) hipLaunchKernelGGL((row_topk_vec_kernel<T, NV, NT>), grid, dim3(NT), 0, s, (const T*)z, ldz, V, top_logp, top_id, lse, k)
#define TKVV(T) do { if (V <= 256 * 2 * 8) TKV(T, 2, 256); else TKV(T, 4, 1024); } while (0)
    if (dt == F32) TKVV(float); else if (dt == F16) TKVV(half_t); else TKVV(bf16_t);
#undef TKVV
#undef TKV
    return;
  }
#define TKC(T, NCH, NT) hipLaunchKernelGGL((row_topk_cached_kernel<T, NCH, NT>), grid, dim3(NT), 0, s, (const T*)z, ldz, V, top_logp, top_id, lse, k)
#define TK(T, K) hipLaunchKernelGGL((row_topk_kernel<T, K>), grid, block, 0, s, (const T*)z, ldz, V, top_logp, top_id, lse, k)
#define TKK(T)                                                         \
  do {                                                                 \
    if (V <= 256 * 16) TKC(T, 16, 256);                                \
    else if (V <= 1024 * 32) TKC(T, 32, 1024);                         \
    else if (k <= 8) TK(T, 8);                                         \
    else TK(T, 16);                                                    \
  } while (0)
  if (dt == F32) TKK(float); else if (dt == F16) TKK(half_t); else TKK(bf16_t);
#undef TKK
#undef TK
#undef TKC
}

// out[r][v] = z[r][v] - lse[r] in fp32 (test access to the full distribution)
template <typename T>
__global__ __launch_bounds__(256) void logprob_rows_kernel(const T* __restrict__ z, int ldz, const float* __restrict__ lse,
                                                           float* __restrict__ out, int V) {
  const int row = blockIdx.y;
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col < V) out[(size_t)row * V + col] = to_f<T>(z[(size_t)row * ldz + col]) - lse[row];
}
void launch_logprob_rows(hipStream_t s, int dt, const void* z, int ldz, const float* lse, float* out, int rows, int V) {
  if (rows <= 0) return;
  dim3 grid((V + 255) / 256, rows), block(256);
  if (dt == F32) hipLaunchKernelGGL(logprob_rows_kernel<float>, grid, block, 0, s, (const float*)z, ldz, lse, out, V);
  else if (dt == F16) hipLaunchKernelGGL(logprob_rows_kernel<half_t>, grid, block, 0, s, (const half_t*)z, ldz, lse, out, V);
  else hipLaunchKernelGGL(logprob_rows_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)z, ldz, lse, out, V);
}

}  // namespace tfm
