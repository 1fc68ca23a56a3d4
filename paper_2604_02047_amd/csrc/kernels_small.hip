// Small kernels of the verification step: ancestor mask, embedding gather, residual +
// RMSNorm, rotary embedding + KV-tail write, argmax, greedy walk, KV compaction.
#include <limits.h>

#include "goose_internal.h"

namespace {

template <typename T>
__device__ inline float to_f32(T v) { return (float)v; }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// ------------------------------------------------------------------------------------------
__global__ void k_set_int(int32_t* dst, int v) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *dst = v;
}

// Ancestor-or-self bit rows, depth and position of every node (Sec. 4, tree attention mask).
// One thread per node climbs its own root path; parent[v] < v makes every climb finite.
// A cache length outside what the launch was sized for (P > P_max) or that leaves no room for the
// tree (P + B > cap) raises GOOSE_FLAG_CAPACITY: the later kernels then clamp their indices and the
// step's results are meaningless.
__device__ inline void build_mask_body(const int32_t* __restrict__ parent, int B, const int32_t* __restrict__ dP,
                                       uint64_t* __restrict__ mask, int32_t* __restrict__ depth,
                                       int32_t* __restrict__ pos, int32_t* __restrict__ flags, int cap, int P_max) {
  const int i = threadIdx.x;
  if (i == 0) {
    const int P = *dP;
    if (P < 0 || P > P_max || P + B > cap) atomicOr(flags, GOOSE_FLAG_CAPACITY);
  }
  if (i >= B) return;
  const int W = (B + 63) >> 6;
  uint64_t w0 = 0, w1 = 0;
  int dep = 0;
  bool bad = (i == 0 && parent[0] != -1);
  int v = i;
  for (int it = 0; it < B; ++it) {
    if (v < 64) w0 |= 1ull << v; else w1 |= 1ull << (v - 64);
    if (v == 0) break;
    int p = parent[v];
    if (p < 0 || p >= v) { bad = true; p = 0; }  // never index outside the tree
    v = p;
    ++dep;
  }
  mask[(size_t)i * W] = w0;
  if (W > 1) mask[(size_t)i * W + 1] = w1;
  depth[i] = dep;
  pos[i] = *dP + dep;
  if (bad) atomicOr(flags, GOOSE_FLAG_BAD_PARENT);
}

__global__ __launch_bounds__(128) void k_build_mask(const int32_t* __restrict__ parent, int B,
                                                    const int32_t* __restrict__ dP, uint64_t* __restrict__ mask,
                                                    int32_t* __restrict__ depth, int32_t* __restrict__ pos,
                                                    int32_t* __restrict__ flags, int cap, int P_max) {
  build_mask_body(parent, B, dP, mask, depth, pos, flags, cap, P_max);
}

// The per-request steps of a batch as single launches: block index = request, taken from a table
// that travels as a kernel argument (rows of request r start at row0 in the stacked buffers).
struct ReqTable { BatchReq r[GOOSE_MAX_REQUESTS]; };

__global__ __launch_bounds__(128) void k_build_mask_batch(const ReqTable t, uint64_t* __restrict__ mask,
                                                          int32_t* __restrict__ depth, int32_t* __restrict__ pos,
                                                          int32_t* __restrict__ flags, int cap) {
  const BatchReq& q = t.r[blockIdx.x];
  build_mask_body(q.parent, q.B, q.dP, mask + (size_t)q.row0 * 2, depth + q.row0, pos + q.row0, flags, cap, q.P_max);
}

// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_embed(const T* __restrict__ E, const int32_t* __restrict__ tokens, int H,
                                               int V, float* __restrict__ x) {
  const int m = blockIdx.x;
  int t = tokens[m];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const T* row = E + (size_t)t * H;
  for (int c = threadIdx.x; c < H; c += 256) x[(size_t)m * H + c] = to_f32(row[c]);
}

template <typename T>
__global__ __launch_bounds__(256) void k_embed_batch(const T* __restrict__ E, const ReqTable t, int H, int V,
                                                     float* __restrict__ x) {
  const BatchReq& q = t.r[blockIdx.y];
  const int i = blockIdx.x;
  if (i >= q.B) return;
  int tok = q.tokens[i];
  tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
  const T* row = E + (size_t)tok * H;
  float* xr = x + (size_t)(q.row0 + i) * H;
  for (int c = threadIdx.x; c < H; c += 256) xr[c] = to_f32(row[c]);
}

// ------------------------------------------------------------------------------------------
// x[m] += sum of S partial GEMM outputs; xn[m] = T(x[m] * rsqrt(mean(x[m]^2) + eps) * g).
// One workgroup per row, four columns per thread per pass (H is a multiple of 4), all loads of a
// pass independent so the few rows still pull their partials at full memory parallelism.
template <typename T>
__device__ inline void store4(T* p, float a, float b, float c, float d);
template <>
__device__ inline void store4<float>(float* p, float a, float b, float c, float d) {
  *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
template <>
__device__ inline void store4<bf16_t>(bf16_t* p, float a, float b, float c, float d) {
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
  *reinterpret_cast<bf16x4*>(p) = v;
}
template <>
__device__ inline void store4<_Float16>(_Float16* p, float a, float b, float c, float d) {
  typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
  f16x4 v = {(_Float16)a, (_Float16)b, (_Float16)c, (_Float16)d};
  *reinterpret_cast<f16x4*>(p) = v;
}

// TERMS = 2 (16-bit types): xn is written as hi + lo, lo = T(v - hi), in groups of eight columns
// (8 hi values, then their 8 lo values; row length 2 * columns): the operand layout of the projections.
// Tg: type of the gains; T: type of xn (fp16 activations may meet bf16 gains).
template <typename Tg, typename T, int NTHR, int TERMS>
__global__ __launch_bounds__(NTHR) void k_resid_norm(float* __restrict__ x, int H, const float* __restrict__ part,
                                                     int S, size_t part_stride, size_t part_ld,
                                                     const Tg* __restrict__ g, float eps, T* __restrict__ xn,
                                                     int ldxn) {
  constexpr int MAXV = 4;  // float4 slots per thread kept in registers (H <= 16 * NTHR)
  const int m = blockIdx.x;
  float* xr = x + (size_t)m * H;
  const int nvec = H >> 2;
  float4 v[MAXV];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int c4 = threadIdx.x + i * NTHR;
    if (c4 < nvec) {
      float4 a = *reinterpret_cast<const float4*>(xr + c4 * 4);
      // the slices are added in index order, four loads in flight at a time (one load per loop
      // round would make every slice its own trip to memory)
      const float* pp = part + (size_t)m * part_ld + c4 * 4;
      int s = 0;
      for (; s + 4 <= S; s += 4) {
        float4 p[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) p[k] = *reinterpret_cast<const float4*>(pp + (size_t)(s + k) * part_stride);
#pragma unroll
        for (int k = 0; k < 4; ++k) { a.x += p[k].x; a.y += p[k].y; a.z += p[k].z; a.w += p[k].w; }
      }
      for (; s < S; ++s) {
        const float4 p = *reinterpret_cast<const float4*>(pp + (size_t)s * part_stride);
        a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
      }
      if (S > 0) *reinterpret_cast<float4*>(xr + c4 * 4) = a;
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
      v[i] = a;
    }
  }
  if (xn == nullptr) return;
  __shared__ float red[NTHR / 64];
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < NTHR / 64; ++w) tot += red[w];
  const float rstd = 1.0f / sqrtf(tot / (float)H + eps);
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int c4 = threadIdx.x + i * NTHR;
    if (c4 < nvec) {
      const Tg* gp = g + c4 * 4;
      const float o0 = (v[i].x * rstd) * to_f32(gp[0]), o1 = (v[i].y * rstd) * to_f32(gp[1]);
      const float o2 = (v[i].z * rstd) * to_f32(gp[2]), o3 = (v[i].w * rstd) * to_f32(gp[3]);
      if (TERMS == 1) {
        store4<T>(xn + (size_t)m * ldxn + c4 * 4, o0, o1, o2, o3);
      } else {  // columns 4 c4 .. 4 c4 + 3 lie inside one group of eight
        T* dst = xn + (size_t)m * ldxn + (size_t)(c4 >> 1) * 16 + (c4 & 1) * 4;
        const T h0 = (T)o0, h1 = (T)o1, h2 = (T)o2, h3 = (T)o3;
        store4<T>(dst, to_f32(h0), to_f32(h1), to_f32(h2), to_f32(h3));
        store4<T>(dst + 8, o0 - to_f32(h0), o1 - to_f32(h1), o2 - to_f32(h2), o3 - to_f32(h3));
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Sum the split-K partials of the fused q|k|v projection, rotate q and k by the node's
// position (half-split pairing (j, j+d/2), angle pos * base^(-2j/d)) and store q for the
// attention kernel, k into cache slot P + m of K[head][slot][d], and v into the TRANSPOSED
// value cache Vt[head][d][slot].  Grid (node, head); thread j owns the pair (j, j + d/2).
template <typename T>
__global__ void k_rope_kv(const float* __restrict__ part, int S, size_t part_stride, size_t part_ld, int n_heads,
                          int head_dim, const int32_t* __restrict__ pos, const double* __restrict__ inv_freq,
                          const int32_t* __restrict__ dP, int cap, T* __restrict__ qout, int ldq,
                          T* __restrict__ kcache, T* __restrict__ vtcache, int32_t* __restrict__ flags) {
  const int m = blockIdx.x, h = blockIdx.y, j = threadIdx.x;
  const int half = head_dim >> 1;
  const int Hq = n_heads * head_dim;
  const int slot = *dP + m;
  if (slot < 0 || slot >= cap) {  // no room for this node: say so instead of writing outside the cache
    if (j == 0 && h == 0) atomicOr(flags, GOOSE_FLAG_CAPACITY);
    return;
  }
  float v6[6] = {0, 0, 0, 0, 0, 0};
  for (int s = 0; s < S; ++s) {
    const float* r = part + s * part_stride + (size_t)m * part_ld + h * head_dim + j;
    v6[0] += r[0];
    v6[1] += r[half];
    v6[2] += r[Hq];
    v6[3] += r[Hq + half];
    v6[4] += r[2 * Hq];
    v6[5] += r[2 * Hq + half];
  }
  // reduce the angle in double, then evaluate in float: |error| ~ 1e-7 rad at any position
  double ang = (double)pos[m] * inv_freq[j];
  const double two_pi = 6.283185307179586476925286766559;
  ang -= two_pi * rint(ang / two_pi);
  float sn, cs;
  sincosf((float)ang, &sn, &cs);
  const float q1 = v6[0] * cs - v6[1] * sn, q2 = v6[1] * cs + v6[0] * sn;
  const float k1 = v6[2] * cs - v6[3] * sn, k2 = v6[3] * cs + v6[2] * sn;
  T* qo = qout + (size_t)m * ldq + h * head_dim + j;
  qo[0] = (T)q1;
  qo[half] = (T)q2;
  const size_t row = ((size_t)h * cap + slot) * head_dim + j;
  kcache[row] = (T)k1;
  kcache[row + half] = (T)k2;
  T* vcol = vtcache + ((size_t)h * head_dim + j) * cap + slot;
  vcol[0] = (T)v6[4];
  vcol[(size_t)half * cap] = (T)v6[5];
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_swiglu_f32(const float* __restrict__ gu, size_t ld, int F,
                                                    float* __restrict__ h, int ldh) {
  const int m = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= F) return;
  const float g = gu[(size_t)m * ld + c], u = gu[(size_t)m * ld + F + c];
  h[(size_t)m * ldh + c] = g / (1.0f + expf(-g)) * u;
}

// ------------------------------------------------------------------------------------------
struct Top2 {
  float v1, v2;
  int i1;
};
__device__ inline Top2 top2_merge(Top2 a, Top2 b) {
  const bool a_first = (a.v1 > b.v1) || (a.v1 == b.v1 && a.i1 < b.i1);
  Top2 r;
  if (a_first) { r.v1 = a.v1; r.i1 = a.i1; r.v2 = fmaxf(a.v2, b.v1); }
  else         { r.v1 = b.v1; r.i1 = b.i1; r.v2 = fmaxf(b.v2, a.v1); }
  return r;
}

// Per-row argmax (lowest index on ties) and top-1 minus top-2 margin.
__global__ __launch_bounds__(256) void k_argmax(const float* __restrict__ logits, size_t ld, int V,
                                                int32_t* __restrict__ argmax, float* __restrict__ margin) {
  const int m = blockIdx.x;
  const float* row = logits + (size_t)m * ld;
  Top2 t = {-INFINITY, -INFINITY, INT_MAX};
  for (int c = threadIdx.x; c < V; c += 256) {
    Top2 e = {row[c], -INFINITY, c};
    t = top2_merge(t, e);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    Top2 o;
    o.v1 = __shfl_xor(t.v1, off, 64);
    o.v2 = __shfl_xor(t.v2, off, 64);
    o.i1 = __shfl_xor(t.i1, off, 64);
    t = top2_merge(t, o);
  }
  __shared__ Top2 red[4];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    Top2 r = top2_merge(top2_merge(red[0], red[1]), top2_merge(red[2], red[3]));
    argmax[m] = r.i1;
    if (margin) margin[m] = r.v1 - r.v2;
  }
}

// Same from the per-workgroup reductions of the LM-head kernel (groups cover ascending column ranges).
__global__ __launch_bounds__(64) void k_argmax_top2(const float4* __restrict__ top2, int n_groups,
                                                    int32_t* __restrict__ argmax, float* __restrict__ margin) {
  const int m = blockIdx.x;
  Top2 t = {-INFINITY, -INFINITY, INT_MAX};
  for (int g = threadIdx.x; g < n_groups; g += 64) {
    const float4 e = top2[(size_t)m * n_groups + g];
    Top2 o = {e.x, e.y, __float_as_int(e.z)};
    t = top2_merge(t, o);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    Top2 o;
    o.v1 = __shfl_xor(t.v1, off, 64);
    o.v2 = __shfl_xor(t.v2, off, 64);
    o.i1 = __shfl_xor(t.i1, off, 64);
    t = top2_merge(t, o);
  }
  if (threadIdx.x == 0) {
    argmax[m] = t.i1;
    if (margin) margin[m] = t.v1 - t.v2;
  }
}

// ------------------------------------------------------------------------------------------
// Logit harvest (Sec. 4 stage 2; App. C, adjacency table tier 1): row tokens[m] of the dense
// [vocab][K] successor tables receives the K most likely next tokens of node m (ids, ordered by
// decreasing logit, equal logits by increasing id) and their softmax probabilities.  When several
// nodes carry the same token the highest node index writes (the others skip the store).
// One workgroup per node, two passes over its row:
//   1. every thread finds the best (logit, id) pair of its strided share and an online
//      log-sum-exp; the K-th best of the 256 thread-bests, tau, is a lower bound of the K-th best
//      of the row (there are K pairs at or above it);
//   2. the pairs at or above tau -- K of them plus a few -- are appended to a short list in LDS,
//      from which K rounds of a workgroup-wide maximum pop the winners in order.
// A row whose list would overflow (many pairs above tau inside one thread's share) takes the
// plain route instead: every thread keeps its best KMAX pairs in sorted registers.
__device__ inline bool cand_before(float av, int ai, float bv, int bi) { return av > bv || (av == bv && ai < bi); }

// Workgroup-wide best of every thread's (v, i); all 256 threads call it.  s_v/s_i: 4-entry LDS scratch.
__device__ inline void block_best(float& v, int& i, float* s_v, int* s_i) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(v, off, 64);
    const int oi = __shfl_xor(i, off, 64);
    if (cand_before(ov, oi, v, i)) { v = ov; i = oi; }
  }
  __syncthreads();  // the previous call's readers are done
  if ((threadIdx.x & 63) == 0) { s_v[threadIdx.x >> 6] = v; s_i[threadIdx.x >> 6] = i; }
  __syncthreads();
  v = s_v[0]; i = s_i[0];
#pragma unroll
  for (int w = 1; w < 4; ++w)
    if (cand_before(s_v[w], s_i[w], v, i)) { v = s_v[w]; i = s_i[w]; }
}

// Sorted insert of (v, c) into a thread's best-first list of N pairs.
template <int N>
__device__ inline void list_insert(float (&tv)[N], int (&ti)[N], float v, int c) {
  if (!cand_before(v, c, tv[N - 1], ti[N - 1])) return;
  tv[N - 1] = v;
  ti[N - 1] = c;
#pragma unroll
  for (int j = N - 1; j > 0; --j) {
    if (cand_before(tv[j], ti[j], tv[j - 1], ti[j - 1])) {
      const float fv = tv[j]; tv[j] = tv[j - 1]; tv[j - 1] = fv;
      const int fi = ti[j]; ti[j] = ti[j - 1]; ti[j - 1] = fi;
    }
  }
}

// K rounds: the workgroup's best head wins, its owner pops it, thread 0 stores the winner.
template <int N>
__device__ inline void pop_rounds(float (&tv)[N], int (&ti)[N], int K, bool writes, int tok, float M, float S,
                                  int32_t* succ_ids, float* succ_scores, float* s_v, int* s_i) {
  for (int k = 0; k < K; ++k) {
    float bv = tv[0];
    int bi = ti[0];
    block_best(bv, bi, s_v, s_i);
    if (ti[0] == bi && bi != INT_MAX) {  // token ids are unique: exactly one owner
#pragma unroll
      for (int j = 0; j < N - 1; ++j) { tv[j] = tv[j + 1]; ti[j] = ti[j + 1]; }
      tv[N - 1] = -INFINITY;
      ti[N - 1] = INT_MAX;
    }
    if (threadIdx.x == 0 && writes) {
      const bool real = bi != INT_MAX;
      succ_ids[(size_t)tok * K + k] = real ? bi : -1;
      succ_scores[(size_t)tok * K + k] = real ? __expf(bv - M) / S : 0.f;
    }
  }
}

template <int KMAX>
__global__ __launch_bounds__(256) void k_harvest_topk(const float* __restrict__ logits, size_t ld, int V,
                                                      const int32_t* __restrict__ tokens, int B, int K, int table_rows,
                                                      int32_t* __restrict__ succ_ids,
                                                      float* __restrict__ succ_scores) {
  constexpr int DEPTH = 16;   // loads in flight per thread: the row was written by the previous kernel
  constexpr int LIST = 4;     // list entries per thread on the short route
  constexpr int CAP = 256 * LIST;
  __shared__ float s_v[4];
  __shared__ int s_i[4];
  __shared__ float s_m[4], s_s[4];
  __shared__ float c_v[CAP];
  __shared__ int c_i[CAP];
  __shared__ int c_n, s_dup;
  const int m = blockIdx.x, tid = threadIdx.x;
  const float* row = logits + (size_t)m * ld;
  if (tid == 0) { c_n = 0; s_dup = 0; }

  // ---- pass 1: thread-best pair and log-sum-exp
  float bv = -INFINITY, mx = -INFINITY, sm = 0.f;
  int bi = INT_MAX;
  for (int c0 = tid; c0 < V; c0 += 256 * DEPTH) {
    float vals[DEPTH];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) vals[u] = (c0 + u * 256 < V) ? row[c0 + u * 256] : NAN;
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      const float v = vals[u];
      if (!(v == v)) continue;  // past the row, or NaN: not a candidate
      if (v > mx) { sm = sm * __expf(mx - v) + 1.f; mx = v; }
      else sm += __expf(v - mx);
      if (v > bv) { bv = v; bi = c0 + u * 256; }  // ids ascend within a thread: '>' keeps the lowest
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float om = __shfl_xor(mx, off, 64), os = __shfl_xor(sm, off, 64);
    const float nm = fmaxf(mx, om);
    sm = (nm == -INFINITY) ? 0.f : sm * __expf(mx - nm) + os * __expf(om - nm);
    mx = nm;
  }
  if ((tid & 63) == 0) { s_m[tid >> 6] = mx; s_s[tid >> 6] = sm; }
  // does this node write?  (a valid token, and no later node with the same token)
  const int tok = tokens[m];
  __syncthreads();
  if (tid > m && tid < B && tokens[tid] == tok) s_dup = 1;
  const float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
  float S = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) S += (s_m[w] == -INFINITY) ? 0.f : s_s[w] * __expf(s_m[w] - M);

  // ---- tau: the K-th best of the thread-bests
  float tau_v = -INFINITY;
  int tau_i = INT_MAX;
  for (int k = 0; k < K; ++k) {
    float wv = bv;
    int wi = bi;
    block_best(wv, wi, s_v, s_i);
    if (wi == bi && bi != INT_MAX) { bv = -INFINITY; bi = INT_MAX; }
    tau_v = wv;
    tau_i = wi;  // (-inf, INT_MAX) once the thread-bests run out: then every pair qualifies
  }
  const bool writes = tok >= 0 && tok < table_rows && s_dup == 0;  // s_dup settled by the barriers above

  // ---- pass 2: pairs at or above tau into the list
  for (int c0 = tid; c0 < V; c0 += 256 * DEPTH) {
    float vals[DEPTH];
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) vals[u] = (c0 + u * 256 < V) ? row[c0 + u * 256] : NAN;
#pragma unroll
    for (int u = 0; u < DEPTH; ++u) {
      const float v = vals[u];
      const int c = c0 + u * 256;
      if (v == v && !cand_before(tau_v, tau_i, v, c)) {
        const int pos = atomicAdd(&c_n, 1);
        if (pos < CAP) { c_v[pos] = v; c_i[pos] = c; }
      }
    }
  }
  __syncthreads();
  const int n = c_n;
  if (n <= CAP) {
    float tv[LIST];
    int ti[LIST];
#pragma unroll
    for (int j = 0; j < LIST; ++j) { tv[j] = -INFINITY; ti[j] = INT_MAX; }
    for (int e = tid; e < n; e += 256) list_insert<LIST>(tv, ti, c_v[e], c_i[e]);
    pop_rounds<LIST>(tv, ti, K, writes, tok, M, S, succ_ids, succ_scores, s_v, s_i);
    return;
  }
  // ---- plain route (wave-uniform: n is shared)
  float tv[KMAX];
  int ti[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) { tv[j] = -INFINITY; ti[j] = INT_MAX; }
  for (int c = tid; c < V; c += 256) {
    const float v = row[c];
    if (v == v) list_insert<KMAX>(tv, ti, v, c);
  }
  pop_rounds<KMAX>(tv, ti, K, writes, tok, M, S, succ_ids, succ_scores, s_v, s_i);
}

// ------------------------------------------------------------------------------------------
// Greedy walk (Alg. UnifiedGreedyWalk).  Every node whose own edge matches (its token equals the prediction
// at its parent) bids for its parent with the key (branch?1:0, node index); the lowest key
// wins, i.e. spine children before branch children, lower index first.  Thread 0 then follows
// the winners from the root; node indices grow along any path, so the walk is finite.
__device__ inline void accept_body(const int32_t* __restrict__ parent, const int32_t* __restrict__ tokens,
                                   const uint8_t* __restrict__ is_spine, const int32_t* __restrict__ argmax, int B,
                                   int32_t* __restrict__ accept_len, int32_t* __restrict__ path,
                                   int32_t* __restrict__ bonus, int32_t* __restrict__ next_root) {
  __shared__ int nxt[GOOSE_MAX_B];
  __shared__ int xh[GOOSE_MAX_B];
  __shared__ int L_sh;
  const int i = threadIdx.x;
  if (i < B) {
    nxt[i] = INT_MAX;
    xh[i] = argmax[i];
  }
  __syncthreads();
  if (i >= 1 && i < B) {
    const int p = parent[i];
    if (p >= 0 && p < i && tokens[i] == xh[p]) {
      const int branch = (is_spine != nullptr && is_spine[i] == 0) ? 1 : 0;
      atomicMin(&nxt[p], (branch << 16) | i);
    }
  }
  __syncthreads();
  if (i == 0) {
    int v = 0, L = 0;
    path[0] = 0;
    while (nxt[v] != INT_MAX && L < B - 1) {
      v = nxt[v] & 0xFFFF;
      path[++L] = v;
    }
    *accept_len = L;
    *bonus = xh[v];
    if (next_root) *next_root = xh[v];
    L_sh = L;
  }
  __syncthreads();
  if (i > L_sh && i < B) path[i] = -1;
}

__global__ __launch_bounds__(128) void k_accept(const int32_t* __restrict__ parent, const int32_t* __restrict__ tokens,
                                                const uint8_t* __restrict__ is_spine,
                                                const int32_t* __restrict__ argmax, int B,
                                                int32_t* __restrict__ accept_len, int32_t* __restrict__ path,
                                                int32_t* __restrict__ bonus, int32_t* __restrict__ next_root) {
  accept_body(parent, tokens, is_spine, argmax, B, accept_len, path, bonus, next_root);
}

__global__ __launch_bounds__(128) void k_accept_batch(const ReqTable t, const int32_t* __restrict__ argmax_all) {
  const BatchReq& q = t.r[blockIdx.x];
  accept_body(q.parent, q.tokens, q.is_spine, argmax_all + q.row0, q.B, q.accept_len, q.path, q.bonus, q.next_root);
}

// ------------------------------------------------------------------------------------------
// Commit of the accepted path: cache slot P + path[j] -> slot P + j, j = 1..L, in every layer and head.
// K[head][slot][d]: one thread owns one 16-byte column chunk of all rows.  Vt[head][d][slot]: one thread
// owns one d-row and moves single elements along it.  Either way a thread walks j upward and
// path[j] >= j, so a slot is always read before the same thread can overwrite it.
__global__ __launch_bounds__(64) void k_compact_k(uint4* __restrict__ kall, int cap, int row_chunks,
                                                  const int32_t* __restrict__ dP, const int32_t* __restrict__ path,
                                                  const int32_t* __restrict__ accept_len) {
  const int c = threadIdx.x;
  if (c >= row_chunks) return;
  uint4* base = kall + (size_t)blockIdx.x * cap * row_chunks;  // blockIdx.x = layer * n_heads + head
  const int P = *dP;
  int L = *accept_len;
  if (L > GOOSE_MAX_B - 1) L = GOOSE_MAX_B - 1;
  for (int j = 1; j <= L; ++j) {
    const int src = path[j];
    if (src < j || src >= GOOSE_MAX_B || P + src >= cap) break;  // malformed path: stop, stay in bounds
    if (src != j) base[(size_t)(P + j) * row_chunks + c] = base[(size_t)(P + src) * row_chunks + c];
  }
}

// The same for bf16 caches in MFMA operand order (32-key blocks; the layouts are spelled out in
// goose.h): thread c moves chunk c of the K row (16 bytes) and column c of the V row (2 bytes).
template <int D>
__device__ inline void compact_tiled_body(bf16_t* __restrict__ kall, bf16_t* __restrict__ vall, int cap,
                                          const int32_t* __restrict__ dP, const int32_t* __restrict__ path,
                                          const int32_t* __restrict__ accept_len) {
  const int c = threadIdx.x;
  bf16_t* kb = kall + (size_t)blockIdx.x * cap * D;  // blockIdx.x = layer * n_heads + head
  bf16_t* vb = vall + (size_t)blockIdx.x * cap * D;
  const int P = *dP;
  int L = *accept_len;
  if (L > GOOSE_MAX_B - 1) L = GOOSE_MAX_B - 1;
  auto k_off = [](int g, int ch) {  // chunk ch = 2*s + hh of slot g
    const int kk = g & 31, i = (((kk >> 2) & 3) << 3) | ((kk >> 4) << 2) | (kk & 3);
    return (((size_t)(g >> 5) * (D / 16) + (ch >> 1)) * 64 + i + 32 * (ch & 1)) * 8;
  };
  auto v_off = [](int g, int col) {
    const int kk = g & 31;
    return ((((size_t)(g >> 5) * (D / 32) + (col >> 5)) * 2 + ((kk >> 3) & 1)) * 64 + (col & 31) + 32 * (kk >> 4)) * 8 +
           (kk & 7);
  };
  for (int j = 1; j <= L; ++j) {
    const int src = path[j];
    if (src < j || src >= GOOSE_MAX_B || P + src >= cap) break;  // malformed path: stop, stay in bounds
    if (src == j) continue;
    if (c < D / 8)
      *reinterpret_cast<uint4*>(kb + k_off(P + j, c)) = *reinterpret_cast<const uint4*>(kb + k_off(P + src, c));
    vb[v_off(P + j, c)] = vb[v_off(P + src, c)];
  }
}

template <int D>
__global__ __launch_bounds__(D) void k_compact_tiled(bf16_t* __restrict__ kall, bf16_t* __restrict__ vall, int cap,
                                                     const int32_t* __restrict__ dP,
                                                     const int32_t* __restrict__ path,
                                                     const int32_t* __restrict__ accept_len) {
  compact_tiled_body<D>(kall, vall, cap, dP, path, accept_len);
}

template <int D>
__global__ __launch_bounds__(D) void k_compact_tiled_batch(const ReqTable t, int cap) {
  const BatchReq& q = t.r[blockIdx.y];
  compact_tiled_body<D>((bf16_t*)q.kall, (bf16_t*)q.vall, cap, q.dP, q.path, q.accept_len);
}

template <typename T>
__global__ void k_compact_vt(T* __restrict__ vall, int cap, int head_dim, const int32_t* __restrict__ dP,
                             const int32_t* __restrict__ path, const int32_t* __restrict__ accept_len) {
  const int c = threadIdx.x;  // d index
  T* base = vall + ((size_t)blockIdx.x * head_dim + c) * cap;
  const int P = *dP;
  int L = *accept_len;
  if (L > GOOSE_MAX_B - 1) L = GOOSE_MAX_B - 1;
  for (int j = 1; j <= L; ++j) {
    const int src = path[j];
    if (src < j || src >= GOOSE_MAX_B || P + src >= cap) break;
    if (src != j) base[P + j] = base[P + src];
  }
}

__global__ void k_new_P(const int32_t* dP, const int32_t* accept_len, int32_t* new_P, int cap, int32_t* flags) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const int p = *dP, l = *accept_len;
    if (p < 0 || l < 0 || p + l + 1 > cap) atomicOr(flags, GOOSE_FLAG_CAPACITY);
    *new_P = p + l + 1;
  }
}

__global__ void k_new_P_batch(const ReqTable t, int cap, int32_t* flags) {  // in place: after the compaction has read the old lengths
  if (threadIdx.x == 0) {
    const BatchReq& q = t.r[blockIdx.x];
    const int p = *q.dP, l = *q.accept_len;
    if (p < 0 || l < 0 || p + l + 1 > cap) atomicOr(flags, GOOSE_FLAG_CAPACITY);
    *q.dP = p + l + 1;
  }
}

}  // namespace

// ============================================================================================
int launch_set_int(int32_t* dst, int v, hipStream_t st) {
  hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, st, dst, v);
  return goose_launch_status();
}

int launch_build_mask(const int32_t* parent, int B, const int32_t* dP, uint64_t* mask, int32_t* depth, int32_t* pos,
                      int32_t* flags, int cap, int P_max, hipStream_t st) {
  hipLaunchKernelGGL(k_build_mask, dim3(1), dim3(128), 0, st, parent, B, dP, mask, depth, pos, flags, cap, P_max);
  return goose_launch_status();
}

int launch_embed(int dtype, const void* E, const int32_t* tokens, int B, int H, int V, float* x, hipStream_t st) {
  if (dtype == GOOSE_DTYPE_BF16)
    hipLaunchKernelGGL(k_embed<bf16_t>, dim3(B), dim3(256), 0, st, (const bf16_t*)E, tokens, H, V, x);
  else if (dtype == GOOSE_DTYPE_F16)
    hipLaunchKernelGGL(k_embed<_Float16>, dim3(B), dim3(256), 0, st, (const _Float16*)E, tokens, H, V, x);
  else
    hipLaunchKernelGGL(k_embed<float>, dim3(B), dim3(256), 0, st, (const float*)E, tokens, H, V, x);
  return goose_launch_status();
}

template <typename Tg, typename T, int TERMS>
static void launch_resid_norm_t(float* x, int H, const float* part, int S, size_t part_stride, size_t part_ld,
                                const void* g, float eps, void* xn, int ldxn, int B, hipStream_t st) {
  if (H > 4 * 256)  // 1024 threads once a row has more than 1024 columns
    hipLaunchKernelGGL((k_resid_norm<Tg, T, 1024, TERMS>), dim3(B), dim3(1024), 0, st, x, H, part, S, part_stride,
                       part_ld, (const Tg*)g, eps, (T*)xn, ldxn);
  else
    hipLaunchKernelGGL((k_resid_norm<Tg, T, 256, TERMS>), dim3(B), dim3(256), 0, st, x, H, part, S, part_stride, part_ld,
                       (const Tg*)g, eps, (T*)xn, ldxn);
}

template <typename Tg, typename T>
static void launch_resid_norm_terms(int terms, float* x, int H, const float* part, int S, size_t part_stride,
                                    size_t part_ld, const void* g, float eps, void* xn, int ldxn, int B,
                                    hipStream_t st) {
  if (terms == 2) launch_resid_norm_t<Tg, T, 2>(x, H, part, S, part_stride, part_ld, g, eps, xn, ldxn, B, st);
  else launch_resid_norm_t<Tg, T, 1>(x, H, part, S, part_stride, part_ld, g, eps, xn, ldxn, B, st);
}

int launch_resid_norm(int gain_dtype, int act_dtype, float* x, int H, const float* part, int S, size_t part_stride,
                      size_t part_ld, const void* g, float eps, void* xn, int ldxn, int terms, int B, hipStream_t st) {
  if ((H & 3) || H > 16 * 1024 || (terms == 2 && (H & 7))) return GOOSE_ERR_SHAPE;
  if (terms != 1 && !(terms == 2 && act_dtype != GOOSE_DTYPE_F32)) return GOOSE_ERR_ARG;
  if (gain_dtype == GOOSE_DTYPE_BF16 && act_dtype == GOOSE_DTYPE_BF16)
    launch_resid_norm_terms<bf16_t, bf16_t>(terms, x, H, part, S, part_stride, part_ld, g, eps, xn, ldxn, B, st);
  else if (gain_dtype == GOOSE_DTYPE_BF16 && act_dtype == GOOSE_DTYPE_F16)
    launch_resid_norm_terms<bf16_t, _Float16>(terms, x, H, part, S, part_stride, part_ld, g, eps, xn, ldxn, B, st);
  else if (gain_dtype == GOOSE_DTYPE_F16 && act_dtype == GOOSE_DTYPE_F16)
    launch_resid_norm_terms<_Float16, _Float16>(terms, x, H, part, S, part_stride, part_ld, g, eps, xn, ldxn, B, st);
  else if (gain_dtype == GOOSE_DTYPE_F32 && act_dtype == GOOSE_DTYPE_F32)
    launch_resid_norm_t<float, float, 1>(x, H, part, S, part_stride, part_ld, g, eps, xn, ldxn, B, st);
  else
    return GOOSE_ERR_ARG;
  return goose_launch_status();
}

int launch_rope_kv(int dtype, const float* part, int S, size_t part_stride, size_t part_ld, int B, int n_heads,
                   int head_dim, const int32_t* pos, const double* inv_freq, const int32_t* dP, int cap, void* qout,
                   int ldq, void* kcache, void* vcache, int32_t* flags, hipStream_t st) {
  dim3 grid(B, n_heads), block(head_dim / 2);
  if (dtype == GOOSE_DTYPE_BF16)
    hipLaunchKernelGGL(k_rope_kv<bf16_t>, grid, block, 0, st, part, S, part_stride, part_ld, n_heads, head_dim, pos,
                       inv_freq, dP, cap, (bf16_t*)qout, ldq, (bf16_t*)kcache, (bf16_t*)vcache, flags);
  else
    hipLaunchKernelGGL(k_rope_kv<float>, grid, block, 0, st, part, S, part_stride, part_ld, n_heads, head_dim, pos,
                       inv_freq, dP, cap, (float*)qout, ldq, (float*)kcache, (float*)vcache, flags);
  return goose_launch_status();
}

int launch_swiglu_f32(const float* gu, size_t ld, int F, float* h, int ldh, int B, hipStream_t st) {
  hipLaunchKernelGGL(k_swiglu_f32, dim3((F + 255) / 256, B), dim3(256), 0, st, gu, ld, F, h, ldh);
  return goose_launch_status();
}

int launch_argmax(const float* logits, size_t ld, int V, int B, int32_t* argmax, float* margin, hipStream_t st) {
  hipLaunchKernelGGL(k_argmax, dim3(B), dim3(256), 0, st, logits, ld, V, argmax, margin);
  return goose_launch_status();
}

// fp32 rows -> the two-term 16-bit operand layout of the projections (groups of eight columns:
// 8 hi values T(v), then their 8 lo values T(v - hi)); columns beyond `cols` up to ld_dst/2 are zero.
template <typename T>
__global__ __launch_bounds__(256) void k_split_operand(const float* __restrict__ src, int cols, int ld_src,
                                                       T* __restrict__ dst, int ld_dst) {
  const int m = blockIdx.y, c = blockIdx.x * 256 + threadIdx.x;
  if (c >= ld_dst / 2) return;
  const float v = c < cols ? src[(size_t)m * ld_src + c] : 0.f;
  const T hi = (T)v;
  T* d = dst + (size_t)m * ld_dst + (size_t)(c >> 3) * 16 + (c & 7);
  d[0] = hi;
  d[8] = (T)(v - to_f32(hi));
}

int launch_split_operand(int dtype, const float* src, int rows, int cols, int ld_src, void* dst, int ld_dst,
                         hipStream_t st) {
  const dim3 grid((ld_dst / 2 + 255) / 256, rows);
  if (dtype == GOOSE_DTYPE_BF16)
    hipLaunchKernelGGL(k_split_operand<bf16_t>, grid, dim3(256), 0, st, src, cols, ld_src, (bf16_t*)dst, ld_dst);
  else if (dtype == GOOSE_DTYPE_F16)
    hipLaunchKernelGGL(k_split_operand<_Float16>, grid, dim3(256), 0, st, src, cols, ld_src, (_Float16*)dst, ld_dst);
  else
    return GOOSE_ERR_ARG;
  return goose_launch_status();
}

// Plain streaming copy of n 16-byte words (profiling aid: a kernel of exactly known HBM traffic).
__global__ __launch_bounds__(256) void k_copy_probe(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

int launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st) {
  hipLaunchKernelGGL(k_copy_probe, dim3(2048), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, bytes / 16);
  return goose_launch_status();
}

int launch_argmax_top2(const void* top2, int n_groups, int B, int32_t* argmax, float* margin, hipStream_t st) {
  hipLaunchKernelGGL(k_argmax_top2, dim3(B), dim3(64), 0, st, (const float4*)top2, n_groups, argmax, margin);
  return goose_launch_status();
}

int launch_harvest_topk(const float* logits, size_t ld, int V, const int32_t* tokens, int B, int K, int table_rows,
                        int32_t* succ_ids, float* succ_scores, hipStream_t st) {
  if (K < 1 || K > 16) return GOOSE_ERR_ARG;
  hipLaunchKernelGGL(k_harvest_topk<16>, dim3(B), dim3(256), 0, st, logits, ld, V, tokens, B, K, table_rows, succ_ids,
                     succ_scores);
  return goose_launch_status();
}

static ReqTable req_table(const BatchReq* reqs, int n) {
  ReqTable t{};
  for (int r = 0; r < n; ++r) t.r[r] = reqs[r];
  return t;
}

int launch_batch_begin(int dtype, const BatchReq* reqs, int n, int max_B, const void* E, int H, int V,
                       uint64_t* mask, int32_t* depth, int32_t* pos, float* x, int32_t* flags, int cap, hipStream_t st) {
  if (n < 1 || n > GOOSE_MAX_REQUESTS) return GOOSE_ERR_ARG;
  const ReqTable t = req_table(reqs, n);
  hipLaunchKernelGGL(k_build_mask_batch, dim3(n), dim3(128), 0, st, t, mask, depth, pos, flags, cap);
  int rc = goose_launch_status();
  if (rc != GOOSE_OK) return rc;
  if (dtype == GOOSE_DTYPE_BF16)
    hipLaunchKernelGGL(k_embed_batch<bf16_t>, dim3(max_B, n), dim3(256), 0, st, (const bf16_t*)E, t, H, V, x);
  else if (dtype == GOOSE_DTYPE_F16)
    hipLaunchKernelGGL(k_embed_batch<_Float16>, dim3(max_B, n), dim3(256), 0, st, (const _Float16*)E, t, H, V, x);
  else
    return GOOSE_ERR_SHAPE;
  return goose_launch_status();
}

int launch_batch_end(const BatchReq* reqs, int n, const int32_t* argmax_all, int n_layers, int n_kv_heads, int cap,
                     int head_dim, int32_t* flags, hipStream_t st) {
  if (n < 1 || n > GOOSE_MAX_REQUESTS) return GOOSE_ERR_ARG;
  const ReqTable t = req_table(reqs, n);
  hipLaunchKernelGGL(k_accept_batch, dim3(n), dim3(128), 0, st, t, argmax_all);
  int rc = goose_launch_status();
  if (rc != GOOSE_OK) return rc;
  if (head_dim == 128)
    hipLaunchKernelGGL(k_compact_tiled_batch<128>, dim3(n_layers * n_kv_heads, n), dim3(128), 0, st, t, cap);
  else if (head_dim == 64)
    hipLaunchKernelGGL(k_compact_tiled_batch<64>, dim3(n_layers * n_kv_heads, n), dim3(64), 0, st, t, cap);
  else
    return GOOSE_ERR_SHAPE;
  rc = goose_launch_status();
  if (rc != GOOSE_OK) return rc;
  hipLaunchKernelGGL(k_new_P_batch, dim3(n), dim3(64), 0, st, t, cap, flags);
  return goose_launch_status();
}

int launch_accept(const int32_t* parent, const int32_t* tokens, const uint8_t* is_spine, const int32_t* argmax, int B,
                  int32_t* accept_len, int32_t* path, int32_t* bonus, int32_t* next_root, hipStream_t st) {
  hipLaunchKernelGGL(k_accept, dim3(1), dim3(128), 0, st, parent, tokens, is_spine, argmax, B, accept_len, path,
                     bonus, next_root);
  return goose_launch_status();
}

int launch_compact(int elem_bytes, void* kall, void* vall, int n_layers, int n_heads, int cap, int head_dim,
                   const int32_t* dP, const int32_t* path, const int32_t* accept_len, int32_t* new_P,
                   int32_t* flags, hipStream_t st) {
  int rc;
  if (elem_bytes == 2) {  // bf16 / fp16 (moved as bit patterns): operand-ordered blocks
    if (head_dim == 128)
      hipLaunchKernelGGL(k_compact_tiled<128>, dim3(n_layers * n_heads), dim3(128), 0, st, (bf16_t*)kall, (bf16_t*)vall,
                         cap, dP, path, accept_len);
    else if (head_dim == 64)
      hipLaunchKernelGGL(k_compact_tiled<64>, dim3(n_layers * n_heads), dim3(64), 0, st, (bf16_t*)kall, (bf16_t*)vall,
                         cap, dP, path, accept_len);
    else
      return GOOSE_ERR_SHAPE;
    rc = goose_launch_status();
  } else {  // fp32: K[head][slot][d], Vt[head][d][slot]
    const int row_chunks = head_dim * elem_bytes / 16;  // <= 64 for head_dim <= 256
    hipLaunchKernelGGL(k_compact_k, dim3(n_layers * n_heads), dim3(64), 0, st, (uint4*)kall, cap, row_chunks, dP, path,
                       accept_len);
    rc = goose_launch_status();
    if (rc != GOOSE_OK) return rc;
    hipLaunchKernelGGL(k_compact_vt<float>, dim3(n_layers * n_heads), dim3(head_dim), 0, st, (float*)vall, cap,
                       head_dim, dP, path, accept_len);
    rc = goose_launch_status();
  }
  if (rc != GOOSE_OK) return rc;
  if (new_P) {
    hipLaunchKernelGGL(k_new_P, dim3(1), dim3(1), 0, st, dP, accept_len, new_P, cap, flags);
    rc = goose_launch_status();
  }
  return rc;
}
