// Plain fp32 kernels for models stored in fp32 (small models; correctness path, not tuned).
#include "goose_internal.h"

namespace {

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// out[m][n] = sum_k A[m][k] * W[n][k].  One wavefront per (n, group of 8 rows): lanes stride
// over k so that the weight row is read coalesced, then the 8 sums are reduced across lanes.
__global__ __launch_bounds__(64) void k_gemm_f32(const float* __restrict__ A, int lda, const float* __restrict__ W,
                                                 int K, int M, float* __restrict__ out, size_t ldo) {
  const int n = blockIdx.x, m0 = blockIdx.y * 8, lane = threadIdx.x;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const float* w = W + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float wv = w[k];
#pragma unroll
    for (int r = 0; r < 8; ++r)
      if (m0 + r < M) acc[r] += A[(size_t)(m0 + r) * lda + k] * wv;
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const float s = wave_sum(acc[r]);
    if (lane == 0 && m0 + r < M) out[(size_t)(m0 + r) * ldo + n] = s;
  }
}

// Tree-masked attention for one (query node, head): scores over slots [0,P) and the
// ancestor-or-self slots of the tail, softmax in fp32, weighted sum of V.
__global__ __launch_bounds__(64) void k_attn_f32(const float* __restrict__ q, int ldq, const float* __restrict__ kc,
                                                 const float* __restrict__ vc, int head_dim, int cap,
                                                 const int32_t* __restrict__ dP, int B,
                                                 const uint64_t* __restrict__ mask, float* __restrict__ o, int ldo,
                                                 int lds_keys, int32_t* __restrict__ flags) {
  extern __shared__ float sm[];
  float* sq = sm;             // [head_dim]
  float* sc = sm + head_dim;  // [lds_keys]
  const int i = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int W = (B + 63) >> 6;
  const int P = *dP;
  int nk = P + B;
  // the launch is sized from the host's upper bound of P: a longer cache is flagged
  // (GOOSE_FLAG_CAPACITY) and the keys beyond the bound are dropped so that nothing is indexed outside LDS
  if ((P < 0 || nk > lds_keys || nk > cap) && i == 0 && h == 0 && lane == 0) atomicOr(flags, GOOSE_FLAG_CAPACITY);
  if (nk > lds_keys) nk = lds_keys;
  if (nk > cap) nk = cap;
  if (nk < 0) nk = 0;
  for (int c = lane; c < head_dim; c += 64) sq[c] = q[(size_t)i * ldq + h * head_dim + c];
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)head_dim);
  const float* kh = kc + (size_t)h * cap * head_dim;
  const float* vh = vc + (size_t)h * head_dim * cap;  // transposed value cache Vt[head][d][slot]
  float mx = -INFINITY;
  for (int s = lane; s < nk; s += 64) {
    bool vis = s < P;
    if (!vis) {
      const int j = s - P;
      vis = (mask[(size_t)i * W + (j >> 6)] >> (j & 63)) & 1ull;
    }
    float d = -INFINITY;
    if (vis) {
      d = 0.f;
      const float* kr = kh + (size_t)s * head_dim;
      for (int c = 0; c < head_dim; ++c) d += sq[c] * kr[c];
      d *= scale;
    }
    sc[s] = d;
    mx = fmaxf(mx, d);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int s = lane; s < nk; s += 64) {
    const float d = sc[s];
    const float p = (d == -INFINITY) ? 0.f : expf(d - mx);
    sc[s] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  __syncthreads();
  for (int c = lane; c < head_dim; c += 64) {
    float acc = 0.f;
    for (int s = 0; s < nk; ++s) {
      const float p = sc[s];
      if (p != 0.f) acc += p * vh[(size_t)c * cap + s];
    }
    o[(size_t)i * ldo + h * head_dim + c] = acc / sum;
  }
}

}  // namespace

int launch_gemm_f32(const float* A, int lda, const float* W, int N, int K, int M, float* out, size_t ldo,
                    hipStream_t st) {
  hipLaunchKernelGGL(k_gemm_f32, dim3(N, (M + 7) / 8), dim3(64), 0, st, A, lda, W, K, M, out, ldo);
  return goose_launch_status();
}

int launch_attn_f32(const float* q, int ldq, const float* kc, const float* vc, int n_heads, int head_dim, int cap,
                    const int32_t* dP, int B, const uint64_t* mask, float* o, int ldo, int P_max, int32_t* flags,
                    hipStream_t st) {
  const int lds_keys = P_max + B;
  const size_t smem = (size_t)(head_dim + lds_keys) * sizeof(float);
  if (smem > 64 * 1024) return GOOSE_ERR_CAPACITY;  // the fp32 path keeps all scores of a row in LDS
  hipLaunchKernelGGL(k_attn_f32, dim3(B, n_heads), dim3(64), smem, st, q, ldq, kc, vc, head_dim, cap, dP, B, mask, o,
                     ldo, lds_keys, flags);
  return goose_launch_status();
}
