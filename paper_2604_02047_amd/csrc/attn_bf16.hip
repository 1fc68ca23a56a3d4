// Tree-masked attention of the B draft-node queries over the cached prefix plus their own
// ancestors (Sec. 4, tree attention mask), bf16 operands, fp32 softmax, for gfx950.
//
// All B queries of a head share the same keys, so the B nodes are the N dimension of an MFMA
// and every K/V byte fetched from HBM is used B times.  Work decomposition:
//   grid = (key splits, heads); a workgroup has one wavefront per 32-query tile.
//   The workgroup stages 64-key tiles in LDS: K as is, V transposed (so that both MFMA
//   operands read 16 contiguous bytes per lane).  Per 32-key sub-tile a wavefront computes
//     S^T[key][query]  = K . Q^T          (v_mfma_f32_32x32x16_bf16, rows = keys)
//     online softmax over keys: in this layout each lane owns ONE query (column l%32) and 16
//     keys, so the running max / sum / rescale are per-lane scalars plus one exchange with the
//     twin lane l^32;
//     O^T[d][query]   += V^T . P^T        (rows = head-dim, columns = the same queries).
//   The MFMA row <-> key assignment is chosen so that the 16 scores a lane holds are 16
//   consecutive keys: the probabilities feed the second MFMA straight from registers.
// Splits write (max, sum, unnormalised O) partials; k_attn_merge combines them in fixed order.
#include "goose_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int TK = 64;            // keys per staged tile
constexpr float NEG_BIG = -1e30f;  // finite stand-in for -inf: keeps exp2(m_old - m_new) well defined

template <int D>
__global__ __launch_bounds__(256) void k_attn_bf16(const bf16_t* __restrict__ q, int ldq,
                                                   const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc,
                                                   int cap, const int32_t* __restrict__ dP, int B,
                                                   const uint64_t* __restrict__ mask, float* __restrict__ att_o,
                                                   float* __restrict__ att_ml, int Bpad) {
  constexpr int KROW = D * 2 + 16;   // bytes per staged K row
  constexpr int VROW = TK * 2 + 16;  // bytes per staged V^T row
  constexpr int DCH = D / 8;         // 16-byte chunks per cache row
  __shared__ __attribute__((aligned(16))) unsigned char Ks[TK * KROW];
  __shared__ __attribute__((aligned(16))) unsigned char Vt[D * VROW];

  const int tid = threadIdx.x, lane = tid & 63, qt = tid >> 6, nthr = blockDim.x;
  const int split = blockIdx.x, nsplit = gridDim.x, h = blockIdx.y;
  const int P = *dP;
  int Ktot = P + B;
  if (Ktot > cap) Ktot = cap;
  // 32-key units dealt evenly to the splits
  const int units = (Ktot + 31) >> 5;
  const int k_begin = (int)(((long)units * split) / nsplit) << 5;
  int k_end = (int)(((long)units * (split + 1)) / nsplit) << 5;
  if (k_end > Ktot) k_end = Ktot;

  const int l31 = lane & 31, hh = lane >> 5;
  const int qi = qt * 32 + l31;
  // row i = l31 of the first MFMA carries key sigma(i) so that register r of lane (q, hh) is key hh*16 + r
  const int sigma = ((l31 >> 2) & 1) * 16 + (l31 & 3) + 4 * (l31 >> 3);

  bf16x8 qf[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qf[s] = *reinterpret_cast<const bf16x8*>(q + (size_t)qi * ldq + h * D + s * 16 + hh * 8);

  const int W = (B + 63) >> 6;
  uint64_t mw0 = 0, mw1 = 0;
  if (qi < B) {
    mw0 = mask[(size_t)qi * W];
    if (W > 1) mw1 = mask[(size_t)qi * W + 1];
  }

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m_run = NEG_BIG, l_run = 0.f;
  const float scale = 1.4426950408889634f / sqrtf((float)D);  // log2(e) / sqrt(d): softmax in base 2

  const bf16_t* kh = kc + (size_t)h * cap * D;
  const bf16_t* vh = vc + (size_t)h * cap * D;

  for (int key0 = k_begin; key0 < k_end; key0 += TK) {
    __syncthreads();  // previous tile fully consumed
    for (int ch = tid; ch < TK * DCH; ch += nthr) {
      const int row = ch / DCH, c = ch % DCH;
      const int key = key0 + row;
      u32x4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
      if (key < k_end) {
        kv = *reinterpret_cast<const u32x4*>(kh + (size_t)key * D + c * 8);
        vv = *reinterpret_cast<const u32x4*>(vh + (size_t)key * D + c * 8);
      }
      *reinterpret_cast<u32x4*>(&Ks[row * KROW + c * 16]) = kv;
      const unsigned short* ve = reinterpret_cast<const unsigned short*>(&vv);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        *reinterpret_cast<unsigned short*>(&Vt[(c * 8 + e) * VROW + row * 2]) = ve[e];
    }
    __syncthreads();

#pragma unroll
    for (int sub = 0; sub < TK / 32; ++sub) {
      const int kb = key0 + sub * 32;
      if (kb >= k_end) break;
      f32x16 sacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[(sub * 32 + sigma) * KROW + s * 32 + hh * 16]);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], sacc, 0, 0, 0);
      }
      // visibility of this lane's 16 keys kb + hh*16 + r for its query
      const int kfirst = kb + hh * 16;
      unsigned vis;
      if (kfirst + 16 <= P) {
        vis = 0xFFFFu;
      } else {
        vis = 0;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kfirst + r;
          bool v = key < P;
          if (!v && key < k_end) {
            const int j = key - P;
            v = ((j < 64 ? mw0 >> j : mw1 >> (j - 64)) & 1ull) != 0;
          }
          vis |= (v ? 1u : 0u) << r;
        }
      }
      float tmax = NEG_BIG;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        sacc[r] = ((vis >> r) & 1u) ? sacc[r] * scale : NEG_BIG;
        tmax = fmaxf(tmax, sacc[r]);
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = exp2f(m_run - m_new);
      m_run = m_new;
      float psum = 0.f;
      bf16x8 pf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = ((vis >> r) & 1u) ? exp2f(sacc[r] - m_new) : 0.f;
        psum += p;
        pf[r >> 3][r & 7] = (__bf16)p;
      }
      l_run = l_run * alpha + psum;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 a =
              *reinterpret_cast<const bf16x8*>(&Vt[(dt * 32 + l31) * VROW + (sub * 32 + hh * 16 + j * 8) * 2]);
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[j], oacc[dt], 0, 0, 0);
        }
      }
    }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < B) {
    const size_t base = ((size_t)h * nsplit + split) * Bpad + qi;
    if (hh == 0) {
      att_ml[base * 2] = m_run;
      att_ml[base * 2 + 1] = l_tot;
    }
    float* orow = att_o + base * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        f32x4 v = {oacc[dt][a * 4], oacc[dt][a * 4 + 1], oacc[dt][a * 4 + 2], oacc[dt][a * 4 + 3]};
        *reinterpret_cast<f32x4*>(orow + dt * 32 + a * 8 + hh * 4) = v;
      }
  }
}

// o[q][h*D + c] = sum_s 2^(m_s - m) O_s[c] / sum_s 2^(m_s - m) l_s, splits taken in index order.
__global__ void k_attn_merge(const float* __restrict__ att_o, const float* __restrict__ att_ml, int nsplit, int Bpad,
                             int D, bf16_t* __restrict__ o, int ldo) {
  const int qi = blockIdx.x, h = blockIdx.y, c = threadIdx.x;
  float mmax = NEG_BIG;
  for (int s = 0; s < nsplit; ++s) mmax = fmaxf(mmax, att_ml[(((size_t)h * nsplit + s) * Bpad + qi) * 2]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const size_t base = ((size_t)h * nsplit + s) * Bpad + qi;
    const float w = exp2f(att_ml[base * 2] - mmax);
    den += w * att_ml[base * 2 + 1];
    num += w * att_o[base * D + c];
  }
  o[(size_t)qi * ldo + h * D + c] = (bf16_t)(num / den);
}

}  // namespace

// Key splits: enough workgroups for the 256 compute units, each split at least 128 keys.
int pick_attn_splits(int n_heads, int keys_max, int max_splits) {
  int s = (256 + n_heads - 1) / n_heads;
  const int by_keys = (keys_max + 127) / 128;
  if (s > by_keys) s = by_keys;
  if (s > max_splits) s = max_splits;
  if (s < 1) s = 1;
  return s;
}

int launch_attn_bf16(const void* q, int ldq, const void* kc, const void* vc, int n_heads, int head_dim, int cap,
                     const int32_t* dP, int B, const uint64_t* mask, int splits, float* att_o, float* att_ml,
                     int Bpad, void* o, int ldo, hipStream_t st) {
  const int QT = (B + 31) / 32;
  dim3 grid(splits, n_heads), block(64 * QT);
  if (head_dim == 128)
    hipLaunchKernelGGL(k_attn_bf16<128>, grid, block, 0, st, (const bf16_t*)q, ldq, (const bf16_t*)kc,
                       (const bf16_t*)vc, cap, dP, B, mask, att_o, att_ml, Bpad);
  else if (head_dim == 64)
    hipLaunchKernelGGL(k_attn_bf16<64>, grid, block, 0, st, (const bf16_t*)q, ldq, (const bf16_t*)kc,
                       (const bf16_t*)vc, cap, dP, B, mask, att_o, att_ml, Bpad);
  else
    return GOOSE_ERR_SHAPE;
  int rc = goose_launch_status();
  if (rc != GOOSE_OK) return rc;
  hipLaunchKernelGGL(k_attn_merge, dim3(B, n_heads), dim3(head_dim), 0, st, att_o, att_ml, splits, Bpad, head_dim,
                     (bf16_t*)o, ldo);
  return goose_launch_status();
}
