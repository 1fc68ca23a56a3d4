// Tree-masked attention of the B draft-node queries over the cached prefix plus their own
// ancestors (Sec. 4, tree attention mask), bf16 operands, fp32 softmax, for gfx950.
//
// All B queries of a head share the same keys, so the B nodes are the N dimension of an MFMA
// and every K/V byte fetched from HBM is used B times.  Cache layout: K[head][slot][d] and
// V TRANSPOSED, Vt[head][d][slot], so that both MFMA operands are 16 contiguous bytes per lane.
// Work decomposition:
//   grid = (key splits, heads); a workgroup has one wavefront per 32-query tile.
//   The workgroup stages 64-key tiles of K and Vt in LDS (double buffered: the next tile is
//   on its way global -> registers while the current one is multiplied).
//   Per 32-key sub-tile a wavefront computes
//     S^T[key][query]  = K . Q^T          (v_mfma_f32_32x32x16_bf16, rows = keys)
//     online softmax over keys: in this layout each lane owns ONE query (column l%32) and 16
//     keys, so the running max / sum / rescale are per-lane scalars plus one exchange with the
//     twin lane l^32;
//     O^T[d][query]   += Vt . P^T         (rows = head-dim, columns = the same queries).
//   The MFMA row <-> key assignment is chosen so that the 16 scores a lane holds are 16
//   consecutive keys: the probabilities feed the second MFMA straight from registers.
// Splits write (max, sum, unnormalised O) partials; k_attn_merge combines them in fixed order.
#include <type_traits>

#include "goose_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

constexpr int TK = 64;             // keys per staged tile
constexpr float NEG_BIG = -1e30f;  // finite stand-in for -inf: keeps exp2(m_old - m_new) well defined

template <int D, int QT>
__global__ __launch_bounds__(64 * QT) void k_attn_bf16(const bf16_t* __restrict__ q, int ldq,
                                                       const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vt,
                                                       int cap, const int32_t* __restrict__ dP, int B,
                                                       const uint64_t* __restrict__ mask, float* __restrict__ att_o,
                                                       float* __restrict__ att_ml, int Bpad) {
  constexpr int NTHR = 64 * QT;
  constexpr int KROW = D * 2 + 16;       // bytes per staged K row
  constexpr int VROW = TK * 2 + 16;      // bytes per staged Vt row
  constexpr int KCH = TK * (D / 8);      // 16-byte chunks of a K tile
  constexpr int VCH = D * (TK / 8);      // 16-byte chunks of a Vt tile
  constexpr int KPT = KCH / NTHR, VPT = VCH / NTHR;
  static_assert(KCH % NTHR == 0 && VCH % NTHR == 0, "tile must divide over the workgroup");
  constexpr int KBYTES = TK * KROW, VBYTES = D * VROW;
  __shared__ __attribute__((aligned(16))) unsigned char Ks[2][KBYTES];
  __shared__ __attribute__((aligned(16))) unsigned char Vs[2][VBYTES];

  const int tid = threadIdx.x, lane = tid & 63, qt = tid >> 6;
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
  const bf16_t* vh = vt + (size_t)h * D * cap;

  // Tile copy global -> registers -> LDS.  Every load is issued unconditionally (a chunk past
  // the end of the split re-reads the split's first keys, always in bounds) so that all 16 loads
  // of a thread are in flight together; keys at or beyond k_end are zeroed on the way into LDS.
  u32x4 kreg[KPT], vreg[VPT];
  auto load_tile = [&](int key0) {
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const int ch = tid + NTHR * i;
      const int row = ch / (D / 8), c = ch % (D / 8);
      const int key = (key0 + row < k_end) ? key0 + row : k_begin;
      kreg[i] = *reinterpret_cast<const u32x4*>(kh + (size_t)key * D + c * 8);
    }
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int ch = tid + NTHR * i;
      const int row = ch / (TK / 8), c = ch % (TK / 8);
      const int key = (key0 + c * 8 < k_end) ? key0 + c * 8 : k_begin;
      vreg[i] = *reinterpret_cast<const u32x4*>(vh + (size_t)row * cap + key);
    }
  };
  auto store_tile = [&](int buf, int key0) {
    const bool ragged = key0 + TK > k_end;  // only the last tile of a split
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const int ch = tid + NTHR * i;
      const int row = ch / (D / 8), c = ch % (D / 8);
      u32x4 v = kreg[i];
      if (ragged && key0 + row >= k_end) v = u32x4{0, 0, 0, 0};
      *reinterpret_cast<u32x4*>(&Ks[buf][row * KROW + c * 16]) = v;
    }
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int ch = tid + NTHR * i;
      const int row = ch / (TK / 8), c = ch % (TK / 8);
      u32x4 v = vreg[i];
      if (ragged) {
        const int key = key0 + c * 8;
        u16x8 e = __builtin_bit_cast(u16x8, v);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (key + j >= k_end) e[j] = 0;
        v = __builtin_bit_cast(u32x4, e);
      }
      *reinterpret_cast<u32x4*>(&Vs[buf][row * VROW + c * 16]) = v;
    }
  };

  auto compute_tile = [&](auto buf_c, int key0) {
    constexpr int buf = decltype(buf_c)::value;
#pragma unroll
    for (int sub = 0; sub < TK / 32; ++sub) {
      const int kb = key0 + sub * 32;
      if (kb >= k_end) break;
      f32x16 sacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[buf][(sub * 32 + sigma) * KROW + s * 32 + hh * 16]);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], sacc, 0, 0, 0);
      }
      // scores -> probabilities.  Sub-tiles that lie wholly inside the prefix need no mask at all
      // (wave-uniform test); only the few tail sub-tiles take the masked path.
      const int kfirst = kb + hh * 16;  // this lane's 16 keys are kfirst .. kfirst+15
      float tmax = NEG_BIG;
      unsigned vis = 0xFFFFu;
      const bool masked = kb + 32 > P;
      if (!masked) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          sacc[r] *= scale;
          tmax = fmaxf(tmax, sacc[r]);
        }
      } else {
        // 16 visibility bits: keys below P are visible, key P+j is visible iff bit j of the ancestor row
        const int j0 = kfirst - P;
        if (j0 >= 0) {
          const uint64_t lo = j0 < 64 ? (mw0 >> j0) | (j0 ? mw1 << (64 - j0) : 0ull) : (j0 < 128 ? mw1 >> (j0 - 64) : 0ull);
          vis = (unsigned)lo & 0xFFFFu;
        } else if (j0 > -16) {
          const int np = -j0;  // 1..15 prefix keys first
          vis = (((1u << np) - 1u) | ((unsigned)mw0 << np)) & 0xFFFFu;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          sacc[r] = ((vis >> r) & 1u) ? sacc[r] * scale : NEG_BIG;
          tmax = fmaxf(tmax, sacc[r]);
        }
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      const bool grew = m_new > m_run;
      m_run = m_new;
      float psum = 0.f;
      bf16x8 pf[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(sacc[r] - m_new);
        if (masked) p = ((vis >> r) & 1u) ? p : 0.f;  // a fully masked row has m_new == NEG_BIG: exp2(0) must not count
        psum += p;
        pf[r >> 3][r & 7] = (__bf16)p;
      }
      l_run = l_run * alpha + psum;
      // the running maximum settles after a few tiles: skip the rescale of O when no lane's maximum grew
      if (__builtin_amdgcn_ballot_w64(grew) != 0) {
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
      }
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(
              &Vs[buf][(dt * 32 + l31) * VROW + (sub * 32 + hh * 16 + j * 8) * 2]);
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[j], oacc[dt], 0, 0, 0);
        }
      }
    }
  };
  const std::integral_constant<int, 0> b0;
  const std::integral_constant<int, 1> b1;

  const int ntiles = (k_end - k_begin + TK - 1) / TK;
  if (ntiles > 0) {
    load_tile(k_begin);
    store_tile(0, k_begin);
    __syncthreads();
    for (int t = 0; t < ntiles; t += 2) {
      const int key0 = k_begin + t * TK;
      const bool more1 = (t + 1) < ntiles;
      if (more1) load_tile(key0 + TK);
      compute_tile(b0, key0);
      if (more1) store_tile(1, key0 + TK);
      __syncthreads();
      if (!more1) break;
      const bool more2 = (t + 2) < ntiles;
      if (more2) load_tile(key0 + 2 * TK);
      compute_tile(b1, key0 + TK);
      if (more2) store_tile(0, key0 + 2 * TK);
      __syncthreads();
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

template <int D>
int launch_qt(int QT, dim3 grid, hipStream_t st, const bf16_t* q, int ldq, const bf16_t* kc, const bf16_t* vt, int cap,
              const int32_t* dP, int B, const uint64_t* mask, float* att_o, float* att_ml, int Bpad) {
  switch (QT) {
    case 1: hipLaunchKernelGGL((k_attn_bf16<D, 1>), grid, dim3(64), 0, st, q, ldq, kc, vt, cap, dP, B, mask, att_o, att_ml, Bpad); break;
    case 2: hipLaunchKernelGGL((k_attn_bf16<D, 2>), grid, dim3(128), 0, st, q, ldq, kc, vt, cap, dP, B, mask, att_o, att_ml, Bpad); break;
    case 3: hipLaunchKernelGGL((k_attn_bf16<D, 4>), grid, dim3(256), 0, st, q, ldq, kc, vt, cap, dP, B, mask, att_o, att_ml, Bpad); break;
    case 4: hipLaunchKernelGGL((k_attn_bf16<D, 4>), grid, dim3(256), 0, st, q, ldq, kc, vt, cap, dP, B, mask, att_o, att_ml, Bpad); break;
    default: return GOOSE_ERR_ARG;
  }
  return goose_launch_status();
}

}  // namespace

// Key splits per head: at least two 64-key tiles per workgroup, about one workgroup per compute
// unit (two for long prefixes).
int pick_attn_splits(int n_heads, int keys_max, int max_splits) {
  // one workgroup per CU (256) measured faster than more, shorter splits: a split of one tile has
  // nothing to overlap its loads with, and every split adds a partial result to merge
  const int tiles = (keys_max + TK - 1) / TK;
  int s = (tiles + 1) / 2;
  const int want = ((tiles > 64 ? 512 : 256) + n_heads - 1) / n_heads;
  if (s > want) s = want;
  if (s > max_splits) s = max_splits;
  if (s < 1) s = 1;
  return s;
}

int launch_attn_bf16(const void* q, int ldq, const void* kc, const void* vt, int n_heads, int head_dim, int cap,
                     const int32_t* dP, int B, const uint64_t* mask, int splits, float* att_o, float* att_ml,
                     int Bpad, void* o, int ldo, hipStream_t st) {
  const int QT = (B + 31) / 32;
  // a 3-tile tree runs the 4-wavefront kernel, which reads query rows up to 128 (the workspace has them)
  if ((QT == 3 ? 4 : QT) * 32 > Bpad) return GOOSE_ERR_ARG;
  dim3 grid(splits, n_heads);
  int rc;
  if (head_dim == 128)
    rc = launch_qt<128>(QT, grid, st, (const bf16_t*)q, ldq, (const bf16_t*)kc, (const bf16_t*)vt, cap, dP, B, mask,
                        att_o, att_ml, Bpad);
  else if (head_dim == 64)
    rc = launch_qt<64>(QT, grid, st, (const bf16_t*)q, ldq, (const bf16_t*)kc, (const bf16_t*)vt, cap, dP, B, mask,
                       att_o, att_ml, Bpad);
  else
    return GOOSE_ERR_SHAPE;
  if (rc != GOOSE_OK) return rc;
  hipLaunchKernelGGL(k_attn_merge, dim3(B, n_heads), dim3(head_dim), 0, st, att_o, att_ml, splits, Bpad, head_dim,
                     (bf16_t*)o, ldo);
  return goose_launch_status();
}
