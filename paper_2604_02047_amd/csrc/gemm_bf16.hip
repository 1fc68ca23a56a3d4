// Skinny-M bf16 GEMM for gfx950: out[m][n] = sum_k A[m][k] * W[n][k], M = tree nodes (<= 128).
//
// The pass is weight-bandwidth bound (every weight byte is used for only M multiply-adds), so
// the kernel is organised around streaming W once, with wide fully-coalesced loads:
//   * W is pre-tiled (launch_pack_bf16) into MFMA-operand order: tile (nt, kt) = 32 output
//     rows x 16 inputs = 1 KiB, lane l of a wavefront owning W[nt*32 + l%32][kt*16 + 8*(l/32) .. +7].
//     One global_load_dwordx4 per lane fetches a whole operand of v_mfma_f32_32x32x16_bf16 and
//     consecutive kt are consecutive in memory, so each wavefront reads one long contiguous run.
//   * The M x K activation block is small and shared: the workgroup stages 64-wide K chunks of it
//     in LDS (double buffered) and every wavefront reads its A operands from there.
//   * 4 wavefronts per workgroup, each owning NT column tiles; split-K over blockIdx.y writes
//     fp32 partials that the next (reduction / rotary / norm) kernel sums in a fixed order.
#include "goose_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int KC = 64;               // k extent of one LDS chunk
constexpr int LDS_ROW = KC * 2 + 16;  // bytes; the 16-byte pad staggers rows across banks

// ------------------------------------------------------------------------------------------
// Re-tile raw row-major bf16 matrices.  Packed row n comes from
//   PACK_PLAIN   : s0 row n
//   PACK_QKV     : q|k|v stacked: source n / rows_each, row n % rows_each
//   PACK_GATE_UP : blocks of 32 rows alternate gate (s0) / up (s1): block b -> (b&1 ? up : gate) rows (b>>1)*32..
// Rows and columns outside the source are zero.
__global__ __launch_bounds__(256) void k_pack_bf16(int mode, const bf16_t* __restrict__ s0,
                                                   const bf16_t* __restrict__ s1, const bf16_t* __restrict__ s2,
                                                   int rows_each, int K, int ktiles, size_t total,
                                                   uint4* __restrict__ dst) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // one 16-byte lane slot
  if (idx >= total) return;
  const int lane = idx & 63;
  const size_t tile = idx >> 6;
  const int kt = tile % ktiles;
  const int nt = tile / ktiles;
  const int n = nt * 32 + (lane & 31);
  const int k0 = kt * 16 + (lane >> 5) * 8;
  const bf16_t* src = nullptr;
  int row = 0;
  if (mode == PACK_PLAIN) {
    src = s0; row = n;
  } else if (mode == PACK_QKV) {
    const int which = n / rows_each;
    row = n % rows_each;
    src = which == 0 ? s0 : (which == 1 ? s1 : (which == 2 ? s2 : nullptr));
  } else {
    const int blk = n >> 5;
    row = (blk >> 1) * 32 + (n & 31);
    src = (blk & 1) ? s1 : s0;
  }
  union { uint4 u; bf16_t e[8]; } v;
  v.u = make_uint4(0, 0, 0, 0);
  if (src != nullptr && row < rows_each) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (k0 + e < K) v.e[e] = src[(size_t)row * K + k0 + e];
  }
  dst[idx] = v.u;
}

// ------------------------------------------------------------------------------------------
template <int MT, int NT, int EPI>
__global__ __launch_bounds__(256) void k_gemm_bf16(const bf16_t* __restrict__ A, int lda,
                                                   const u32x4* __restrict__ Wp, int ntiles, int ksteps_total,
                                                   int chunks_per_split, int B, void* __restrict__ out, size_t ldo,
                                                   size_t split_stride) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][MT * 32 * LDS_ROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tile0 = (blockIdx.x * 4 + wave) * NT;
  const int nchunks_total = ksteps_total >> 2;
  const int c_begin = blockIdx.y * chunks_per_split;
  const int c_end = min(c_begin + chunks_per_split, nchunks_total);
  const int nch = c_end - c_begin;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][t][r] = 0.f;

  bool active[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) active[t] = (tile0 + t) < ntiles;

  // per-thread slots of the cooperative A-chunk copy: MT*32 rows x 8 sixteen-byte segments
  u32x4 areg[MT];
  auto load_a = [&](int c) {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int seg = tid + 256 * i;
      const int row = seg >> 3, c16 = seg & 7;
      areg[i] = *reinterpret_cast<const u32x4*>(A + (size_t)row * lda + (size_t)c * KC + c16 * 8);
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int seg = tid + 256 * i;
      const int row = seg >> 3, c16 = seg & 7;
      *reinterpret_cast<u32x4*>(&lds[buf][row * LDS_ROW + c16 * 16]) = areg[i];
    }
  };
  u32x4 wreg[2][NT][4];
  auto load_w = [&](int c, int slot) {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (active[t]) {
        const u32x4* p = Wp + ((size_t)(tile0 + t) * ksteps_total + (size_t)c * 4) * 64 + lane;
#pragma unroll
        for (int s = 0; s < 4; ++s) wreg[slot][t][s] = __builtin_nontemporal_load(p + s * 64);
      }
    }
  };
  auto compute = [&](int buf, int slot) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 a[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 32 + (lane & 31);
        a[mt] = *reinterpret_cast<const bf16x8*>(&lds[buf][row * LDS_ROW + s * 32 + (lane >> 5) * 16]);
      }
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        if (active[t]) {
          const bf16x8 b = __builtin_bit_cast(bf16x8, wreg[slot][t][s]);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[mt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b, acc[mt][t], 0, 0, 0);
        }
      }
    }
  };

  if (nch > 0) {
    load_a(c_begin);
    load_w(c_begin, 0);
    store_a(0);
    __syncthreads();
    for (int i = 0; i < nch; i += 2) {
      // even step: compute from (lds 0, wreg 0) while chunk i+1 streams into (lds 1, wreg 1)
      const bool more1 = (i + 1) < nch;
      if (more1) { load_a(c_begin + i + 1); load_w(c_begin + i + 1, 1); }
      compute(0, 0);
      if (more1) store_a(1);
      __syncthreads();
      if (!more1) break;
      const bool more2 = (i + 2) < nch;
      if (more2) { load_a(c_begin + i + 2); load_w(c_begin + i + 2, 0); }
      compute(1, 1);
      if (more2) store_a(0);
      __syncthreads();
    }
  }

  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  if (EPI == EPI_PARTIAL) {
    float* o = reinterpret_cast<float*>(out) + blockIdx.y * split_stride;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (!active[t]) continue;
      const int col = (tile0 + t) * 32 + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < B) o[(size_t)row * ldo + col] = acc[mt][t][r];
        }
    }
  } else {  // EPI_SWIGLU: tile pair (gate, up) -> h = silu(gate) * up
    static_assert(EPI != EPI_SWIGLU || NT == 2, "SwiGLU epilogue needs the gate and up tiles in one wavefront");
    if (active[0] && active[NT - 1]) {
      bf16_t* hq = reinterpret_cast<bf16_t*>(out);
      const int col = (tile0 >> 1) * 32 + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const float g = acc[mt][0][r], u = acc[mt][NT - 1][r];
          if (row < B) hq[(size_t)row * ldo + col] = (bf16_t)(g / (1.0f + __expf(-g)) * u);
        }
    }
  }
}

template <int MT, int NT, int EPI>
int launch_one(const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit, void* out, size_t ldo,
               size_t split_stride, hipStream_t st) {
  const int ntiles = Npad / 32, ksteps = Kpad / 16, nchunks = ksteps / 4;
  const int cps = (nchunks + ksplit - 1) / ksplit;
  dim3 grid((ntiles + 4 * NT - 1) / (4 * NT), ksplit);
  hipLaunchKernelGGL((k_gemm_bf16<MT, NT, EPI>), grid, dim3(256), 0, st, (const bf16_t*)A, lda, (const u32x4*)Wp,
                     ntiles, ksteps, cps, B, out, ldo, split_stride);
  return goose_launch_status();
}

template <int NT, int EPI>
int launch_mt(int MT, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit, void* out,
              size_t ldo, size_t split_stride, hipStream_t st) {
  switch (MT) {
    case 1: return launch_one<1, NT, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, st);
    case 2: return launch_one<2, NT, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, st);
    case 3: return launch_one<3, NT, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, st);
    case 4: return launch_one<4, NT, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, st);
  }
  return GOOSE_ERR_ARG;
}

}  // namespace

int launch_pack_bf16(int mode, const void* s0, const void* s1, const void* s2, int rows_each, int K, int Npad,
                     int Kpad, void* dst, hipStream_t st) {
  const size_t total = (size_t)(Npad / 32) * (Kpad / 16) * 64;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(k_pack_bf16, dim3(blocks), dim3(256), 0, st, mode, (const bf16_t*)s0, (const bf16_t*)s1,
                     (const bf16_t*)s2, rows_each, K, Kpad / 16, total, (uint4*)dst);
  return goose_launch_status();
}

// Split-K factor: enough workgroups to cover the 256 compute units about twice, but every
// split keeps at least 4 chunks (256 inputs) so the fp32 partial traffic stays small.
int pick_ksplit(int Npad, int Kpad, int max_ksplit) {
  const int ntiles = Npad / 32;
  const int wgs_n = (ntiles + 3) / 4;  // NT = 1
  const int nchunks = Kpad / KC;
  int ks = (384 + wgs_n - 1) / wgs_n;
  if (ks > nchunks / 4) ks = nchunks / 4;
  if (ks > max_ksplit) ks = max_ksplit;
  if (ks < 1) ks = 1;
  // no empty split: ceil(nchunks / ks) * (ks - 1) < nchunks
  while (ks > 1 && ((nchunks + ks - 1) / ks) * (ks - 1) >= nchunks) --ks;
  return ks;
}

int launch_gemm_bf16(int epi, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit,
                     void* out, size_t ldo, size_t out_split_stride, hipStream_t st) {
  if (B < 1 || B > GOOSE_MAX_B || (Npad & 31) || (Kpad & 63) || ksplit < 1) return GOOSE_ERR_ARG;
  const int MT = (B + 31) / 32;
  if (epi == EPI_SWIGLU) {
    if (ksplit != 1 || (Npad & 63)) return GOOSE_ERR_ARG;
    return launch_mt<2, EPI_SWIGLU>(MT, A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, st);
  }
  return launch_mt<1, EPI_PARTIAL>(MT, A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, st);
}
