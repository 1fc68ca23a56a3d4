// Many-row GEMM of 16-bit operands (bf16 or fp16) for gfx950: out[m][n] = sum_k A[m][k] * W[n][k] for the stacked rows of a
// batch of requests, 128 < M <= 512 (the batch sweep of App. D).  Same operands and the same
// results, bit for bit, as the skinny kernel of gemm_bf16.hip (each accumulator takes its k-steps
// in ascending order there and here), but organised for the matrix cores rather than for the
// weight stream alone: with hundreds of rows a weight byte is used often enough that the pass
// sits near the ridge between HBM and MFMA, and what limits a kernel there is the operand traffic
// inside the chip (L2 -> compute unit, LDS -> registers) per matrix instruction.
//
//   * A wavefront owns MT x NT tiles of 32 x 32 outputs (MT = 4 row tiles, NT = 2 column tiles:
//     128 accumulator registers; 8 x 2 or 4 x 4 would halve the operand traffic again but the
//     compiler spills them): an A operand read from LDS feeds NT instructions, a weight operand MT.
//   * A workgroup = 4 wavefronts on neighbouring column tiles sharing one chunk of MT*32 rows:
//     the chunk's K slices (KC = 64 inputs) are staged in LDS, double buffered, as in the skinny
//     kernel; the weights go global -> registers in operand order, two stages ahead.
//   * Row chunks of one column group run on ONE XCD in neighbouring launch slots (workgroups are
//     dealt to the 8 XCDs round-robin), so the later chunks find the weights in that XCD's L2.
//   Measured on MI355X (28672 x 4096 gate/up, 512 rows): 135 us = 0.89 PFLOP/s, 36 % of the bf16
//   MFMA peak; the chunked skinny kernel takes 178 us.  One workgroup per compute unit (registers),
//   measured with parts compiled out: matrix instructions alone 85 us (a single wavefront per SIMD
//   issues them at 57 % of the nominal rate), everything but them 80 us, together 135 us -- the two
//   overlap only in part.  A third LDS buffer with the next stage's operands read across the
//   barrier, and exact wait counts, changed nothing.
//   * Epilogues: fp32 split-K partials, or SwiGLU (the gate tile and the up tile of 32 hidden
//     columns are the two column tiles of one wavefront: no exchange needed).
#include <type_traits>

#include "goose_internal.h"
#include "mma16.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int NW = 4;   // wavefronts per workgroup
constexpr int NT = 2;   // column tiles per wavefront

// KC: inputs per stage; TERMS: terms of the activation operand (gemm_bf16.hip): with two, every weight
// operand meets the hi and then the lo operand of its rows, as in the skinny kernel
template <int MT, int EPI, int KC, bool F16, int TERMS>
__global__ __launch_bounds__(64 * NW) void k_gemm_rows(const typename Mma16<F16>::T* A, int lda, const u32x4* __restrict__ Wp,
                                                       int ntiles, int ksteps_total, int stages_per_split, int B,
                                                       void* __restrict__ out, size_t ldo, size_t split_stride, int gx,
                                                       int nsplit, int nchunk, float out_scale,
                                                       int32_t* __restrict__ flags) {
  typedef typename Mma16<F16>::T T;
  typedef typename Mma16<F16>::v8 op8;
  constexpr int LDS_ROW = KC * 2 * TERMS + 16;  // bytes; an odd number of 16-byte units: rows start in different banks
  constexpr int NTHR = 64 * NW;
  constexpr int STEPS = KC / 16;
  constexpr int ASEG = MT * 32 * (KC / 8) * TERMS;  // 16-byte segments of one A stage
  constexpr int APT = ASEG / NTHR;
  static_assert(ASEG % NTHR == 0, "A stage must divide evenly over the workgroup");
  constexpr int STAGE_BYTES = MT * 32 * LDS_ROW;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // 2 * STAGE_BYTES
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // work item = (column group bx, split-K range by, row chunk); see the XCD note above
  const int xcd = blockIdx.x & 7, slot_id = blockIdx.x >> 3;
  const int j = slot_id / nchunk, chunk = slot_id - j * nchunk;
  const int t = j * 8 + xcd;
  if (t >= gx * nsplit) return;  // the grid is rounded up to whole groups of 8
  const int by = t / gx, bx = t - by * gx;
  const int row_base = chunk * MT * 32;
  A += (size_t)row_base * lda;
  const int tile0 = (bx * NW + wave) * NT;

  const int nstages_total = ksteps_total / STEPS;
  const int s_begin = by * stages_per_split;
  const int s_end = min(s_begin + stages_per_split, nstages_total);
  const int nst = s_end - s_begin;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

  // both operand streams run two stages ahead in registers (slots st % 2, compile-time indices)
  u32x4 areg[2][APT];
  const T* a_src[APT];
  int a_dst[APT];
#pragma unroll
  for (int i = 0; i < APT; ++i) {
    const int seg = tid + NTHR * i;
    const int row = seg / (KC / 8 * TERMS), c16 = seg % (KC / 8 * TERMS);
    a_src[i] = A + (size_t)row * lda + c16 * 8;
    a_dst[i] = row * LDS_ROW + c16 * 16;
  }
  u32x4 wreg[2][STEPS][NT];
  const u32x4* wbase[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    // a tile past the last one redoes the last tile (uniform control flow) and is not stored
    const int tl = tile0 + nt < ntiles ? tile0 + nt : ntiles - 1;
    wbase[nt] = Wp + (size_t)tl * ksteps_total * 64 + lane;
  }
  auto load_a = [&](int st, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int i = 0; i < APT; ++i) areg[slot][i] = *reinterpret_cast<const u32x4*>(a_src[i] + (size_t)st * KC * TERMS);
  };
  auto store_a = [&](int buf, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int i = 0; i < APT; ++i) *reinterpret_cast<u32x4*>(&lds[buf * STAGE_BYTES + a_dst[i]]) = areg[slot][i];
  };
  auto load_w = [&](int st, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) wreg[slot][s][nt] = wbase[nt][((size_t)st * STEPS + s) * 64];
  };
  const int a_frag = (lane & 31) * LDS_ROW + (lane >> 5) * 16 * TERMS;
  auto stage = [&](auto slot_c, int st, auto next_a, auto refill) {
    constexpr int slot = decltype(slot_c)::value, buf = slot;
    const std::integral_constant<int, slot ^ 1> nslot;
    if (refill) load_a(st + 2, slot_c);  // this slot's previous content (stage st) is in LDS already
    __builtin_amdgcn_sched_barrier(0);
    // the A operands of step s+1 are read from LDS before the matrix instructions of step s issue
    op8 af[2][MT][TERMS];
    auto read_a = [&](int s, int which) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < TERMS; ++t)
          af[which][mt][t] = *reinterpret_cast<const op8*>(
              &lds[buf * STAGE_BYTES + mt * 32 * LDS_ROW + a_frag + s * 32 * TERMS + t * 16]);
    };
    read_a(0, 0);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (s + 1 < STEPS) read_a(s + 1, (s + 1) & 1);
      op8 b[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[nt] = __builtin_bit_cast(op8, wreg[slot][s][nt]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int t = 0; t < TERMS; ++t) acc[mt][nt] = Mma16<F16>::mfma(af[s & 1][mt][t], b[nt], acc[mt][nt]);
      if (refill) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wreg[slot][s][nt] = wbase[nt][((size_t)(st + 2) * STEPS + s) * 64];
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (next_a) store_a(buf ^ 1, nslot);
    __syncthreads();
  };
  const std::true_type yes;
  const std::integral_constant<int, 0> c0;
  const std::integral_constant<int, 1> c1;

  if (nst > 0) {
    int i = 0;
    if (nst >= 4) {
      // long range: both slots filled unconditionally, so that the wait counts at the loop head are exact
      load_a(s_begin, c0);
      load_w(s_begin, c0);
      load_a(s_begin + 1, c1);
      load_w(s_begin + 1, c1);
      store_a(0, c0);
      __syncthreads();
      for (; i + 3 < nst; i += 2) {
        stage(c0, s_begin + i, yes, yes);
        stage(c1, s_begin + i + 1, yes, yes);
      }
    } else {
      load_a(s_begin, c0);
      load_w(s_begin, c0);
      if (nst > 1) { load_a(s_begin + 1, c1); load_w(s_begin + 1, c1); }
      store_a(0, c0);
      __syncthreads();
    }
    for (; i < nst; ++i) {  // the last stages (i is even on entry)
      const bool na = (i + 1) < nst, rf = (i + 2) < nst;
      if ((i & 1) == 0) stage(c0, s_begin + i, na, rf);
      else stage(c1, s_begin + i, na, rf);
    }
  }

  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  if (EPI == EPI_PARTIAL) {
    float* o = reinterpret_cast<float*>(out) + by * split_stride;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      if (tile0 + nt >= ntiles) continue;
      const int col = (tile0 + nt) * 32 + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < B) o[(size_t)row * ldo + col] = acc[mt][nt][r] * out_scale;
        }
    }
  } else {  // EPI_SWIGLU: every tile holds the gate rows (columns 0-15) and the up rows (16-31) of 16 outputs
    // One row tile at a time, the wavefront passes its accumulators through LDS (register r of lane l
    // at [r][l]; the staging buffers are free after the last barrier) and walks the outputs two
    // columns at a time in a rolled loop, as the skinny kernel does: the gate values of columns 2p,
    // 2p+1 sit at lanes 2p, 2p+1 of a half, the up values 16 lanes further.  (Unrolled over all 128
    // accumulator registers this epilogue was 25 KB of code that runs once: 17 us of instruction fetch.)
    static_assert(2 * STAGE_BYTES >= NW * NT * 16 * 64 * 4, "the accumulators of one row tile must fit the staging buffers");
    T* hq = reinterpret_cast<T*>(out);
    float* mine = reinterpret_cast<float*>(lds) + (size_t)wave * (NT * 16 * 64);
    bool clamped = false;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      __builtin_amdgcn_wave_barrier();  // (LDS operations of one wavefront complete in order)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(nt * 16 + r) * 64 + lane] = acc[mt][nt][r] * out_scale;
      __builtin_amdgcn_wave_barrier();
#pragma unroll 1
      for (int e = lane; e < NT * 16 * 16; e += 64) {
        const int pr = e & 7, half = (e >> 3) & 1, rr = (e >> 4) & 15, nt = e >> 8;  // column pair, lane half, register, tile
        if (tile0 + nt >= ntiles) continue;
        const int row = row_base + mt * 32 + 8 * (rr >> 2) + 4 * half + (rr & 3);
        const int col = (tile0 + nt) * 16 + 2 * pr;
        const float* src = &mine[(nt * 16 + rr) * 64 + half * 32 + 2 * pr];
        const float2 g = *reinterpret_cast<const float2*>(src);
        const float2 u = *reinterpret_cast<const float2*>(src + 16);
        float h0 = swiglu_f32(g.x, u.x), h1 = swiglu_f32(g.y, u.y);
        if (F16) {  // beyond fp16: clamp, and say so (GOOSE_FLAG_RANGE)
          if (fabsf(h0) > 65504.0f) { h0 = copysignf(65504.0f, h0); clamped = clamped || row < B; }
          if (fabsf(h1) > 65504.0f) { h1 = copysignf(65504.0f, h1); clamped = clamped || row < B; }
        }
        if (row < B) {
          const T a0 = (T)h0, a1 = (T)h1;
          T* dst = hq + (size_t)row * ldo + term_pos(TERMS, col);
          union { T t[2]; unsigned u; } pk;
          pk.t[0] = a0; pk.t[1] = a1;
          *reinterpret_cast<unsigned*>(dst) = pk.u;
          if (TERMS == 2) {
            pk.t[0] = (T)(h0 - (float)a0); pk.t[1] = (T)(h1 - (float)a1);
            *reinterpret_cast<unsigned*>(dst + 8) = pk.u;
          }
        }
      }
    }
    if (F16 && clamped && flags != nullptr) atomicOr(flags, GOOSE_FLAG_RANGE);
  }
}

template <int MT, int EPI, int KC, bool F16, int TERMS>
int launch_rows(const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit, void* out, size_t ldo,
                size_t split_stride, float out_scale, int32_t* flags, hipStream_t st) {
  constexpr int LDS_BYTES = 2 * MT * 32 * (KC * 2 * TERMS + 16);
  static bool configured = false;  // more LDS than a kernel gets by default: ask once
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_rows<MT, EPI, KC, F16, TERMS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) { goose_note_hip_error(e, "hipFuncSetAttribute(k_gemm_rows)", __LINE__); return GOOSE_ERR_HIP; }
    configured = true;
  }
  const int ntiles = Npad / 32, ksteps = Kpad / 16;
  const int gx = (ntiles + NW * NT - 1) / (NW * NT);
  const int nchunk = (B + MT * 32 - 1) / (MT * 32);
  const int granules = Kpad / 128;                        // split-K ranges are multiples of 128 inputs,
  const int gps = (granules + ksplit - 1) / ksplit;       // the same ranges as the skinny kernel's
  const dim3 grid((gx * ksplit + 7) / 8 * 8 * nchunk);
  hipLaunchKernelGGL((k_gemm_rows<MT, EPI, KC, F16, TERMS>), grid, dim3(64 * NW), LDS_BYTES, st,
                     (const typename Mma16<F16>::T*)A, lda,
                     (const u32x4*)Wp, ntiles, ksteps, gps * (128 / KC), B, out, ldo, split_stride, gx, ksplit, nchunk, out_scale,
                     flags);
  return goose_launch_status();
}

template <int EPI>
int launch_rows_any(bool f16, int terms, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit,
                    void* out, size_t ldo, size_t split_stride, float out_scale, int32_t* flags, hipStream_t st) {
  if (terms == 2)
    return f16 ? launch_rows<4, EPI, 64, true, 2>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, out_scale, flags, st)
               : launch_rows<4, EPI, 64, false, 2>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, out_scale, flags, st);
  return f16 ? launch_rows<4, EPI, 64, true, 1>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, out_scale, flags, st)
             : launch_rows<4, EPI, 64, false, 1>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, out_scale, flags, st);
}

}  // namespace

// A must hold whole chunks of 128 readable rows.
int launch_gemm_rows_16(int dtype, int epi, const void* A, int lda, int terms, const void* Wp, int Npad, int Kpad, int B,
                        int ksplit, void* out, size_t ldo, size_t out_split_stride, float out_scale, int32_t* flags,
                        hipStream_t st) {
  if (dtype != GOOSE_DTYPE_BF16 && dtype != GOOSE_DTYPE_F16) return GOOSE_ERR_ARG;
  const bool f16 = dtype == GOOSE_DTYPE_F16;
  if (B < 1 || B > GOOSE_MAX_ROWS || (Npad & 31) || (Kpad % 128) || ksplit < 1 || (terms != 1 && terms != 2))
    return GOOSE_ERR_ARG;
  if (epi == EPI_SWIGLU) {
    if (ksplit != 1 || (Npad & 63)) return GOOSE_ERR_ARG;
    return launch_rows_any<EPI_SWIGLU>(f16, terms, A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, out_scale, flags, st);
  }
  if (epi != EPI_PARTIAL) return GOOSE_ERR_ARG;
  return launch_rows_any<EPI_PARTIAL>(f16, terms, A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, out_scale,
                                      flags, st);
}
