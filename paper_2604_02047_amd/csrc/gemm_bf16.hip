// Skinny-M bf16 GEMM for gfx950: out[m][n] = sum_k A[m][k] * W[n][k], M = tree nodes (<= 128).
//
// The pass is weight-bandwidth bound (every weight byte is used for only M multiply-adds), so
// the kernel is organised around streaming W once, with wide fully-coalesced loads:
//   * W is pre-tiled (launch_pack_bf16) into MFMA-operand order: tile (nt, kt) = 32 output
//     rows x 16 inputs = 1 KiB, lane l of a wavefront owning W[nt*32 + l%32][kt*16 + 8*(l/32) .. +7].
//     One global_load_dwordx4 per lane fetches a whole operand of v_mfma_f32_32x32x16_bf16 and
//     consecutive kt are consecutive in memory, so each wavefront reads one long contiguous run.
//   * The M x K activation block is small and shared: the workgroup stages 128-wide K slices of it
//     in LDS (double buffered) and every wavefront reads its A operands from there.
//   * 2 or 4 wavefronts per workgroup, one column tile each; split-K over blockIdx.y writes
//     fp32 partials that the next (reduction / rotary / norm) kernel sums in a fixed order.
#include <stdlib.h>

#include <type_traits>

#include "goose_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int KC = 128;              // k extent of one LDS stage
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
// One workgroup = NW compute wavefronts + 1 loader wavefront.
//   * Compute wavefront w owns column tile blockIdx.x*NW + w (32 columns) and all MT row tiles;
//     blockIdx.y selects the split-K range.  Its only global loads are weight operands, kept in a
//     register ring of RING stages (8 loads = 8 KiB each): a slot is refilled for stage st+RING
//     right after the MFMAs of stage st consumed it.  Loads retire in order, so with nothing else
//     in the wavefront's load queue the compiler can wait for exactly the operand it needs and
//     RING*8 - 1 loads stay in flight all the time.
//   * The loader wavefront copies the A stages global -> registers -> LDS, two stages ahead of
//     the multiply (its waits never stall the weight stream).
//   * One barrier per stage (KC = 128 inputs) hands LDS buffers back and forth.
// EPI_SWIGLU: even wavefronts hold gate tiles, odd ones the matching up tiles; the up tile
// is handed over through LDS and the even wavefront writes h = silu(gate) * up.
template <int MT, int NW, int EPI, int RING>
__global__ __launch_bounds__(64 * (NW + 1)) void k_gemm_bf16(const bf16_t* __restrict__ A, int lda,
                                                             const u32x4* __restrict__ Wp, int ntiles,
                                                             int ksteps_total, int stages_per_split, int B,
                                                             void* __restrict__ out, size_t ldo,
                                                             size_t split_stride, int dbg) {
  constexpr int STEPS = KC / 16;               // MFMA k-steps per stage
  constexpr int APL = MT * 32 * (KC / 8) / 64;  // 16-byte segments of one A stage per loader lane
  constexpr int STAGE_BYTES = MT * 32 * LDS_ROW;
  constexpr int SWAP_BYTES = (EPI == EPI_SWIGLU) ? (NW / 2) * MT * 16 * 64 * 4 : 0;
  constexpr int LDS_BYTES = 2 * STAGE_BYTES > SWAP_BYTES ? 2 * STAGE_BYTES : SWAP_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nstages_total = ksteps_total / STEPS;
  const int s_begin = blockIdx.y * stages_per_split;
  const int s_end = min(s_begin + stages_per_split, nstages_total);
  const int nst = s_end - s_begin;
  const std::integral_constant<int, 0> c0;
  const std::integral_constant<int, 1> c1;
  const std::integral_constant<int, 2> c2;
  const std::true_type yes;

  if (wave == NW && (dbg & 2)) return;  // DEBUG: no loader, no barriers
  if (wave == NW) {
    // ---------------- loader wavefront: A stage st -> LDS buffer st & 1, published by the barrier
    // that ends stage st - 1.  Registers hold the stage after that one while it is in flight.
    // lane l copies segment (row l/16 + 4*i, 16-byte column l%16) for i = 0..APL-1
    const bf16_t* src0 = A + (size_t)(lane >> 4) * lda + (lane & 15) * 8;
    const int dst0 = (lane >> 4) * LDS_ROW + (lane & 15) * 16;
    const size_t src_step = (size_t)4 * lda;
    constexpr int dst_step = 4 * LDS_ROW;
    // The multiply loop runs an even number of stages; a phantom last stage gets zeros.
    const int nst2 = (nst + 1) & ~1;
    if constexpr (APL <= 16) {
      u32x4 areg[2][APL];
      auto load_a = [&](int i, auto r_c) {   // stage i of this split, zeros past the end
        constexpr int r = decltype(r_c)::value;
        if (i < nst) {
#pragma unroll
          for (int k = 0; k < APL; ++k)
            areg[r][k] = *reinterpret_cast<const u32x4*>(src0 + k * src_step + (size_t)(s_begin + i) * KC);
        } else {
#pragma unroll
          for (int k = 0; k < APL; ++k) areg[r][k] = u32x4{0, 0, 0, 0};
        }
      };
      auto store_a = [&](int buf, auto r_c) {
        constexpr int r = decltype(r_c)::value;
#pragma unroll
        for (int k = 0; k < APL; ++k)
          *reinterpret_cast<u32x4*>(&lds[buf * STAGE_BYTES + dst0 + k * dst_step]) = areg[r][k];
      };
      if (nst > 0) {
        load_a(0, c0);
        load_a(1, c1);
        store_a(0, c0);
        __syncthreads();
        // during stage i: fetch stage i+2 into the register set that stage i used, publish stage i+1
        for (int i = 0; i < nst2; i += 2) {
          if (i + 2 < nst2) load_a(i + 2, c0);
          store_a(1, c1);
          __syncthreads();
          if (i + 3 < nst2) load_a(i + 3, c1);
          if (i + 2 < nst2) store_a(0, c0);
          __syncthreads();
        }
      }
    } else {
      // tall A blocks (3 or 4 row tiles): one stage of look-ahead, copied in chunks of 16 segments
      // so that the loader never needs more registers than the compute wavefronts
      auto copy_stage = [&](int i, int buf) {
#pragma unroll
        for (int h = 0; h < APL; h += 16) {
          u32x4 t[16];
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (h + k < APL)
              t[k] = (i < nst) ? *reinterpret_cast<const u32x4*>(src0 + (h + k) * src_step + (size_t)(s_begin + i) * KC)
                               : u32x4{0, 0, 0, 0};
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (h + k < APL) *reinterpret_cast<u32x4*>(&lds[buf * STAGE_BYTES + dst0 + (h + k) * dst_step]) = t[k];
        }
      };
      if (nst > 0) {
        copy_stage(0, 0);
        __syncthreads();
        for (int i = 0; i < nst2; ++i) {
          if (i + 1 < nst2) copy_stage(i + 1, (i + 1) & 1);
          __syncthreads();
        }
      }
    }
    if (EPI == EPI_SWIGLU) __syncthreads();  // the epilogue's hand-over barrier
    return;
  }

  // ---------------- compute wavefronts
  const int tile = blockIdx.x * NW + wave;
  const bool active = tile < ntiles;
  // a wavefront past the last tile redoes the last tile (no divergent control flow in the
  // pipeline) and skips the store
  const int tile_ld = active ? tile : ntiles - 1;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  // Weight stream: a register ring of two stages (16 operand loads = 16 KiB per wavefront), issued
  // and awaited BY HAND.  These wavefronts have nothing else in their vector-memory queue and loads
  // retire in order, so "at most 15 loads outstanding" is exactly "the oldest one has arrived":
  // the ring stays full all the time.  (Left to the compiler, the wait counts are merged
  // conservatively around the loop and half of the ring drains at every stage.)
  // The compiler does not know that these registers are written asynchronously, so the code is
  // shaped to give it no reason to touch them in between: ONE loop block, every register defined
  // by one asm and consumed by the next wait asm in the same block, no separate tail code.  To
  // that end the loop always runs an even number of stages and always refills: past the end of
  // the split the refill re-reads the first KiB of the matrix (always cached) and a phantom odd
  // stage multiplies zeros staged by the loader.  After the loop everything is awaited before the
  // registers are reused.
  static_assert(RING == 2, "the hand-scheduled weight stream is written for a ring of two stages");
  u32x4 wreg[2][STEPS];
  const u32x4* wdummy = Wp + lane;
  const u32x4* wbase = Wp + (size_t)tile_ld * ksteps_total * 64 + lane;
  auto issue = [&](u32x4& dst, const u32x4* p) {
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(dst) : "v"(p) : "memory");
  };
  auto stage_ptr = [&](int i) { return (i < nst) ? wbase + (size_t)(s_begin + i) * STEPS * 64 : wdummy; };
  const int a_frag = (lane & 31) * LDS_ROW + (lane >> 5) * 16;
  auto half = [&](auto buf_c, int i) {
    constexpr int buf = decltype(buf_c)::value, slot = buf;
    const u32x4* pn = stage_ptr(i + 2);
    const int pstep = (i + 2 < nst) ? 64 : 0;  // the stand-in load keeps hitting the same KiB
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      asm volatile("s_waitcnt vmcnt(15)" : "+v"(wreg[slot][s]));
      const bf16x8 b = __builtin_bit_cast(bf16x8, wreg[slot][s]);
      if (dbg & 1) {  // DEBUG: no LDS reads, no MFMA
        acc[0][s] += __builtin_bit_cast(f32x16, (u32x4[4]){wreg[slot][s], wreg[slot][s], wreg[slot][s], wreg[slot][s]})[s];
      } else {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(
            &lds[buf * STAGE_BYTES + mt * 32 * LDS_ROW + a_frag + s * 32]);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[mt], 0, 0, 0);
      }
      }
      issue(wreg[slot][s], pn + s * pstep);
    }
    if (!(dbg & 2)) __syncthreads();
  };
  if (nst > 0) {
    const int nst2 = (nst + 1) & ~1;
    {
      const u32x4* p0 = stage_ptr(0);
      const u32x4* p1 = stage_ptr(1);
      const int st1 = (1 < nst) ? 64 : 0;
#pragma unroll
      for (int s = 0; s < STEPS; ++s) issue(wreg[0][s], p0 + s * 64);
#pragma unroll
      for (int s = 0; s < STEPS; ++s) issue(wreg[1][s], p1 + s * st1);
    }
    if (!(dbg & 2)) __syncthreads();
    for (int i = 0; i < nst2; i += 2) {
      half(c0, i);
      half(c1, i + 1);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the stand-in refills still target the ring
    __builtin_amdgcn_sched_barrier(0);
  }

  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  if (EPI == EPI_PARTIAL) {
    if (!active) return;
    float* o = reinterpret_cast<float*>(out) + blockIdx.y * split_stride;
    const int col = tile * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < B) o[(size_t)row * ldo + col] = acc[mt][r];
      }
  } else {  // EPI_SWIGLU (the last loop barrier already separates the A stages from this reuse of LDS)
    float* swap = reinterpret_cast<float*>(lds) + (size_t)(wave >> 1) * MT * 16 * 64;
    if (active && (wave & 1)) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) swap[(mt * 16 + r) * 64 + lane] = acc[mt][r];
    }
    __syncthreads();
    if (active && !(wave & 1)) {
      bf16_t* hq = reinterpret_cast<bf16_t*>(out);
      const int col = (tile >> 1) * 32 + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const float g = acc[mt][r], u = swap[(mt * 16 + r) * 64 + lane];
          if (row < B) hq[(size_t)row * ldo + col] = (bf16_t)(g / (1.0f + __expf(-g)) * u);
        }
    }
  }
}

template <int MT, int NW, int EPI>
int launch_one(const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit, void* out, size_t ldo,
               size_t split_stride, int ring, hipStream_t st) {
  const int ntiles = Npad / 32, ksteps = Kpad / 16, nstages = Kpad / KC;
  const int sps = (nstages + ksplit - 1) / ksplit;
  dim3 grid((ntiles + NW - 1) / NW, ksplit), block(64 * (NW + 1));
  (void)ring;
  static const int dbg = []() { const char* v = getenv("GOOSE_DBG"); return v ? atoi(v) : 0; }();
  hipLaunchKernelGGL((k_gemm_bf16<MT, NW, EPI, 2>), grid, block, 0, st, (const bf16_t*)A, lda, (const u32x4*)Wp,
                     ntiles, ksteps, sps, B, out, ldo, split_stride, dbg);
  return goose_launch_status();
}

template <int NW, int EPI>
int launch_mt(int MT, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int ksplit, void* out,
              size_t ldo, size_t split_stride, int ring, hipStream_t st) {
  switch (MT) {
    case 1: return launch_one<1, NW, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, ring, st);
    case 2: return launch_one<2, NW, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, ring, st);
    case 3: return launch_one<3, NW, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, ring, st);
    case 4: return launch_one<4, NW, EPI>(A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, split_stride, ring, st);
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

// Workgroup width (wavefronts = column tiles per workgroup) and split-K factor for a shape.
// Streaming needs about 1000 wavefronts with 8 KiB of loads in flight each to keep HBM busy, so
// split K until tiles * ksplit reaches that, but keep every split at least 4 stages long; use
// the 4-wide workgroup (more sharing of the staged A block) whenever that still leaves >= 256
// workgroups.
void pick_gemm_config(int Npad, int Kpad, int max_ksplit, int* nw_out, int* ksplit_out) {
  const int ntiles = Npad / 32, nstages = Kpad / KC;
  int ks = (1024 + ntiles - 1) / ntiles;
  if (ks > nstages / 4) ks = nstages / 4;
  if (ks > max_ksplit) ks = max_ksplit;
  if (ks < 1) ks = 1;
  while (ks > 1 && ((nstages + ks - 1) / ks) * (ks - 1) >= nstages) --ks;  // no empty split
  *nw_out = (((ntiles + 3) / 4) * ks >= 256) ? 4 : 2;
  *ksplit_out = ks;
}

int launch_gemm_bf16(int epi, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int nw, int ksplit,
                     void* out, size_t ldo, size_t out_split_stride, hipStream_t st) {
  if (B < 1 || B > GOOSE_MAX_B || (Npad & 31) || (Kpad % KC) || ksplit < 1) return GOOSE_ERR_ARG;
  const int MT = (B + 31) / 32;
  if (MT == 4) nw = 2;  // 4 row tiles x 4 column wavefronts would exceed the register file (spills)
  static const int ring = []() {
    const char* v = getenv("GOOSE_RING");
    const int r = v ? atoi(v) : 3;
    return (r >= 2 && r <= 4) ? r : 3;
  }();
  if (epi == EPI_SWIGLU) {
    if (ksplit != 1 || (Npad & 63)) return GOOSE_ERR_ARG;
    if (nw == 4) return launch_mt<4, EPI_SWIGLU>(MT, A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, ring, st);
    return launch_mt<2, EPI_SWIGLU>(MT, A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, ring, st);
  }
  if (nw == 4)
    return launch_mt<4, EPI_PARTIAL>(MT, A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, ring, st);
  return launch_mt<2, EPI_PARTIAL>(MT, A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, ring, st);
}
