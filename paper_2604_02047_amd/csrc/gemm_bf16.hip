// Skinny-M GEMM of 16-bit operands (bf16 or fp16) for gfx950: out[m][n] = sum_k A[m][k] * W[n][k],
// M = tree nodes (<= 128).
//
// The pass is weight-bandwidth bound (every weight byte is used for only M multiply-adds), so
// the kernel is organised around streaming W once, with wide fully-coalesced loads:
//   * W is pre-tiled (launch_pack_16) into MFMA-operand order: tile (nt, kt) = 32 output
//     rows x 16 inputs = 1 KiB, lane l of a wavefront owning W[nt*32 + l%32][kt*16 + 8*(l/32) .. +7].
//     One global_load_dwordx4 per lane fetches a whole operand of v_mfma_f32_32x32x16_{bf16,f16} and
//     consecutive kt are consecutive in memory, so each wavefront reads one long contiguous run.
//   * The M x K activation block is small and shared: the workgroup stages 128-wide K slices of it
//     in LDS (double buffered) and every wavefront reads its A operands from there.
//   * 2 or 4 wavefronts per workgroup, one column tile each; split-K over blockIdx.y writes
//     fp32 partials that the next (reduction / rotary / norm) kernel sums in a fixed order.
#include <stdlib.h>

#include <type_traits>

#include "goose_internal.h"
#include "mma16.h"
#include <climits>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int KGRAN = 128;  // granularity of K padding and of split-K ranges (inputs)

// ------------------------------------------------------------------------------------------
// Re-tile raw row-major matrices of 16-bit elements (moved as bit patterns: bf16 or fp16).  Packed row n comes from
//   PACK_PLAIN   : s0 row n
//   PACK_QKV     : q|k|v stacked: rows_each rows of s0, then rows_kv rows of s1, then rows_kv rows of s2
//   PACK_GATE_UP : blocks of 32 rows alternate gate (s0) / up (s1): block b -> (b&1 ? up : gate) rows (b>>1)*32..
// Rows and columns outside the source are zero.
// cvt_exp > 0: the source is bf16 and every weight w is RE-ENCODED as the fp16 value w * 2^cvt_exp
// (the projections then run the fp16 matrix instruction, whose activation operand keeps 11
// instead of 8 significant bits, and scale their sums by 2^-cvt_exp).  With cvt_exp = 8 the
// re-encoding is exact for 2^-32 <= |w| < 256 (eight significant bits always fit); a weight outside
// that range is saturated or rounded and raises GOOSE_FLAG_WEIGHT_RANGE.
__global__ __launch_bounds__(256) void k_pack_bf16(int mode, const bf16_t* __restrict__ s0,
                                                   const bf16_t* __restrict__ s1, const bf16_t* __restrict__ s2,
                                                   int rows_each, int rows_kv, int K, int ktiles, size_t total,
                                                   uint4* __restrict__ dst, int cvt_exp, int32_t* __restrict__ flags) {
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;  // one 16-byte lane slot
  if (idx >= total) return;
  const int lane = idx & 63;
  const size_t tile = idx >> 6;
  const int kt = tile % ktiles;
  const int nt = tile / ktiles;
  const int n = nt * 32 + (lane & 31);
  const int k0 = kt * 16 + (lane >> 5) * 8;
  const bf16_t* src = nullptr;
  int row = 0, limit = rows_each;
  if (mode == PACK_PLAIN) {
    src = s0; row = n;
  } else if (mode == PACK_QKV) {  // q rows, then k rows, then v rows (k and v may be narrower: grouped queries)
    if (n < rows_each) { src = s0; row = n; }
    else if (n < rows_each + rows_kv) { src = s1; row = n - rows_each; limit = rows_kv; }
    else if (n < rows_each + 2 * rows_kv) { src = s2; row = n - rows_each - rows_kv; limit = rows_kv; }
  } else {
    const int blk = n >> 5;
    row = (blk >> 1) * 32 + (n & 31);
    src = (blk & 1) ? s1 : s0;
  }
  union { uint4 u; bf16_t e[8]; _Float16 h[8]; } v;
  v.u = make_uint4(0, 0, 0, 0);
  if (src != nullptr && row < limit) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (k0 + e < K) v.e[e] = src[(size_t)row * K + k0 + e];
    if (cvt_exp > 0) {
      bool inexact = false;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float w = ldexpf((float)v.e[e], cvt_exp);
        const float c = fminf(fmaxf(w, -65504.0f), 65504.0f);
        const _Float16 hv = (_Float16)c;
        inexact = inexact || (float)hv != w;
        v.h[e] = hv;
      }
      if (inexact && flags != nullptr) atomicOr(flags, GOOSE_FLAG_WEIGHT_RANGE);
    }
  }
  dst[idx] = v.u;
}

// ------------------------------------------------------------------------------------------
// One workgroup = NW wavefronts, wavefront w owns column tile blockIdx.x*NW + w (32 columns) and
// all MT row tiles.  blockIdx.y selects the split-K range.
//
// Operand A (activations), TERMS = 1 or 2.  With two terms an activation is carried as the sum of
// two 16-bit values, a = hi + lo with lo = T(a - hi): the rounding of the projection's input then
// drops from 2^-9 to 2^-17 relative, at the price of a second matrix instruction per weight piece
// (the matrix cores idle most of the time at these row counts) and twice the bytes of the small
// operand.  Storage is interleaved in groups of eight inputs: the 16 bytes of hi values of inputs
// 8j..8j+7 are followed by the 16 bytes of their lo values (row length 2*K elements).
//
// Per stage (128 inputs):
//   - A goes global -> LDS directly (global_load_lds, 16 bytes per lane, no registers): every
//     wavefront copies its share of the next stage's rows while the current stage is consumed.  The
//     hardware puts lane i's 16 bytes at base + 16 i, so rows cannot be padded; bank conflicts of the
//     operand reads are avoided by a swizzle instead: the unit (16 bytes) at position p of row r
//     holds the row's unit p ^ (r % 16), arranged by choosing which unit each lane fetches.
//   - every wavefront keeps two stages (16 KiB) of its own weight pieces in flight in registers,
//     refilled right after the matrix instructions that consumed them;
//   - one s_barrier.  These loads complete in order as far as the wait counter goes, and nothing
//     tells the compiler that a direct-to-LDS load must have landed before another wavefront reads
//     the buffer, so the wait before each barrier is written out by hand: everything up to and
//     including the A copy issued this stage (the weight loads issued after it stay in flight).
// out_scale multiplies every sum before the epilogue uses it (an exact power of two: weights that
// were re-encoded as scaled fp16, see launch_pack_16).
// EPI_SWIGLU: even tiles are gate tiles, odd ones the matching up tiles; the up tile
// is handed over through LDS and the even wavefront writes h = silu(gate) * up (in TERMS terms).
// EPI_TOP2: besides the optional plain output, every workgroup reduces its columns to one
// (largest, second largest, index of largest) triple per row, for the greedy argmax.
// CHUNKED: more than MT*32 rows, computed as several row chunks that read the same weights (1-D
// grid in an XCD-aware order, ordinary loads so that the chunks share the L2); otherwise the
// weights are read once by the whole grid, with non-temporal loads that keep them from displacing
// the L2's other lines.  F16: fp16 instead of bf16 operands (and SwiGLU output).
#define GOOSE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }  // s_waitcnt vmcnt(n) only

template <int MT, int NW, int TERMS, int EPI, bool CHUNKED = false, bool F16 = false>
__global__ __launch_bounds__(64 * NW) void k_gemm_bf16(const typename Mma16<F16>::T* __restrict__ A, int lda,
                                                            const u32x4* __restrict__ Wp, int ntiles, int ksteps_total,
                                                            int stages_per_split, int B, void* __restrict__ out,
                                                            size_t ldo, size_t split_stride,
                                                            float4* __restrict__ top2, int n_valid, int gx, int nsplit,
                                                            int nchunk, float out_scale, int32_t* __restrict__ flags) {
  typedef typename Mma16<F16>::T T;
  typedef typename Mma16<F16>::v8 op8;
  constexpr int KC = 128, STEPS = KC / 16;
  constexpr int NWAVES = NW;
  constexpr int SU = 16 * TERMS;                       // 16-byte units per row per stage
  constexpr int ROW_BYTES = SU * 16;
  constexpr int STAGE_BYTES = MT * 32 * ROW_BYTES;
  constexpr int ROWS_PER_COPY = 64 / SU;               // rows one wavefront-wide copy instruction fills
  constexpr int COPIES = MT * 32 / ROWS_PER_COPY;
  constexpr int CPW = COPIES / NWAVES;                 // copy instructions per wavefront per stage
  static_assert(COPIES % NWAVES == 0, "the A copy must divide evenly over the wavefronts");
  constexpr int SWAP_BYTES = (EPI == EPI_SWIGLU) ? (NW / 2) * MT * 16 * 64 * 4 : 0;
  constexpr int CT_ROW = 33;  // floats per row of a transposed-read C tile (odd: conflict-free row scans)
  constexpr int TOP2_BYTES = (EPI == EPI_TOP2) ? NW * MT * 32 * (CT_ROW * 4 + 16) : 0;
  constexpr int EPI_BYTES = SWAP_BYTES > TOP2_BYTES ? SWAP_BYTES : TOP2_BYTES;
  constexpr int TAIL_BYTES = EPI_BYTES;
  // Two buffers as two separate arrays: the compiler then knows that the copy into one does not
  // touch what is read from the other (with one array it makes every operand read wait for the copy
  // just issued, i.e. for all loads in flight).  The epilogues reuse the first.
  constexpr int LDS0_BYTES = STAGE_BYTES > TAIL_BYTES ? STAGE_BYTES : TAIL_BYTES;
  static_assert(LDS0_BYTES + STAGE_BYTES <= 160 * 1024, "LDS of one compute unit");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS0_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char lds1[STAGE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave;  // this wavefront's column tile
  // Work item = (column-tile group bx, split-K range by, row chunk of MT*32 rows).  One chunk: the
  // plain 2-D grid.  Several chunks: a 1-D grid; workgroups are dealt to the 8 XCDs round-robin in
  // launch order and the chunks of one (bx, by) read the same weights, so they take consecutive
  // slots of ONE XCD: its L2 then serves all but the first.
  constexpr bool STREAM = !CHUNKED;
  int bx = blockIdx.x, by = blockIdx.y, row_base = 0, ngroups = gridDim.x;
  if (CHUNKED) {
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int j = slot / nchunk, chunk = slot - j * nchunk;
    const int t = j * 8 + xcd;
    if (t >= gx * nsplit) return;  // the grid is rounded up to whole groups of 8
    by = t / gx;
    bx = t - by * gx;
    row_base = chunk * MT * 32;
    ngroups = gx;
  }
  const int tile = bx * NW + wt;
  const bool active = tile < ntiles;
  // a wavefront past the last tile redoes the last tile (no divergent control flow in the
  // pipeline, which lets the compiler count outstanding loads exactly) and skips the store
  const int tile_ld = active ? tile : ntiles - 1;
  const int nstages_total = ksteps_total / STEPS;
  const int s_begin = by * stages_per_split;
  const int s_end = min(s_begin + stages_per_split, nstages_total);
  const int nst = s_end - s_begin;
  const int s0 = s_begin;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  // ---- this wavefront's share of the A copy: copy instruction c of the stage fills rows
  // c*ROWS_PER_COPY ..; lane i fetches the unit that belongs at position i % SU of row i / SU
  // (swizzled, see above)
  const u32x4* a_src[CPW];
  const int row_units = lda >> 3;  // 16-byte units per operand row
#pragma unroll
  for (int q = 0; q < CPW; ++q) {
    const int c = wave * CPW + q;
    const int row = c * ROWS_PER_COPY + lane / SU, pos = lane % SU;
    const int unit = (pos & ~15) | ((pos ^ row) & 15);
    a_src[q] = reinterpret_cast<const u32x4*>(A) + (size_t)(row_base + row) * row_units +
               (size_t)s_begin * SU + unit;
  }
  auto copy_a = [&](int i, auto buf_c) {  // stage i -> LDS buffer buf
    constexpr int buf = decltype(buf_c)::value;
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
      const int c = wave * CPW + q;  // (wavefront-uniform)
      unsigned char* dst = (buf ? lds1 : lds) + c * 1024;
#if defined(__HIP_DEVICE_COMPILE__)  // (the host pass knows no such builtin and would silently drop the kernel's stub)
      __builtin_amdgcn_global_load_lds(a_src[q] + (size_t)i * SU, GOOSE_LDS_PTR(dst), 16, 0, 0);
#else
      (void)dst;
#endif
    }
  };
  u32x4 wreg[2][STEPS];
  const u32x4* wbase = Wp + (size_t)tile_ld * ksteps_total * 64 + (size_t)s0 * STEPS * 64 + lane;
  auto load_w = [&](int i, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
    const u32x4* p = wbase + (size_t)i * STEPS * 64;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) wreg[slot][s] = STREAM ? __builtin_nontemporal_load(p + s * 64) : p[s * 64];
  };
  // operand reads: lane l holds row l % 32 (of row tile mt) and the eight inputs 8*(l/32).. of a k-step
  const int a_row = (lane & 31) * ROW_BYTES, a_x = lane & 15, a_hh = lane >> 5;
  auto barrier = [&]() {  // (raw: __syncthreads would also drain every load in flight)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  // one stage (slot = i % 2, compile-time so that no register array is indexed dynamically; the
  // LDS buffer alternates with it)
  auto stage = [&](auto slot_c, int i, auto next_a, auto refill) {
    constexpr int slot = decltype(slot_c)::value, buf = slot;
    const unsigned char* abuf = buf ? lds1 : lds;
    if (next_a) copy_a(i + 1, std::integral_constant<int, buf ^ 1>());  // (its readers passed the barrier that ended stage i-1)
    __builtin_amdgcn_sched_barrier(0);   // keep the issue order: the scheduler would sink these loads
    const u32x4* pn = wbase + (size_t)(i + 2) * STEPS * 64;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      const op8 b = __builtin_bit_cast(op8, wreg[slot][s]);
      // (terms outside, row tiles inside: consecutive matrix instructions then go to different
      // accumulators instead of waiting for each other; every accumulator still takes hi before lo)
#pragma unroll
      for (int t = 0; t < TERMS; ++t) {
        const int unit = (2 * s + a_hh) * TERMS + t;
        const int pos = (unit & ~15) | ((unit ^ a_x) & 15);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const op8 a = *reinterpret_cast<const op8*>(&abuf[mt * 32 * ROW_BYTES + a_row + pos * 16]);
          acc[mt] = Mma16<F16>::mfma(a, b, acc[mt]);
        }
      }
      if (refill) wreg[slot][s] = STREAM ? __builtin_nontemporal_load(pn + s * 64) : pn[s * 64];
      __builtin_amdgcn_sched_barrier(0);
    }
    // the next stage's A (issued above, before this stage's weight refills) must have landed in
    // LDS before anyone reads it; the STEPS refills issued after it may stay in flight
    if (next_a) {
      if (refill) __builtin_amdgcn_s_waitcnt(vmcnt_imm(STEPS));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    barrier();
  };
  const std::true_type yes;
  const std::integral_constant<int, 0> c0;
  const std::integral_constant<int, 1> c1;

  if (nst > 0) {
    int i = 0;
    copy_a(0, std::integral_constant<int, 0>());
    if (nst >= 4) {
      // long range: both slots are filled unconditionally, so that the compiler's wait counts at
      // the loop head are exact (it merges all paths into the loop, and a path with fewer loads
      // in flight would make every iteration drain the ring)
      load_w(0, c0);
      load_w(1, c1);
      // stage 0 of both streams has arrived, stage 1 of the weights is in flight: the state every
      // stage below starts from.  (The compiler counts the copies to LDS and the register loads as
      // two kinds that may overtake each other, and falls back to waiting for ALL loads wherever it
      // has to wait for one with both kinds pending; so the waits are placed here and before each
      // barrier by hand, and inside a stage everything it consumes is known to be there.)
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(STEPS));
      barrier();
      for (; i + 3 < nst; i += 2) {  // steady state: no conditionals inside
        stage(c0, i, yes, yes);
        stage(c1, i + 1, yes, yes);
      }
    } else {
      load_w(0, c0);
      if (nst > 1) load_w(1, c1);
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      barrier();
    }
    for (; i < nst; ++i) {  // the last stages (i is even on entry)
      const bool na = (i + 1) < nst, rf = (i + 2) < nst;
      if ((i & 1) == 0) stage(c0, i, na, rf);
      else stage(c1, i, na, rf);
    }
  }

  const bool writer = active;

  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  if (EPI == EPI_PARTIAL) {
    if (!writer) return;
    float* o = reinterpret_cast<float*>(out) + by * split_stride;
    const int col = tile * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row_base + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < B) o[(size_t)row * ldo + col] = acc[mt][r] * out_scale;
      }
  } else if (EPI == EPI_TOP2) {
    constexpr int ROWS = MT * 32;
    float* o = reinterpret_cast<float*>(out);
    float* ct = reinterpret_cast<float*>(lds) + wt * ROWS * CT_ROW;
    float4* red4 = reinterpret_cast<float4*>(lds + NW * ROWS * CT_ROW * 4);
    const int col = tile * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const float v = acc[mt][r] * out_scale;
        if (o != nullptr && active && row_base + row < B) o[(size_t)(row_base + row) * ldo + col] = v;
        ct[row * CT_ROW + (lane & 31)] = v;
      }
    __syncthreads();
    // lane = row: scan the tile's 32 columns in ascending order (the lowest index wins a tie)
    {
      for (int row = lane; row < ROWS; row += 64) {
        float v1 = -INFINITY, v2 = -INFINITY;
        int i1 = INT_MAX;
        const int c_end = active ? min(32, n_valid - tile * 32) : 0;
        for (int cc = 0; cc < c_end; ++cc) {
          const float v = ct[row * CT_ROW + cc];
          if (v > v1) { v2 = v1; v1 = v; i1 = tile * 32 + cc; }
          else v2 = fmaxf(v2, v);
        }
        red4[wt * ROWS + row] = make_float4(v1, v2, __int_as_float(i1), 0.f);
      }
    }
    __syncthreads();
    if (wave == 0) {
      for (int row = lane; row < ROWS; row += 64) {
        float4 t = red4[row];
#pragma unroll
        for (int w = 1; w < NW; ++w) {  // column ranges ascend with w
          const float4 e = red4[w * ROWS + row];
          if (e.x > t.x) { t.y = fmaxf(t.x, e.y); t.x = e.x; t.z = e.z; }
          else t.y = fmaxf(t.y, e.x);
        }
        if (row_base + row < B) top2[(size_t)(row_base + row) * ngroups + bx] = t;
      }
    }
  } else {  // EPI_SWIGLU
    float* swap = reinterpret_cast<float*>(lds) + (size_t)(wt >> 1) * MT * 16 * 64;
    if (writer && (wt & 1)) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) swap[(mt * 16 + r) * 64 + lane] = acc[mt][r] * out_scale;
    }
    __syncthreads();
    if (writer && !(wt & 1)) {
      T* hq = reinterpret_cast<T*>(out);
      const int col = (tile >> 1) * 32 + (lane & 31);
      // position of column `col` in a row of TERMS terms (two terms: groups of eight hi values, then their lo values)
      const size_t cpos = TERMS == 1 ? (size_t)col : (size_t)(col >> 3) * 16 + (col & 7);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const float g = acc[mt][r] * out_scale, u = swap[(mt * 16 + r) * 64 + lane];
          float hval = g / (1.0f + __expf(-g)) * u;
          if (F16 && fabsf(hval) > 65504.0f) {  // beyond fp16: clamp, and say so (GOOSE_FLAG_RANGE)
            hval = copysignf(65504.0f, hval);
            if (flags != nullptr && row < B) atomicOr(flags, GOOSE_FLAG_RANGE);
          }
          if (row < B) {
            const T hi = (T)hval;
            hq[(size_t)row * ldo + cpos] = hi;
            if (TERMS == 2) hq[(size_t)row * ldo + cpos + 8] = (T)(hval - (float)hi);
          }
        }
    }
  }
}

struct GemmCall {
  const void* A; int lda; const void* Wp; int Npad, Kpad, B, ksplit; void* out; size_t ldo, split_stride;
  hipStream_t st; void* top2; int n_valid; bool f16; int terms; float out_scale; int32_t* flags;
};

template <int MT, int NW, int TERMS, int EPI, bool CHUNKED, bool F16>
int launch_k(const GemmCall& g, dim3 grid, int gx, int gps, int nchunk) {
  hipLaunchKernelGGL((k_gemm_bf16<MT, NW, TERMS, EPI, CHUNKED, F16>), grid, dim3(64 * NW), 0, g.st,
                     (const typename Mma16<F16>::T*)g.A, g.lda, (const u32x4*)g.Wp, g.Npad / 32, g.Kpad / 16, gps, g.B,
                     g.out, g.ldo, g.split_stride, (float4*)g.top2, g.n_valid, gx, g.ksplit, nchunk, g.out_scale, g.flags);
  return goose_launch_status();
}

template <int MT, int NW, int EPI, bool CHUNKED>
int launch_terms(const GemmCall& g, dim3 grid, int gx, int gps, int nchunk) {
  if (g.terms == 2)
    return g.f16 ? launch_k<MT, NW, 2, EPI, CHUNKED, true>(g, grid, gx, gps, nchunk)
                 : launch_k<MT, NW, 2, EPI, CHUNKED, false>(g, grid, gx, gps, nchunk);
  return g.f16 ? launch_k<MT, NW, 1, EPI, CHUNKED, true>(g, grid, gx, gps, nchunk)
               : launch_k<MT, NW, 1, EPI, CHUNKED, false>(g, grid, gx, gps, nchunk);
}

template <int MT, int NW, int EPI>
int launch_one(const GemmCall& g) {
  const int ntiles = g.Npad / 32;
  const int gx = (ntiles + NW - 1) / NW;
  const int nchunk = (g.B + MT * 32 - 1) / (MT * 32);  // more than 128 rows: chunks of 4 row tiles
  const dim3 grid = nchunk == 1 ? dim3(gx, g.ksplit) : dim3((gx * g.ksplit + 7) / 8 * 8 * nchunk);
  const int granules = g.Kpad / KGRAN;                      // split-K ranges are multiples of 128 inputs
  const int gps = (granules + g.ksplit - 1) / g.ksplit;     // granules (= stages) per split
  if constexpr (MT == 4) {
    if (nchunk > 1) return launch_terms<MT, NW, EPI, true>(g, grid, gx, gps, nchunk);
  }
  return launch_terms<MT, NW, EPI, false>(g, grid, gx, gps, nchunk);
}

template <int NW, int EPI>
int launch_mt(int MT, const GemmCall& g) {
  switch (MT) {
    case 1: return launch_one<1, NW, EPI>(g);
    case 2: return launch_one<2, NW, EPI>(g);
    case 3: return launch_one<3, NW, EPI>(g);
    case 4: return launch_one<4, NW, EPI>(g);
  }
  return GOOSE_ERR_ARG;
}

}  // namespace

int launch_pack_16(int mode, const void* s0, const void* s1, const void* s2, int rows_each, int K, int Npad,
                     int Kpad, void* dst, hipStream_t st, int rows_kv, int cvt_exp, int32_t* flags) {
  if (rows_kv <= 0) rows_kv = rows_each;
  const size_t total = (size_t)(Npad / 32) * (Kpad / 16) * 64;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(k_pack_bf16, dim3(blocks), dim3(256), 0, st, mode, (const bf16_t*)s0, (const bf16_t*)s1,
                     (const bf16_t*)s2, rows_each, rows_kv, K, Kpad / 16, total, (uint4*)dst, cvt_exp, flags);
  return goose_launch_status();
}

// Workgroup width (wavefronts = column tiles per workgroup) and split-K factor for a shape.
// Measured on MI355X: the stream wants about 768 wavefronts in flight; every extra split costs an
// fp32 tile written and re-read (and flushed at the kernel boundary), so take the smallest power of
// two that reaches it, with every split at least 4 stages long; the 4-wide workgroup (more sharing
// of the staged A block) whenever it leaves enough workgroups.
void pick_gemm_config(int Npad, int Kpad, int max_ksplit, int* nw_out, int* ksplit_out) {
  const int ntiles = Npad / 32, nstages = Kpad / KGRAN;
  const int want = (768 + ntiles - 1) / ntiles;
  int ks = 1;
  while (ks < want) ks *= 2;
  while (ks > 1 && (ks > nstages / 4 || ks > max_ksplit)) ks /= 2;
  while (ks > 1 && ((nstages + ks - 1) / ks) * (ks - 1) >= nstages) --ks;  // no empty split
  *nw_out = (((ntiles + 3) / 4) * ks >= 160) ? 4 : 2;
  *ksplit_out = ks;
}

static bool dtype16(int dtype, bool* f16) {
  *f16 = dtype == GOOSE_DTYPE_F16;
  return dtype == GOOSE_DTYPE_BF16 || dtype == GOOSE_DTYPE_F16;
}

int launch_gemm_top2_16(int dtype, const void* A, int lda, int terms, const void* Wp, int Npad, int Kpad, int B, int nw,
                        float* out, size_t ldo, void* top2, int n_valid, float out_scale, hipStream_t st) {
  bool f16;
  if (!dtype16(dtype, &f16)) return GOOSE_ERR_ARG;
  if (B < 1 || B > GOOSE_MAX_ROWS || (Npad & 31) || (Kpad % KGRAN) || !top2 || n_valid < 1 || n_valid > Npad)
    return GOOSE_ERR_ARG;
  if ((terms != 1 && terms != 2) || lda < Kpad * terms || (lda & 7)) return GOOSE_ERR_ARG;
  const int MT = B > 128 ? 4 : (B + 31) / 32;
  const GemmCall g{A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, st, top2, n_valid, f16, terms, out_scale, nullptr};
  return nw == 4 ? launch_mt<4, EPI_TOP2>(MT, g) : launch_mt<2, EPI_TOP2>(MT, g);
}

int launch_gemm_16(int dtype, int epi, const void* A, int lda, int terms, const void* Wp, int Npad, int Kpad, int B,
                   int nw, int ksplit, void* out, size_t ldo, size_t out_split_stride, float out_scale, int32_t* flags,
                   hipStream_t st) {
  bool f16;
  if (!dtype16(dtype, &f16)) return GOOSE_ERR_ARG;
  if (B < 1 || B > GOOSE_MAX_ROWS || (Npad & 31) || (Kpad % KGRAN) || ksplit < 1) return GOOSE_ERR_ARG;
  if ((terms != 1 && terms != 2) || lda < Kpad * terms || (lda & 7)) return GOOSE_ERR_ARG;
  if (epi != EPI_PARTIAL && epi != EPI_SWIGLU) return GOOSE_ERR_ARG;
  if (epi == EPI_SWIGLU && (ksplit != 1 || (Npad & 63))) return GOOSE_ERR_ARG;
  if (B > 128)  // the kernel blocked for the matrix cores
    return launch_gemm_rows_16(dtype, epi, A, lda, terms, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, out_scale,
                               flags, st);
  const int MT = (B + 31) / 32;
  if (epi == EPI_SWIGLU) {
    const GemmCall g{A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, st, nullptr, 0, f16, terms, out_scale, flags};
    return nw == 4 ? launch_mt<4, EPI_SWIGLU>(MT, g) : launch_mt<2, EPI_SWIGLU>(MT, g);
  }
  const GemmCall g{A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, st, nullptr, 0, f16, terms, out_scale, flags};
  return nw == 4 ? launch_mt<4, EPI_PARTIAL>(MT, g) : launch_mt<2, EPI_PARTIAL>(MT, g);
}
