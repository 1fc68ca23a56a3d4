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
//   PACK_GATE_UP : blocks of 16 rows alternate gate (s0) / up (s1): block b -> (b&1 ? up : gate) rows (b>>1)*16..,
//                  so that every 32-row tile holds the gate rows AND the up rows of its 16 output columns
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
    const int blk = n >> 4;
    row = (blk >> 1) * 16 + (n & 15);
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
// EPI_SWIGLU: every tile holds the gate rows (columns 0-15 of the tile) and the up rows (columns
// 16-31) of 16 outputs, so a wavefront forms h = silu(gate) * up (in TERMS terms) from its own
// accumulators.  Tiles (of EPI_SWIGLU and EPI_PARTIAL) are dealt to the wavefronts with a stride of
// the grid width (wavefront w of workgroup g takes tile g + w * gridDim.x), and the grid is as wide
// as the chip when the tiles allow: 688 tiles then load 256 compute units with at most three weight streams each instead of
// 172 with four.
// EPI_TOP2: besides the optional plain output, every workgroup reduces its columns to one
// (largest, second largest, index of largest) triple per row, for the greedy argmax.
// CHUNKED: more than MT*32 rows, computed as several row chunks that read the same weights (1-D
// grid in an XCD-aware order, ordinary loads so that the chunks share the L2); otherwise the
// weights are read once by the whole grid, with non-temporal loads that keep them from displacing
// the L2's other lines.  F16: fp16 instead of bf16 operands (and SwiGLU output).
// word 3 of a raw buffer descriptor on this target (32-bit untyped data, range checking on the byte offset)
#define GOOSE_BUFFER_WORD3 0x00020000
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
  // copy instructions per wavefront per stage: the same number for every wavefront (the wait counts
  // below are immediates); where the copies do not divide evenly the last ones are issued twice
  constexpr int CPW = (COPIES + NWAVES - 1) / NWAVES;
  // SwiGLU: every wavefront passes its accumulators through LDS as fp32
  constexpr int SWAP_BYTES = (EPI == EPI_SWIGLU) ? NW * MT * 16 * 64 * 4 : 0;
  constexpr int CT_ROW = 33;  // floats per row of a transposed-read C tile (odd: conflict-free row scans)
  constexpr int TOP2_BYTES = (EPI == EPI_TOP2) ? NW * MT * 32 * (CT_ROW * 4 + 16) : 0;
  constexpr int EPI_BYTES = SWAP_BYTES > TOP2_BYTES ? SWAP_BYTES : TOP2_BYTES;
  constexpr int TAIL_BYTES = EPI_BYTES;
  // Ring depth D: every wavefront keeps D stages of its weight pieces in flight in registers and the
  // workgroup D stages of A in LDS.
#ifndef GOOSE_RING_MAX
#define GOOSE_RING_MAX 2
#endif
  constexpr int LDS_BUDGET = 144 * 1024;
  constexpr int D_FIT = (LDS_BUDGET - (TAIL_BYTES > STAGE_BYTES ? TAIL_BYTES - STAGE_BYTES : 0)) / STAGE_BYTES;
  constexpr int D = D_FIT >= GOOSE_RING_MAX ? GOOSE_RING_MAX : (D_FIT < 2 ? 2 : D_FIT);
  static_assert(D >= 2 && D <= 4, "ring depth");
  // The buffers are separate arrays: the compiler then knows that the copy into one does not touch
  // what is read from another (with one array it makes every operand read wait for the copy just
  // issued, i.e. for all loads in flight).  The epilogues reuse the first.
  constexpr int LDS0_BYTES = STAGE_BYTES > TAIL_BYTES ? STAGE_BYTES : TAIL_BYTES;
  static_assert(LDS0_BYTES + (D - 1) * STAGE_BYTES <= 160 * 1024, "LDS of one compute unit");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS0_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char lds1[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char lds2[D > 2 ? STAGE_BYTES : 16];
  __shared__ __attribute__((aligned(1024))) unsigned char lds3[D > 3 ? STAGE_BYTES : 16];
  auto lds_buf = [&](auto buf_c) -> unsigned char* {
    constexpr int b = decltype(buf_c)::value;
    return b == 0 ? lds : (b == 1 ? lds1 : (b == 2 ? lds2 : lds3));
  };
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // (in a scalar register: it selects buffer descriptors)
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
  const int tile = EPI == EPI_TOP2 ? bx * NW + wt : bx + ngroups * wt;
  const bool active = tile < ntiles;
  // a wavefront without a tile runs the same pipeline (no divergent control flow: the compiler can
  // then count outstanding loads exactly) on an empty weight range, i.e. on zeros that cost no
  // memory traffic, and skips the store
  const int tile_ld = active ? tile : 0;
  const int nstages_total = ksteps_total / STEPS;
  const int s_begin = by * stages_per_split;
  const int s_end = min(s_begin + stages_per_split, nstages_total);
  const int nst = s_end - s_begin;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  // Code that runs once per workgroup is fetched from memory at a few tens of nanoseconds per 64
  // bytes (the instruction cache starts every launch cold), which at these launch lengths costs as
  // much as the data.  So there is ONE loop body for every stage -- no separate prologue, tail or
  // short-range variants: loads that fall outside the K range are issued all the same and made
  // harmless.  The weights are read through a buffer descriptor that covers exactly this
  // wavefront's pieces of its K range: a load beyond it returns zeros without touching memory; the A
  // copy of a stage beyond the range re-reads the last stage (it meets zero weights).  The stages
  // computed are rounded up to a multiple of D.
  // ---- this wavefront's share of the A copy: copy instruction c of the stage fills rows
  // c*ROWS_PER_COPY ..; lane i fetches the unit that belongs at position i % SU of row i / SU
  // (swizzled, see above)
  const u32x4* a_src[CPW];
  const int row_units = lda >> 3;  // 16-byte units per operand row
#pragma unroll
  for (int q = 0; q < CPW; ++q) {
    const int c = min(wave * CPW + q, COPIES - 1);
    const int row = c * ROWS_PER_COPY + lane / SU, pos = lane % SU;
    const int unit = (pos & ~15) | ((pos ^ row) & 15);
    a_src[q] = reinterpret_cast<const u32x4*>(A) + (size_t)(row_base + row) * row_units +
               (size_t)s_begin * SU + unit;
  }
  auto copy_a = [&](int i, auto buf_c) {  // stage i -> LDS buffer buf
    const int ic = min(i, nst - 1);
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
      const int c = min(wave * CPW + q, COPIES - 1);  // (wavefront-uniform)
      unsigned char* dst = lds_buf(buf_c) + c * 1024;
#if defined(__HIP_DEVICE_COMPILE__)  // (the host pass knows no such builtin and would silently drop the kernel's stub)
      __builtin_amdgcn_global_load_lds(a_src[q] + (size_t)ic * SU, GOOSE_LDS_PTR(dst), 16, 0, 0);
#else
      (void)dst;
#endif
    }
  };
  u32x4 wreg[D][STEPS];
#if defined(__HIP_DEVICE_COMPILE__)
  const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<u32x4*>(Wp + ((size_t)tile_ld * ksteps_total + (size_t)s_begin * STEPS) * 64), 0,
      (active && nst > 0 ? nst : 0) * STEPS * 1024, GOOSE_BUFFER_WORD3);
#endif
  const int w_lane = lane * 16;
  auto load_w = [&](int i, auto slot_c) {  // (beyond the range: zeros, no memory traffic)
    constexpr int slot = decltype(slot_c)::value;
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int s = 0; s < STEPS; ++s)
      wreg[slot][s] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, w_lane, (i * STEPS + s) * 1024, STREAM ? 2 : 0);
#endif
  };
  // operand reads: lane l holds row l % 32 (of row tile mt) and the eight inputs 8*(l/32).. of a k-step
  const int a_row = (lane & 31) * ROW_BYTES, a_x = lane & 15, a_hh = lane >> 5;
  auto barrier = [&]() {  // (raw: __syncthreads would also drain every load in flight)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  // Loads complete in order as far as the wait counter goes.  Stage j issues, in this order, the A copy
  // of stage j+D-1 (into the buffer whose readers passed the barrier that ended stage j-1) and, one
  // after each k-step's matrix instructions, the refills of its own register slot with the weights
  // of stage j+D.  Before the barrier that ends stage j the A copy of stage j+1 must have landed; the
  // STEADY_WAIT loads issued after that copy may stay in flight.
  constexpr int STEADY_WAIT = (D - 2) * (STEPS + CPW) + STEPS;
  static_assert(STEADY_WAIT <= 63, "wait counter");
  // The operand reads of a k-step are issued PD k-steps ahead of the matrix instructions that use
  // them (a compute unit runs one wavefront per SIMD here, so nothing else hides the LDS latency).
  constexpr int MPS = MT * TERMS;                                   // matrix instructions per k-step
  constexpr int PD = MPS >= 4 ? 1 : (MPS >= 2 ? 2 : 4), NB = PD + 1;
  // one stage (slot = i % D, compile-time so that no register array is indexed dynamically; the
  // LDS buffer goes with it)
  auto stage = [&](auto slot_c, int i) {
    constexpr int slot = decltype(slot_c)::value;
    const unsigned char* abuf = lds_buf(slot_c);
    copy_a(i + D - 1, std::integral_constant<int, (slot + D - 1) % D>());
    __builtin_amdgcn_sched_barrier(0);   // keep the issue order: the scheduler would sink these loads
    op8 af[NB][TERMS][MT];
    auto read_a = [&](int s, op8 (&dst)[TERMS][MT]) {
#pragma unroll
      for (int t = 0; t < TERMS; ++t) {
        const int unit = (2 * s + a_hh) * TERMS + t;
        const int pos = (unit & ~15) | ((unit ^ a_x) & 15);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          dst[t][mt] = *reinterpret_cast<const op8*>(&abuf[mt * 32 * ROW_BYTES + a_row + pos * 16]);
      }
    };
#pragma unroll
    for (int s = 0; s < PD; ++s) read_a(s, af[s % NB]);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (s + PD < STEPS) read_a(s + PD, af[(s + PD) % NB]);
      const op8 b = __builtin_bit_cast(op8, wreg[slot][s]);
      // (terms outside, row tiles inside: consecutive matrix instructions then go to different
      // accumulators instead of waiting for each other; every accumulator still takes hi before lo)
#pragma unroll
      for (int t = 0; t < TERMS; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = Mma16<F16>::mfma(af[s % NB][t][mt], b, acc[mt]);
#if defined(__HIP_DEVICE_COMPILE__)
      wreg[slot][s] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, w_lane, ((i + D) * STEPS + s) * 1024, STREAM ? 2 : 0);
#endif
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(STEADY_WAIT));
    barrier();
  };
  const std::integral_constant<int, 0> c0;
  const std::integral_constant<int, 1> c1;
  const std::integral_constant<int, 2> c2;
  const std::integral_constant<int, 3> c3;

  if (nst > 0) {
    // the ring is filled in the order the stages themselves would have issued these loads, so that
    // one wait count fits the whole loop
    load_w(0, c0);
    copy_a(0, c0);
    load_w(1, c1);
    if constexpr (D > 2) { copy_a(1, c1); load_w(2, c2); }
    if constexpr (D > 3) { copy_a(2, c2); load_w(3, c3); }
    // stage 0 of both streams has arrived, later stages are in flight: the state every stage
    // starts from.  (The compiler counts the copies to LDS and the register loads as two kinds that
    // may overtake each other, and falls back to waiting for ALL loads wherever it has to wait for
    // one with both kinds pending; so the waits are placed here and before each barrier by hand, and
    // inside a stage everything it consumes is known to be there.)
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(STEADY_WAIT));
    barrier();
    for (int i = 0; i < nst; i += D) {
      stage(c0, i);
      stage(c1, i + 1);
      if constexpr (D > 2) stage(c2, i + 2);
      if constexpr (D > 3) stage(c3, i + 3);
    }
    // the copies issued by the last stages still target the LDS buffers that the epilogues reuse
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    barrier();
  }
  const bool writer = active;

  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  if (EPI == EPI_PARTIAL) {
    if (!writer) return;
    // through a buffer descriptor over rows [0, B) of this split's slab: stores to rows >= B fall
    // outside it and are dropped, so no store needs a branch or an address computation of its own
    const int col = tile * 32 + (lane & 31);
#if defined(__HIP_DEVICE_COMPILE__)
    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<float*>(out) + by * split_stride, 0, (int)((size_t)B * ldo * 4), GOOSE_BUFFER_WORD3);
    const int ldo4 = (int)ldo * 4;
    const int voff = (row_base + 4 * (lane >> 5)) * ldo4 + col * 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, acc[mt][r] * out_scale), orsrc, voff,
                                              (mt * 32 + 8 * (r >> 2) + (r & 3)) * ldo4, 0);
#endif
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
    // The wavefront leaves its accumulators in LDS (register r of lane l at [r][l]) and walks its
    // tile's 16 output columns two at a time in a short loop (compact code; the 16-bit results leave
    // as 4-byte stores): the gate values of columns 2p, 2p+1 sit at lanes 2p, 2p+1 of a half, the up
    // values 16 lanes further.  Nothing is shared between wavefronts: no barrier.
    constexpr int TILE_F = MT * 16 * 64;  // floats of one wavefront's accumulators
    float* mine = reinterpret_cast<float*>(lds) + (size_t)wt * TILE_F;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mine[(mt * 16 + r) * 64 + lane] = acc[mt][r] * out_scale;
    __builtin_amdgcn_wave_barrier();  // (LDS operations of one wavefront complete in order)
    if (writer) {
      T* hq = reinterpret_cast<T*>(out);
      bool clamped = false;
      for (int e = lane; e < MT * 16 * 16; e += 64) {
        const int pr = e & 7, half = (e >> 3) & 1, rr = (e >> 4) & 15, mt = e >> 8;  // column pair, lane half, register, row tile
        const int row = row_base + mt * 32 + 8 * (rr >> 2) + 4 * half + (rr & 3);
        const int col = tile * 16 + 2 * pr;
        const float* src = &mine[(mt * 16 + rr) * 64 + half * 32 + 2 * pr];
        const float2 g = *reinterpret_cast<const float2*>(src);
        const float2 u = *reinterpret_cast<const float2*>(src + 16);
        float h0 = swiglu_f32(g.x, u.x), h1 = swiglu_f32(g.y, u.y);
        if (F16) {  // beyond fp16: clamp, and say so (GOOSE_FLAG_RANGE)
          if (fabsf(h0) > 65504.0f) { h0 = copysignf(65504.0f, h0); clamped = clamped || row < B; }
          if (fabsf(h1) > 65504.0f) { h1 = copysignf(65504.0f, h1); clamped = clamped || row < B; }
        }
        if (row < B) {
          // position of column `col` in a row of TERMS terms (two terms: groups of eight hi values, then their lo values)
          const size_t cpos = TERMS == 1 ? (size_t)col : (size_t)(col >> 3) * 16 + (col & 7);
          const T a0 = (T)h0, a1 = (T)h1;
          T* dst = hq + (size_t)row * ldo + cpos;
          union { T t[2]; unsigned u; } pk;
          pk.t[0] = a0; pk.t[1] = a1;
          *reinterpret_cast<unsigned*>(dst) = pk.u;
          if (TERMS == 2) {
            pk.t[0] = (T)(h0 - (float)a0); pk.t[1] = (T)(h1 - (float)a1);
            *reinterpret_cast<unsigned*>(dst + 8) = pk.u;
          }
        }
      }
      if (F16 && clamped && flags != nullptr) atomicOr(flags, GOOSE_FLAG_RANGE);
    }
  }
}

struct GemmCall {
  const void* A; int lda; const void* Wp; int Npad, Kpad, B, ksplit; void* out; size_t ldo, split_stride;
  hipStream_t st; void* top2; int n_valid; bool f16; int terms; float out_scale; int32_t* flags;
  int gx = 0;  // grid width in workgroups per K range (0: chosen by launch_one)
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
  int gx = (ntiles + NW - 1) / NW;
  // SwiGLU tiles stand alone and are dealt with a stride of the grid width: a grid as wide as the
  // chip (or as the tiles allow) spreads the weight streams over more compute units
  if (g.gx > 0) gx = g.gx;
  else if (EPI == EPI_SWIGLU && gx < 256) gx = ntiles < 256 ? ntiles : 256;
  // the same for the split-K products: tiles of one K range are dealt with a stride of the grid width,
  // and the grid is widened until all ranges together fill the chip
  if (g.gx == 0 && EPI == EPI_PARTIAL && gx * g.ksplit < 256) {
    const int want = (256 + g.ksplit - 1) / g.ksplit;
    gx = want < ntiles ? (want > gx ? want : gx) : ntiles;
  }
  const int nchunk = (g.B + MT * 32 - 1) / (MT * 32);  // more than 128 rows: chunks of 4 row tiles
  const dim3 grid = nchunk == 1 ? dim3(gx, g.ksplit) : dim3((gx * g.ksplit + 7) / 8 * 8 * nchunk);
  const int granules = g.Kpad / KGRAN;                      // split-K ranges are multiples of 128 inputs
  const int gps = (granules + g.ksplit - 1) / g.ksplit;     // granules (= stages) per split
  if constexpr (MT == 4) {
    if (nchunk > 1) return launch_terms<MT, NW, EPI, true>(g, grid, gx, gps, nchunk);
  }
  return launch_terms<MT, NW, EPI, false>(g, grid, gx, gps, nchunk);
}

// five-wavefront workgroups (single row chunk only): see launch_gemm_16
template <int MT, int EPI>
int launch_five(const GemmCall& g) {
  const int granules = g.Kpad / KGRAN;
  const int gps = (granules + g.ksplit - 1) / g.ksplit;
  return launch_terms<MT, 5, EPI, false>(g, dim3(g.gx, g.ksplit), g.gx, gps, 1);
}
template <int EPI>
int launch_mt5(int MT, const GemmCall& g) {
  switch (MT) {
    case 1: return launch_five<1, EPI>(g);
    case 2: return launch_five<2, EPI>(g);
    case 3: return launch_five<3, EPI>(g);
    case 4: return launch_five<4, EPI>(g);
  }
  return GOOSE_ERR_ARG;
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

// Workgroup width (wavefronts = column tiles per workgroup) and split-K factor for a shape, for a
// context whose passes have up to max_rows rows (a property of the context, not of the call: the
// split decides the order of the sums, and a request must get the same bits at any batch size).
// Measured on MI355X: the stream wants 160 or more four-wavefront workgroups; every extra split
// costs an fp32 tile written and re-read by the residual kernel, which is bound by how fast 64-128
// workgroups can pull those slices.  So: the smallest power of two of splits that reaches the
// workgroup count, every split at least 4 stages long.  With at most two row tiles (64 rows) half
// the splits of two-wavefront workgroups stream as fast when that still gives 256 workgroups (the
// 7B O and down projections: 4 splits instead of 8, and a microsecond less in each residual
// kernel); with more rows the narrower workgroup's extra copies of the A block cost more than that.
void pick_gemm_config(int Npad, int Kpad, int max_ksplit, int max_rows, int* nw_out, int* ksplit_out) {
  const int ntiles = Npad / 32, nstages = Kpad / KGRAN;
  const int groups4 = (ntiles + 3) / 4, groups2 = (ntiles + 1) / 2;
  auto allowed = [&](int ks) {
    return ks == 1 || (ks <= nstages / 4 && ks <= max_ksplit && ((nstages + ks - 1) / ks) * (ks - 1) < nstages);
  };
  int ks = 1;
  while (groups4 * ks < 160 && allowed(ks * 2)) ks *= 2;
  int nw = groups4 * ks >= 160 ? 4 : 2;
  if (nw == 4 && ks >= 2 && max_rows <= 64 && groups2 * (ks / 2) >= 256) {
    ks /= 2;
    nw = 2;
  }
  *nw_out = nw;
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
  // More four-tile workgroups than compute units would run as one round plus a few stragglers (or
  // with some units loaded twice, which then take twice as long: a unit pulls only so many bytes
  // per microsecond).  Where five tiles per workgroup fit all tiles into one round of at most 256
  // workgroups, take those: 33B gate/up, 1120 tiles = 256 workgroups of five wavefronts.
  const int ntiles = Npad / 32;
  const int gx5 = 256 / ksplit;
  const bool five = nw == 4 && ((ntiles + 3) / 4) * ksplit > 256 && gx5 * 5 >= ntiles;
  if (epi == EPI_SWIGLU) {
    GemmCall g{A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, st, nullptr, 0, f16, terms, out_scale, flags};
    if (five) { g.gx = gx5; return launch_mt5<EPI_SWIGLU>(MT, g); }
    return nw == 4 ? launch_mt<4, EPI_SWIGLU>(MT, g) : launch_mt<2, EPI_SWIGLU>(MT, g);
  }
  GemmCall g{A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, st, nullptr, 0, f16, terms, out_scale, flags};
  if (five) { g.gx = gx5; return launch_mt5<EPI_PARTIAL>(MT, g); }
  return nw == 4 ? launch_mt<4, EPI_PARTIAL>(MT, g) : launch_mt<2, EPI_PARTIAL>(MT, g);
}
