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
__global__ __launch_bounds__(256) void k_pack_bf16(int mode, const bf16_t* __restrict__ s0,
                                                   const bf16_t* __restrict__ s1, const bf16_t* __restrict__ s2,
                                                   int rows_each, int rows_kv, int K, int ktiles, size_t total,
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
  union { uint4 u; bf16_t e[8]; } v;
  v.u = make_uint4(0, 0, 0, 0);
  if (src != nullptr && row < limit) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (k0 + e < K) v.e[e] = src[(size_t)row * K + k0 + e];
  }
  dst[idx] = v.u;
}

// ------------------------------------------------------------------------------------------
// One workgroup = NW wavefronts, wavefront w owns column tile blockIdx.x*NW + w (32 columns) and
// all MT row tiles.  blockIdx.y selects the split-K range.  Per stage (KC = 128 inputs; a 256-wide
// stage, half as many barriers, measured no faster):
//   - every wavefront keeps RING stages of its own weight pieces (8 KiB each) and of its share of
//     the A copy in flight in registers,
//   - the workgroup publishes the next A stage registers -> LDS (LDS double buffer),
//   - one barrier.
// Measured with parts compiled out: the matrix instructions, the LDS reads and the barriers cost
// nothing; the A copy costs about 5 us of the gate/up projection and about 1 us of the others;
// the rest is the weight stream itself plus the fixed cost of a dependent launch.
// EPI_SWIGLU: even wavefronts hold gate tiles, odd ones the matching up tiles; the up tile
// is handed over through LDS and the even wavefront writes h = silu(gate) * up.
// EPI_TOP2: besides the optional plain output, every workgroup reduces its columns to one
// (largest, second largest, index of largest) triple per row, for the greedy argmax.
// CHUNKED: more than MT*32 rows, computed as several row chunks that read the same weights (1-D
// grid in an XCD-aware order, ordinary loads so that the chunks share the L2); otherwise the
// weights are read once by the whole grid, with non-temporal loads that keep them from displacing
// the L2's other lines.  F16: fp16 instead of bf16 operands (and SwiGLU output).
template <int MT, int NW, int EPI, int KC, int RING, bool CHUNKED = false, bool F16 = false>
__global__ __launch_bounds__(64 * NW) void k_gemm_bf16(const typename Mma16<F16>::T* __restrict__ A, int lda,
                                                       const u32x4* __restrict__ Wp, int ntiles, int ksteps_total,
                                                       int stages_per_split, int B, void* __restrict__ out,
                                                       size_t ldo, size_t split_stride,
                                                       float4* __restrict__ top2, int n_valid, int gx, int nsplit,
                                                       int nchunk) {
  typedef typename Mma16<F16>::T T;
  typedef typename Mma16<F16>::v8 op8;
  constexpr int LDS_ROW = KC * 2 + 16;  // bytes; the 16-byte pad staggers rows across banks
  constexpr int NTHR = 64 * NW;
  constexpr int STEPS = KC / 16;                    // MFMA k-steps per stage
  constexpr int ASEG = MT * 32 * (KC / 8);           // 16-byte segments of one A stage
  constexpr int APT = ASEG / NTHR;                   // segments per thread
  static_assert(ASEG % NTHR == 0, "A stage must divide evenly over the workgroup");
  constexpr int STAGE_BYTES = MT * 32 * LDS_ROW;
  constexpr int SWAP_BYTES = (EPI == EPI_SWIGLU) ? (NW / 2) * MT * 16 * 64 * 4 : 0;
  constexpr int CT_ROW = 33;  // floats per row of a transposed-read C tile (odd: conflict-free row scans)
  constexpr int TOP2_BYTES = (EPI == EPI_TOP2) ? NW * MT * 32 * (CT_ROW * 4 + 16) : 0;
  constexpr int EPI_BYTES = SWAP_BYTES > TOP2_BYTES ? SWAP_BYTES : TOP2_BYTES;
  constexpr int LDS_BYTES = 2 * STAGE_BYTES > EPI_BYTES ? 2 * STAGE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
    A += (size_t)row_base * lda;
    ngroups = gx;
  }
  const int tile = bx * NW + wave;
  const bool active = tile < ntiles;
  // a wavefront past the last tile redoes the last tile (no divergent control flow in the
  // pipeline, which lets the compiler count outstanding loads exactly) and skips the store
  const int tile_ld = active ? tile : ntiles - 1;
  const int nstages_total = ksteps_total / STEPS;
  const int s_begin = by * stages_per_split;
  const int s_end = min(s_begin + stages_per_split, nstages_total);
  const int nst = s_end - s_begin;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

  // Both operand streams run RING stages ahead in registers.  Memory operations complete in
  // order as far as the wait counter is concerned, so a value can only be awaited together with
  // everything issued before it: whatever is consumed soon must not have been issued after
  // loads that are meant to stay in flight.  Hence stage st issues the A copy of stage st+RING
  // and the weight pieces of stage st+RING (into the slots stage st just freed) and consumes only
  // what was issued RING stages ago; RING * (8 + APT) loads per wavefront stay outstanding.
  static_assert(RING == 2 || RING == 4, "ring depth");
  u32x4 areg[RING][APT];
  const T* a_src[APT];
  int a_dst[APT];
#pragma unroll
  for (int i = 0; i < APT; ++i) {
    const int seg = tid + NTHR * i;
    const int row = seg / (KC / 8), c16 = seg % (KC / 8);
    a_src[i] = A + (size_t)row * lda + c16 * 8;
    a_dst[i] = row * LDS_ROW + c16 * 16;
  }
  u32x4 wreg[RING][STEPS];
  const u32x4* wbase = Wp + (size_t)tile_ld * ksteps_total * 64 + lane;
  auto load_a = [&](int st, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int i = 0; i < APT; ++i) areg[slot][i] = *reinterpret_cast<const u32x4*>(a_src[i] + (size_t)st * KC);
  };
  auto store_a = [&](int buf, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
#pragma unroll
    for (int i = 0; i < APT; ++i) *reinterpret_cast<u32x4*>(&lds[buf * STAGE_BYTES + a_dst[i]]) = areg[slot][i];
  };
  auto load_w = [&](int st, auto slot_c) {
    constexpr int slot = decltype(slot_c)::value;
    const u32x4* p = wbase + (size_t)st * STEPS * 64;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) wreg[slot][s] = STREAM ? __builtin_nontemporal_load(p + s * 64) : p[s * 64];
  };
  const int a_frag = (lane & 31) * LDS_ROW + (lane >> 5) * 16;
  // one stage (slot = st % RING, compile-time so that no register array is indexed dynamically;
  // the LDS buffer alternates with the stage's parity)
  auto stage = [&](auto slot_c, int st, auto next_a, auto refill) {
    constexpr int slot = decltype(slot_c)::value, buf = slot & 1;
    const std::integral_constant<int, (slot + 1) % RING> nslot;
    if (refill) load_a(st + RING, slot_c);  // this slot's previous content (stage st) is in LDS already
    __builtin_amdgcn_sched_barrier(0);      // keep the issue order: the scheduler would sink these loads
    const u32x4* pn = wbase + (size_t)(st + RING) * STEPS * 64;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      const op8 b = __builtin_bit_cast(op8, wreg[slot][s]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const op8 a = *reinterpret_cast<const op8*>(&lds[buf * STAGE_BYTES + mt * 32 * LDS_ROW + a_frag + s * 32]);
        acc[mt] = Mma16<F16>::mfma(a, b, acc[mt]);
      }
      if (refill) wreg[slot][s] = STREAM ? __builtin_nontemporal_load(pn + s * 64) : pn[s * 64];
      __builtin_amdgcn_sched_barrier(0);
    }
    if (next_a) store_a(buf ^ 1, nslot);
    __syncthreads();
  };
  const std::true_type yes;
  const std::integral_constant<int, 0> c0;
  const std::integral_constant<int, 1> c1;
  const std::integral_constant<int, 2> c2;
  const std::integral_constant<int, 3> c3;

  if (nst > 0) {
    int i = 0;
    if (nst >= 2 * RING) {
      // long range: every slot is filled unconditionally, so that the compiler's wait counts at
      // the loop head are exact (it merges all paths into the loop, and a path with fewer loads
      // in flight would make every iteration drain the ring)
      load_a(s_begin, c0);
      load_w(s_begin, c0);
      load_a(s_begin + 1, c1);
      load_w(s_begin + 1, c1);
      if constexpr (RING == 4) {
        load_a(s_begin + 2, c2);
        load_w(s_begin + 2, c2);
        load_a(s_begin + 3, c3);
        load_w(s_begin + 3, c3);
      }
      store_a(0, c0);
      __syncthreads();
      for (; i + 2 * RING - 1 < nst; i += RING) {  // steady state: no conditionals inside
        stage(c0, s_begin + i, yes, yes);
        stage(c1, s_begin + i + 1, yes, yes);
        if constexpr (RING == 4) {
          stage(c2, s_begin + i + 2, yes, yes);
          stage(c3, s_begin + i + 3, yes, yes);
        }
      }
    } else {
      load_a(s_begin, c0);
      load_w(s_begin, c0);
      if (nst > 1) { load_a(s_begin + 1, c1); load_w(s_begin + 1, c1); }
      if constexpr (RING == 4) {
        if (nst > 2) { load_a(s_begin + 2, c2); load_w(s_begin + 2, c2); }
        if (nst > 3) { load_a(s_begin + 3, c3); load_w(s_begin + 3, c3); }
      }
      store_a(0, c0);
      __syncthreads();
    }
    for (; i < nst; ++i) {  // the last stages (i is a multiple of RING on entry)
      const bool na = (i + 1) < nst, rf = (i + RING) < nst;
      switch (i % RING) {
        case 0: stage(c0, s_begin + i, na, rf); break;
        case 1: stage(c1, s_begin + i, na, rf); break;
        case 2: if constexpr (RING == 4) stage(c2, s_begin + i, na, rf); break;
        default: if constexpr (RING == 4) stage(c3, s_begin + i, na, rf); break;
      }
    }
  }

  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  if (EPI == EPI_PARTIAL) {
    if (!active) return;
    float* o = reinterpret_cast<float*>(out) + by * split_stride;
    const int col = tile * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row_base + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < B) o[(size_t)row * ldo + col] = acc[mt][r];
      }
  } else if (EPI == EPI_TOP2) {  // (the last loop barrier already separates the A stages from this reuse of LDS)
    constexpr int ROWS = MT * 32;
    float* o = reinterpret_cast<float*>(out);
    float* ct = reinterpret_cast<float*>(lds) + wave * ROWS * CT_ROW;
    float4* red = reinterpret_cast<float4*>(lds + NW * ROWS * CT_ROW * 4);
    const int col = tile * 32 + (lane & 31);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (o != nullptr && active && row_base + row < B) o[(size_t)(row_base + row) * ldo + col] = acc[mt][r];
        ct[row * CT_ROW + (lane & 31)] = acc[mt][r];
      }
    __syncthreads();
    // lane = row: scan the tile's 32 columns in ascending order (the lowest index wins a tie)
    for (int row = lane; row < ROWS; row += 64) {
      float v1 = -INFINITY, v2 = -INFINITY;
      int i1 = INT_MAX;
      const int c_end = active ? min(32, n_valid - tile * 32) : 0;
      for (int cc = 0; cc < c_end; ++cc) {
        const float v = ct[row * CT_ROW + cc];
        if (v > v1) { v2 = v1; v1 = v; i1 = tile * 32 + cc; }
        else v2 = fmaxf(v2, v);
      }
      red[wave * ROWS + row] = make_float4(v1, v2, __int_as_float(i1), 0.f);
    }
    __syncthreads();
    if (wave == 0) {
      for (int row = lane; row < ROWS; row += 64) {
        float4 t = red[row];
#pragma unroll
        for (int w = 1; w < NW; ++w) {  // column ranges ascend with w
          const float4 e = red[w * ROWS + row];
          if (e.x > t.x) { t.y = fmaxf(t.x, e.y); t.x = e.x; t.z = e.z; }
          else t.y = fmaxf(t.y, e.x);
        }
        if (row_base + row < B) top2[(size_t)(row_base + row) * ngroups + bx] = t;
      }
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
      T* hq = reinterpret_cast<T*>(out);
      const int col = (tile >> 1) * 32 + (lane & 31);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const float g = acc[mt][r], u = swap[(mt * 16 + r) * 64 + lane];
          if (row < B) hq[(size_t)row * ldo + col] = (T)(g / (1.0f + __expf(-g)) * u);
        }
    }
  }
}

struct GemmCall {
  const void* A; int lda; const void* Wp; int Npad, Kpad, B, ksplit; void* out; size_t ldo, split_stride;
  hipStream_t st; void* top2; int n_valid; bool f16;
};

template <int MT, int NW, int EPI, bool CHUNKED, bool F16>
int launch_k(const GemmCall& g, dim3 grid, int gx, int gps, int nchunk) {
  hipLaunchKernelGGL((k_gemm_bf16<MT, NW, EPI, 128, 2, CHUNKED, F16>), grid, dim3(64 * NW), 0, g.st,
                     (const typename Mma16<F16>::T*)g.A, g.lda, (const u32x4*)g.Wp, g.Npad / 32, g.Kpad / 16, gps, g.B,
                     g.out, g.ldo, g.split_stride, (float4*)g.top2, g.n_valid, gx, g.ksplit, nchunk);
  return goose_launch_status();
}

template <int MT, int NW, int EPI>
int launch_one(const GemmCall& g) {
  const int ntiles = g.Npad / 32;
  const int gx = (ntiles + NW - 1) / NW;
  const int nchunk = (g.B + MT * 32 - 1) / (MT * 32);  // more than 128 rows: chunks of 4 row tiles
  const dim3 grid = nchunk == 1 ? dim3(gx, g.ksplit) : dim3((gx * g.ksplit + 7) / 8 * 8 * nchunk);
  const int granules = g.Kpad / KGRAN;                      // split-K ranges are multiples of 128 inputs
  const int gps = (granules + g.ksplit - 1) / g.ksplit;     // granules (= stages) per split
  // two stages of each stream in flight measured best (four: every projection 2-3 us slower)
  if constexpr (MT == 4) {
    if (nchunk > 1)
      return g.f16 ? launch_k<MT, NW, EPI, true, true>(g, grid, gx, gps, nchunk)
                   : launch_k<MT, NW, EPI, true, false>(g, grid, gx, gps, nchunk);
  }
  return g.f16 ? launch_k<MT, NW, EPI, false, true>(g, grid, gx, gps, nchunk)
               : launch_k<MT, NW, EPI, false, false>(g, grid, gx, gps, nchunk);
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
                     int Kpad, void* dst, hipStream_t st, int rows_kv) {
  if (rows_kv <= 0) rows_kv = rows_each;
  const size_t total = (size_t)(Npad / 32) * (Kpad / 16) * 64;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(k_pack_bf16, dim3(blocks), dim3(256), 0, st, mode, (const bf16_t*)s0, (const bf16_t*)s1,
                     (const bf16_t*)s2, rows_each, rows_kv, K, Kpad / 16, total, (uint4*)dst);
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

int launch_gemm_top2_16(int dtype, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int nw,
                        float* out, size_t ldo, void* top2, int n_valid, hipStream_t st) {
  bool f16;
  if (!dtype16(dtype, &f16)) return GOOSE_ERR_ARG;
  if (B < 1 || B > GOOSE_MAX_ROWS || (Npad & 31) || (Kpad % KGRAN) || !top2 || n_valid < 1 || n_valid > Npad)
    return GOOSE_ERR_ARG;
  const int MT = B > 128 ? 4 : (B + 31) / 32;
  const GemmCall g{A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, st, top2, n_valid, f16};
  return nw == 4 ? launch_mt<4, EPI_TOP2>(MT, g) : launch_mt<2, EPI_TOP2>(MT, g);
}

int launch_gemm_16(int dtype, int epi, const void* A, int lda, const void* Wp, int Npad, int Kpad, int B, int nw,
                   int ksplit, void* out, size_t ldo, size_t out_split_stride, hipStream_t st) {
  bool f16;
  if (!dtype16(dtype, &f16)) return GOOSE_ERR_ARG;
  if (B < 1 || B > GOOSE_MAX_ROWS || (Npad & 31) || (Kpad % KGRAN) || ksplit < 1) return GOOSE_ERR_ARG;
  if (epi != EPI_PARTIAL && epi != EPI_SWIGLU) return GOOSE_ERR_ARG;
  if (epi == EPI_SWIGLU && (ksplit != 1 || (Npad & 63))) return GOOSE_ERR_ARG;
  if (B > 128) {
    // the kernel blocked for the matrix cores; GOOSE_ROWS_KERNEL=0 (tuning aid) keeps the skinny kernel in row chunks
    static const bool rows_kernel = !getenv("GOOSE_ROWS_KERNEL") || atoi(getenv("GOOSE_ROWS_KERNEL")) != 0;
    if (rows_kernel)
      return launch_gemm_rows_16(dtype, epi, A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, st);
  }
  const int MT = B > 128 ? 4 : (B + 31) / 32;
  if (epi == EPI_SWIGLU) {
    const GemmCall g{A, lda, Wp, Npad, Kpad, B, 1, out, ldo, 0, st, nullptr, 0, f16};
    return nw == 4 ? launch_mt<4, EPI_SWIGLU>(MT, g) : launch_mt<2, EPI_SWIGLU>(MT, g);
  }
  const GemmCall g{A, lda, Wp, Npad, Kpad, B, ksplit, out, ldo, out_split_stride, st, nullptr, 0, f16};
  return nw == 4 ? launch_mt<4, EPI_PARTIAL>(MT, g) : launch_mt<2, EPI_PARTIAL>(MT, g);
}
