// Tree-masked attention of the B draft-node queries over the cached prefix plus their own
// ancestors (Sec. 4, tree attention mask), fused with the rotary embedding of q and k and the
// write of the new K/V rows; bf16 or fp16 operands, fp32 softmax, for gfx950.
//
// All B queries of a head share the same keys, so the B nodes are the N dimension of an MFMA and
// every K/V byte fetched from HBM is used B times.  The caches are stored in MFMA OPERAND ORDER
// (see goose.h): a 32-key block of one head is D/16 x 1 KiB of K and D/16 x 1 KiB of V, each
// 1 KiB piece being the 64 lanes x 16 bytes of one operand load.  A wavefront therefore streams
// its key blocks global -> registers -> MFMA with perfectly coalesced loads: no LDS staging, no
// barriers (k_attn_fused).  Trees of more than 64 nodes at head size 128 take k_attn_wide instead,
// which brings every block into LDS once per workgroup: with three or four query tiles the
// per-wavefront loads of the same block are what limits the kernel.
//
// Per 32-key block and 32-query tile:
//     S^T[key][query]  = K . Q^T          (v_mfma_f32_32x32x16_{bf16,f16}, rows = keys)
//     online softmax over keys: each lane owns ONE query (column l%32) and 16 keys, so the
//     running max / sum / rescale are per-lane scalars plus one exchange with the twin lane l^32;
//     O^T[d][query]   += V^T . P^T        (rows = head-dim, columns = the same queries).
// The MFMA row <-> key assignment (sigma, baked into the K block layout) makes the 16 scores a
// lane holds 16 consecutive keys, so the probabilities feed the second MFMA from registers.
//
// Work decomposition: grid = (key splits, heads); a workgroup = NQH query tiles x NG key groups
// of one wavefront each.  The prefix blocks [0, ceil(P/32)) are dealt to splits and groups; the
// LAST split also owns the tree itself: it sums the split-K slices of the k|v projections of the
// B nodes, rotates k, stores both into LDS (for this pass) and into cache slots P+i (for later
// cycles), and attends to them under the ancestor mask.  Every wavefront rotates its own q
// operand from the projection slices (lane-local: the rotation pairs (j, j+d/2) live in the same
// lane).  Groups are merged through LDS; splits write (max, sum, unnormalised O) partials that
// k_attn_merge combines in fixed order (a single split writes the normalised 16-bit rows itself).

#include "goose_internal.h"
#include "mma16.h"

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

constexpr float NEG_BIG = -1e30f;  // finite stand-in for -inf: keeps exp2(m_old - m_new) well defined
constexpr int TAIL_COST = 3;       // a tree block costs the last split about this many prefix blocks

// lane row i of the first MFMA carries key sigma(i) of its block; inverse below
__device__ __host__ inline int sigma_inv(int kk) { return (((kk >> 2) & 3) << 3) | ((kk >> 4) << 2) | (kk & 3); }

// element offset of chunk (s, hh) of key slot g in the operand-ordered K cache of one head
template <int D>
__device__ inline size_t k_chunk_off(int g, int s, int hh) {
  return (((size_t)(g >> 5) * (D / 16) + s) * 64 + sigma_inv(g & 31) + 32 * hh) * 8;
}
// element offset of (slot g, column c) in the operand-ordered V cache of one head
template <int D>
__device__ inline size_t v_elem_off(int g, int c) {
  const int kk = g & 31;
  return ((((size_t)(g >> 5) * (D / 32) + (c >> 5)) * 2 + ((kk >> 3) & 1)) * 64 + (c & 31) + 32 * (kk >> 4)) * 8 +
         (kk & 7);
}

// The attention output feeds the O projection, whose activation type may differ from the caches'
// (fp16 operands over a bf16 cache): a float as the 16 bits of that type.
__device__ inline unsigned short out_bits16(float f, bool f16) {
  return f16 ? __builtin_bit_cast(unsigned short, (_Float16)f) : __builtin_bit_cast(unsigned short, (__bf16)f);
}
__device__ inline float out_back16(unsigned short b, bool f16) {
  return f16 ? (float)__builtin_bit_cast(_Float16, b) : (float)__builtin_bit_cast(__bf16, b);
}
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

// what the kernels need of one request (see AttnSeg); the table travels as a kernel argument
struct SegDev {
  int32_t row0, B, P_max;
  void* kc;
  void* vc;
  const int32_t* dP;
  const uint64_t* mask;
};
// TS = 1 for a single request (short kernel argument block, no indexing), else ATTN_MAX_SEGS
template <int TS>
struct SegTable { SegDev s[TS]; };

// F16: fp16 instead of bf16 storage (caches, operands, probabilities, output).
template <int D, int NG, int NQH, bool F16, int TS>
__global__ __launch_bounds__(64 * NG * NQH) void k_attn_fused(
    // (what the first cache loads depend on comes first: the leading kernel arguments are preloaded)
    const SegTable<TS> segs, int n_heads, int n_kv_heads, int cap, const float* part, int ks, size_t part_stride,
    size_t part_ld, const float2* cs, const typename Mma16<F16>::T* __restrict__ gq,
    const typename Mma16<F16>::T* __restrict__ gk, float eps, float* __restrict__ att_o, float* __restrict__ att_ml,
    int Bpad, unsigned short* o_out, int ldo, int oterms, int o_f16, int32_t* __restrict__ flags) {
  typedef typename Mma16<F16>::T T;
  typedef typename Mma16<F16>::v8 op8;
  typedef typename Mma16<F16>::v4 op4;
  // this workgroup's request: its rows of the stacked buffers, its caches, length and mask
  const SegDev& sg = segs.s[TS == 1 ? 0 : blockIdx.z];
  const int B = sg.B, row0 = sg.row0;
  T* const kc = static_cast<T*>(sg.kc);
  T* const vc = static_cast<T*>(sg.vc);
  const uint64_t* const mask = sg.mask;
  part += (size_t)row0 * part_ld;
  cs += (size_t)row0 * (D / 2);
  o_out += (size_t)row0 * ldo;
  constexpr int NTHR = 64 * NG * NQH;
  constexpr int NS = D / 16;               // operand loads (1 KiB pieces) per block, for K and for V
  constexpr int TROWS = NQH * 32;          // tree rows the LDS buffers hold (>= B for this instantiation)
  constexpr int KROW = D * 2 + 16;         // bytes per K / Q row in LDS (padded)
  constexpr int VROW = TROWS * 2 + 16;     // bytes per V^T row in LDS (padded)
  constexpr int TAIL_BYTES = 3 * TROWS * KROW + D * VROW;  // tree keys, tree values, rotated queries (two terms)
  constexpr int OREGS = (D / 32) * 16;                     // accumulator floats per lane
  constexpr int MERGE_BYTES = NG > 1 ? NG * NQH * (OREGS + 4) * 64 * 4 : 0;  // every wavefront's state
  constexpr int LDS_BYTES = TAIL_BYTES > MERGE_BYTES ? TAIL_BYTES : MERGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
  unsigned char* Kt = lds;                  // tree keys   [i][c]  (rotated)
  unsigned char* Vt = lds + TROWS * KROW;   // tree values [c][i]  (transposed)
  unsigned char* Qs = Vt + D * VROW;        // rotated queries [i][c]: the 16-bit value ...
  unsigned char* Ql = Qs + TROWS * KROW;    // ... and the 16-bit remainder of the fp32 query (q = Qs + Ql to 2^-17)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = wave % NG, qh = wave / NG;  // key group, query tile
  // head = the fast grid index: workgroups are dealt to the 8 XCDs round-robin, so head h runs on
  // XCD h % 8, where the projection kernel's workgroup of the same 128 columns ran (q, k and v
  // of head h sit 32 and 64 column groups apart): its partial sums are still in that XCD's L2
  const int split = blockIdx.y, nsplit = gridDim.y;
  int h = blockIdx.x;
  if (n_kv_heads != n_heads && (n_kv_heads & 7) == 0) {
    // grouped queries: the heads of one KV head stream the same cache blocks, so they share an XCD
    // (KV head j on XCD j % 8) and all but the first find the blocks in its L2; 8 | n_kv_heads
    // makes this a permutation of the heads
    const int grp = (int)((unsigned)n_heads / (unsigned)n_kv_heads), xcd = h & 7, s = h >> 3;
    const int t = (int)((unsigned)s / (unsigned)grp);
    h = (xcd + 8 * t) * grp + (s - t * grp);
  }
  const int l31 = lane & 31, hh = lane >> 5;
  // grouped queries: `group` query heads share KV head kvh; their projections sit at columns
  // [0,Hq) q, [Hq, Hq+Hkv) k, [Hq+Hkv, Hq+2Hkv) v of the fused projection
  const int group = (int)((unsigned)n_heads / (unsigned)n_kv_heads), kvh = (int)((unsigned)h / (unsigned)group);
  const int Hq = n_heads * D, Hkv = n_kv_heads * D;
  const int kcol = Hq + kvh * D - h * D, vcol = kcol + Hkv;  // relative to this head's q columns
  const bool tail_writer = h == kvh * group;                 // one head of the group stores the tree's K/V
  int P = *sg.dP;   // (used further down: the loads below do not wait for it)
  const bool last = blockIdx.y == gridDim.y - 1;
  // ---- q of all query tiles (every split), k and v of the tree (last split): sum the split-K
  // slices, rotate q and k, bf16 into LDS.  One item = 4 columns j0.. and their rotation partners
  // j0+d/2..: 16 neighbouring lanes read 256 contiguous bytes of a projection row.  The loads of
  // the first two slices of all of a thread's items are issued together: the buffer was written
  // by another kernel, so every dependent load is a trip to memory.
  const int nbt = (B + 31) >> 5;
  const int rows = nbt * 32;
  constexpr int NIT = TROWS * (D / 8) / NTHR;
  static_assert(TROWS * (D / 8) % NTHR == 0 && NIT >= 1, "items must divide over the workgroup");
  // Items are handled UG at a time.  With at most two per thread (trees of up to 64 nodes) their
  // loads are issued here, before anything waits for the cache length; larger trees take them two
  // at a time in a loop further down (registers, and code that runs once is fetched at memory speed).
  constexpr bool HOLD = NIT <= 2;
  constexpr int UG = HOLD ? NIT : 2;
  static_assert(NIT % UG == 0, "item groups");
  const float* prow[UG];
  f32x4 acc[UG][6], acc1[UG][6];  // q lo/hi, k lo/hi, v lo/hi of the first / second slice
  f32x4 c01[UG], c23[UG];         // the rotation angles: cos, sin of columns j0, j0+1 / j0+2, j0+3
  bool kv[UG];
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  const bool two = ks > 1;
  auto load_items = [&](int u0) {
#pragma unroll
    for (int u = 0; u < UG; ++u) {
      const int it = tid + (u0 + u) * NTHR;
      const int i = it / (D / 8), j0 = (it % (D / 8)) * 4;
      prow[u] = part + (size_t)i * part_ld + h * D + j0;  // row i < Bpad exists in the buffer
      kv[u] = last && i < B;
      const float* p1 = prow[u] + part_stride;
#pragma unroll
      for (int w = 0; w < 3; ++w) {
        const bool on = w == 0 || kv[u];
        const int col = w == 0 ? 0 : (w == 1 ? kcol : vcol);
        acc[u][2 * w] = on ? *reinterpret_cast<const f32x4*>(prow[u] + col) : zero4;
        acc[u][2 * w + 1] = on ? *reinterpret_cast<const f32x4*>(prow[u] + col + D / 2) : zero4;
        acc1[u][2 * w] = (on && two) ? *reinterpret_cast<const f32x4*>(p1 + col) : zero4;
        acc1[u][2 * w + 1] = (on && two) ? *reinterpret_cast<const f32x4*>(p1 + col + D / 2) : zero4;
      }
      c01[u] = *reinterpret_cast<const f32x4*>(cs + (size_t)i * (D / 2) + j0);
      c23[u] = *reinterpret_cast<const f32x4*>(cs + (size_t)i * (D / 2) + j0 + 2);
    }
  };
  if (HOLD) load_items(0);
  // a cache length the launch was not sized for, or one that leaves no room for the tree: flagged
  // (GOOSE_FLAG_CAPACITY), and clamped so that nothing is indexed outside the cache
  if ((P < 0 || P > sg.P_max || P > cap - B) && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
    atomicOr(flags, GOOSE_FLAG_CAPACITY);
  if (P > cap - B) P = cap - B;
  if (P < 0) P = 0;

  // ---- prefix blocks of this split, then of this key group
  const int nbp = (P + 31) >> 5;
  int b_lo, b_hi;
  if (nsplit == 1) {
    b_lo = 0; b_hi = nbp;
  } else {
    // (unsigned 32-bit divisions: block counts times split counts stay far below 2^32, and a 64-bit
    // division is a hundred instructions of code that every wavefront would fetch and run once)
    const int tc = nbt * TAIL_COST;
    const int per = (int)((unsigned)(nbp + tc + nsplit - 1) / (unsigned)nsplit);
    int pl = per - tc;
    pl = pl < 0 ? 0 : (pl > nbp ? nbp : pl);
    const int rest = nbp - pl;  // dealt evenly to splits 0 .. nsplit-2
    if (last) { b_lo = rest; b_hi = nbp; }
    else {
      const unsigned den = (unsigned)(nsplit - 1);
      b_lo = (int)((unsigned)(rest * split) / den);
      b_hi = (int)((unsigned)(rest * (split + 1)) / den);
    }
  }
  // a wavefront whose query tile lies wholly beyond the tree
  // walks no blocks; it still takes part in the prologue and in the barriers
  const bool idle = qh * 32 >= B;
  const int nb_split = idle ? 0 : b_hi - b_lo;
  const int blk0 = b_lo + (nb_split * g) / NG;
  const int nblk = b_lo + (nb_split * (g + 1)) / NG - blk0;
  // This wavefront's block sequence: its prefix blocks (operands from the cache), then, in the
  // last split, the tree blocks t = g, g+NG, .. (operands from LDS).
  const int ntail = (last && !idle) ? (nbt - g + NG - 1) / NG : 0;
  const int total = nblk + (ntail > 0 ? ntail : 0);

  const T* kh = kc + (size_t)kvh * cap * D;
  const T* vh = vc + (size_t)kvh * cap * D;
  // One block of operands in registers.  The K pieces are free again after the first MFMA chain
  // and the V pieces after the second, so the next block's loads are issued right there: they fly
  // during the softmax and the second chain (the loop below exists once: code executed once per
  // wavefront is all instruction-issue time, so the kernel is kept short).
  u32x4 kreg[NS], vreg[NS];
  auto fetch_k = [&](int idx) {
    if (idx < nblk) {
      const u32x4* kp = reinterpret_cast<const u32x4*>(kh + (size_t)(blk0 + idx) * 32 * D) + lane;
#pragma unroll
      for (int s = 0; s < NS; ++s) kreg[s] = kp[s * 64];
    } else {
      const int t = g + NG * (idx - nblk);
      const unsigned char* kp = Kt + (t * 32 + ((l31 >> 2) & 1) * 16 + (l31 & 3) + 4 * (l31 >> 3)) * KROW + hh * 16;
#pragma unroll
      for (int s = 0; s < NS; ++s) kreg[s] = *reinterpret_cast<const u32x4*>(kp + s * 32);
    }
  };
  auto fetch_v = [&](int idx) {
    if (idx < nblk) {
      const u32x4* vp = reinterpret_cast<const u32x4*>(vh + (size_t)(blk0 + idx) * 32 * D) + lane;
#pragma unroll
      for (int s = 0; s < NS; ++s) vreg[s] = vp[s * 64];
    } else {
      const int t = g + NG * (idx - nblk);
      const unsigned char* vp = Vt + l31 * VROW + (t * 32 + hh * 16) * 2;
#pragma unroll
      for (int s = 0; s < NS; ++s) vreg[s] = *reinterpret_cast<const u32x4*>(vp + (s >> 1) * 32 * VROW + (s & 1) * 16);
    }
  };
  // the first block is on its way while q (and the tree's k, v) are prepared
  if (nblk > 0) { fetch_k(0); fetch_v(0); }

  auto finish_items = [&](int u0) {
#pragma unroll
    for (int u = 0; u < UG; ++u)
#pragma unroll
      for (int w = 0; w < 6; ++w) acc[u][w] += acc1[u][w];
    for (int sl = 2; sl < ks; ++sl) {
#pragma unroll
      for (int u = 0; u < UG; ++u) {
        const float* p = prow[u] + sl * part_stride;
#pragma unroll
        for (int w = 0; w < 3; ++w)
          if (w == 0 || kv[u]) {
            const int col = w == 0 ? 0 : (w == 1 ? kcol : vcol);
            acc[u][2 * w] += *reinterpret_cast<const f32x4*>(p + col);
            acc[u][2 * w + 1] += *reinterpret_cast<const f32x4*>(p + col + D / 2);
          }
      }
    }
    if (gq != nullptr) {
      // per-head RMSNorm of q and k over the head's D columns: the D/8 items of a row sit in
      // neighbouring lanes, so the sum of squares is a short butterfly
#pragma unroll
      for (int u = 0; u < UG; ++u) {
        const int j0 = ((tid + (u0 + u) * NTHR) % (D / 8)) * 4;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          float ss = 0.f;
#pragma unroll
          for (int e = 0; e < 4; ++e) ss += acc[u][2 * w][e] * acc[u][2 * w][e] + acc[u][2 * w + 1][e] * acc[u][2 * w + 1][e];
#pragma unroll
          for (int off = 1; off < D / 8; off <<= 1) ss += __shfl_xor(ss, off, 64);
          const float rstd = 1.0f / sqrtf(ss / (float)D + eps);
          const T* g = w == 0 ? gq : gk;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[u][2 * w][e] *= rstd * (float)g[j0 + e];
            acc[u][2 * w + 1][e] *= rstd * (float)g[j0 + D / 2 + e];
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UG; ++u) {
      const int it = tid + (u0 + u) * NTHR;
      const int i = it / (D / 8), j0 = (it % (D / 8)) * 4;
      const float co[4] = {c01[u][0], c01[u][2], c23[u][0], c23[u][2]}, si[4] = {c01[u][1], c01[u][3], c23[u][1], c23[u][3]};
      // the query keeps two terms (the scores of a row share the query's rounding error, which
      // therefore does not average out over the keys as the keys' own rounding does)
      op4 rl, rh, rl2, rh2;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float ql = acc[u][0][e] * co[e] - acc[u][1][e] * si[e];
        const float qh = acc[u][1][e] * co[e] + acc[u][0][e] * si[e];
        rl[e] = (T)ql;
        rh[e] = (T)qh;
        rl2[e] = (T)(ql - (float)rl[e]);
        rh2[e] = (T)(qh - (float)rh[e]);
      }
      *reinterpret_cast<op4*>(Qs + i * KROW + j0 * 2) = rl;
      *reinterpret_cast<op4*>(Qs + i * KROW + (j0 + D / 2) * 2) = rh;
      *reinterpret_cast<op4*>(Ql + i * KROW + j0 * 2) = rl2;
      *reinterpret_cast<op4*>(Ql + i * KROW + (j0 + D / 2) * 2) = rh2;
      if (last && i < rows) {  // rows of the tree's blocks beyond B are zero (kv false)
        op4 kl, kh4, vl, vh4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kl[e] = (T)(acc[u][2][e] * co[e] - acc[u][3][e] * si[e]);
          kh4[e] = (T)(acc[u][3][e] * co[e] + acc[u][2][e] * si[e]);
          vl[e] = (T)acc[u][4][e];
          vh4[e] = (T)acc[u][5][e];
        }
        if (kv[u] && tail_writer) {
          // key row of slot P+i into the cache: columns j0..j0+3 sit in chunk (j0/16, (j0/8)%2) at j0%8
          T* kw = const_cast<T*>(kh);
          *reinterpret_cast<op4*>(kw + k_chunk_off<D>(P + i, j0 >> 4, (j0 >> 3) & 1) + (j0 & 7)) = kl;
          *reinterpret_cast<op4*>(kw + k_chunk_off<D>(P + i, (j0 + D / 2) >> 4, (j0 >> 3) & 1) + (j0 & 7)) = kh4;
        }
        *reinterpret_cast<op4*>(Kt + i * KROW + j0 * 2) = kl;
        *reinterpret_cast<op4*>(Kt + i * KROW + (j0 + D / 2) * 2) = kh4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          *reinterpret_cast<T*>(Vt + (j0 + e) * VROW + i * 2) = vl[e];
          *reinterpret_cast<T*>(Vt + (j0 + D / 2 + e) * VROW + i * 2) = vh4[e];
        }
      }
    }
  };
  if (HOLD) {
    finish_items(0);
  } else {
#pragma unroll 1
    for (int u0 = 0; u0 < NIT; u0 += UG) {
      load_items(u0);
      finish_items(u0);
    }
  }
  __syncthreads();

  // ---- this wavefront's q operand and ancestor row
  const int qi = qh * 32 + l31;
  op8 qf[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const op8*>(Qs + qi * KROW + (16 * s + 8 * hh) * 2);
  uint64_t mw0 = 0, mw1 = 0;
  if (qi < B) {
    const int W = (B + 63) >> 6;
    mw0 = mask[(size_t)qi * W];
    if (W > 1) mw1 = mask[(size_t)qi * W + 1];
  }
  if (nblk == 0 && total > 0) { fetch_k(0); fetch_v(0); }  // a tree block first: it is in LDS only now

  // ---- the tree's values into the cache, node index fastest so that neighbouring lanes fill
  // neighbouring bytes (the keys went out above)
  // (eight consecutive slots of one column are 16 contiguous bytes of the cache: one store per
  // (column, 8-slot group) where the group lies inside the tree, single elements at its two ends)
  if (last && tail_writer) {
    T* vw = const_cast<T*>(vh);
    const int g_lo = P >> 3, ngrp = ((P + B - 1) >> 3) - g_lo + 1;
    for (int it = tid; it < ngrp * D; it += NTHR) {
      const int c = it % D, G = g_lo + it / D;
      const int i0 = (G << 3) - P;  // tree node of the group's first slot (may be negative)
      const unsigned char* src = Vt + c * VROW;
      T* dst = vw + v_elem_off<D>(G << 3, c);
      if (i0 >= 0 && i0 + 8 <= B) {
        op8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = *reinterpret_cast<const T*>(src + (i0 + e) * 2);
        *reinterpret_cast<op8*>(dst) = v;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (i0 + e >= 0 && i0 + e < B) dst[e] = *reinterpret_cast<const T*>(src + (i0 + e) * 2);
      }
    }
  }

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m_run = NEG_BIG, l_run = 0.f;
  const float scale = 1.4426950408889634f / sqrtf((float)D);  // log2(e) / sqrt(d): softmax in base 2

  for (int idx = 0; idx < total; ++idx) {
    // visibility of this lane's 16 keys
    bool masked = false, ragged = false;
    unsigned vis = 0xFFFFu;
    if (idx >= nblk) {  // tree block: the ancestor bits of nodes j0 .. j0+15
      masked = true;
      const int j0 = (g + NG * (idx - nblk)) * 32 + hh * 16;
      vis = (unsigned)(j0 < 64 ? mw0 >> j0 : mw1 >> (j0 - 64)) & 0xFFFFu;
    } else {
      const int nvalid = P - (blk0 + idx) * 32;  // >= 32 except in the ragged last prefix block
      if (nvalid < 32) {
        // stale slots at or beyond P may hold anything: scores are replaced, values zeroed
        masked = ragged = true;
        const int mine = nvalid - hh * 16;
        vis = mine >= 16 ? 0xFFFFu : (mine <= 0 ? 0u : ((1u << mine) - 1u));
      }
    }
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s)
      sacc = Mma16<F16>::mfma(__builtin_bit_cast(op8, kreg[s]), qf[s], sacc);
#pragma unroll
    for (int s = 0; s < NS; ++s) {  // the query's second term, read from LDS as it is used
      const op8 ql = *reinterpret_cast<const op8*>(Ql + qi * KROW + (16 * s + 8 * hh) * 2);
      sacc = Mma16<F16>::mfma(__builtin_bit_cast(op8, kreg[s]), ql, sacc);
    }
    if (idx + 1 < total) fetch_k(idx + 1);
    if (masked) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = ((vis >> r) & 1u) ? sacc[r] : NEG_BIG;  // also drops NaNs of stale keys
    }
    float tmax = NEG_BIG;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sacc[r] = fmaxf(sacc[r] * scale, NEG_BIG);
      tmax = fmaxf(tmax, sacc[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    const bool grew = m_new > m_run;
    m_run = m_new;
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(sacc[r] - m_new);
    if (masked) {  // a fully masked row has m_new == NEG_BIG: exp2(0) must not count
#pragma unroll
      for (int r = 0; r < 16; ++r) p[r] = ((vis >> r) & 1u) ? p[r] : 0.f;
    }
    if (ragged) {  // stale values -> 0 (here `vis` depends on the key half only, as the V operand's keys do)
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const unsigned bits = (vis >> ((s & 1) * 8)) & 0xFFu;
        u16x8 e = __builtin_bit_cast(u16x8, vreg[s]);
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (!((bits >> k) & 1u)) e[k] = 0;
        vreg[s] = __builtin_bit_cast(u32x4, e);
      }
    }
    float psum = 0.f;
    op8 pf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      psum += p[r];
      pf[r >> 3][r & 7] = (T)p[r];
    }
    l_run = l_run * alpha + psum;
    // the running maximum settles after a few blocks: skip the rescale of O when no lane's maximum grew
    if (__builtin_amdgcn_ballot_w64(grew) != 0) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        oacc[dt] = Mma16<F16>::mfma(__builtin_bit_cast(op8, vreg[dt * 2 + j]), pf[j], oacc[dt]);
    if (idx + 1 < total) fetch_v(idx + 1);
  }

  // ---- merge the key groups of a query tile through LDS, in one round: every wavefront leaves its
  // state there ((m, l), then the accumulator four registers at a time: piece q of lane l at float
  // 256 q + 4 l), and then owns QPW of the accumulator's register quads: it combines those quads of
  // all NG groups, in group order, and writes them out.  No wavefront waits for another's sums, and
  // the output stage is spread over all of them.
  constexpr int QUADS = (D / 32) * 4, QPW = QUADS / NG;
  static_assert(QUADS % NG == 0, "register quads must divide over the key groups");
  f32x4 res[QPW];
  float l_sum = l_run;
  if (NG > 1) {
    __syncthreads();  // every wavefront is done with the tree and query buffers
    float* mbuf = reinterpret_cast<float*>(lds);
    constexpr int WFLOATS = (QUADS + 1) * 256;
    {
      float* dst = mbuf + (size_t)(qh * NG + g) * WFLOATS + lane * 4;
      *reinterpret_cast<f32x4*>(dst) = f32x4{m_run, l_run, 0.f, 0.f};
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int a = 0; a < 4; ++a)
          *reinterpret_cast<f32x4*>(dst + 256 * (1 + dt * 4 + a)) =
              f32x4{oacc[dt][a * 4], oacc[dt][a * 4 + 1], oacc[dt][a * 4 + 2], oacc[dt][a * 4 + 3]};
    }
    __syncthreads();
    const float* src = mbuf + (size_t)(qh * NG) * WFLOATS + lane * 4;
    float mj[NG], lj[NG];
    float m_all = NEG_BIG;
#pragma unroll
    for (int j = 0; j < NG; ++j) {
      const f32x4 ml = *reinterpret_cast<const f32x4*>(src + (size_t)j * WFLOATS);
      mj[j] = ml[0];
      lj[j] = ml[1];
      m_all = fmaxf(m_all, mj[j]);
    }
    l_sum = 0.f;
#pragma unroll
    for (int q = 0; q < QPW; ++q) res[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NG; ++j) {
      const float w = __builtin_amdgcn_exp2f(mj[j] - m_all);
      l_sum += w * lj[j];
#pragma unroll
      for (int q = 0; q < QPW; ++q)
        res[q] += w * *reinterpret_cast<const f32x4*>(src + (size_t)j * WFLOATS + 256 * (1 + g * QPW + q));
    }
    m_run = m_all;
  } else {
#pragma unroll
    for (int q = 0; q < QPW; ++q)
      res[q] = f32x4{oacc[q >> 2][(q & 3) * 4], oacc[q >> 2][(q & 3) * 4 + 1], oacc[q >> 2][(q & 3) * 4 + 2],
                     oacc[q >> 2][(q & 3) * 4 + 3]};
  }

  // ---- output: C layout of O^T, register r of lane (q, hh) is d = dt*32 + 8*(r/4) + 4*hh + r%4;
  // quad (dt, a) = registers 4a .. 4a+3 of block dt = columns dt*32 + a*8 + hh*4 ..
  const float l_tot = l_sum + __shfl_xor(l_sum, 32, 64);
  if (qi >= B) return;
  if (nsplit == 1) {
    const float inv = 1.0f / l_tot;
    unsigned short* orow = o_out + (size_t)qi * ldo;
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
      const int quad = g * QPW + q;
      u16x4 v, v2;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float f = res[q][e] * inv;
        v[e] = out_bits16(f, o_f16);
        v2[e] = out_bits16(f - out_back16(v[e], o_f16), o_f16);
      }
      unsigned short* dst = orow + term_pos(oterms, h * D + quad * 8 + hh * 4);  // four columns inside one group of eight
      *reinterpret_cast<u16x4*>(dst) = v;
      if (oterms == 2) *reinterpret_cast<u16x4*>(dst + 8) = v2;
    }
  } else {
    const size_t base = ((size_t)h * nsplit + split) * Bpad + row0 + qi;
    if (hh == 0 && g == 0) {
      att_ml[base * 2] = m_run;
      att_ml[base * 2 + 1] = l_tot;
    }
    float* orow = att_o + base * D;
#pragma unroll
    for (int q = 0; q < QPW; ++q) *reinterpret_cast<f32x4*>(orow + (g * QPW + q) * 8 + hh * 4) = res[q];
  }
}

// ---- Trees of more than 64 nodes (three or four 32-query tiles), head size 128 ------------------
// In k_attn_fused every wavefront loads the key blocks it walks itself, so a block is pulled into
// the compute unit once per query tile; with three or four tiles that traffic (not HBM) bounds the
// kernel.  Here the workgroup (2 key groups x NQH query tiles, one wavefront each) brings every
// block in ONCE, global -> LDS without passing registers (global_load_lds, 1 KiB per instruction,
// which is exactly one operand piece of the operand-ordered caches), into a ring of RING slots of
// one block (8 KiB of K + 8 KiB of V) each; the wavefronts read their operands from the ring.  The
// prefix blocks of the split are taken two per step, block 2j by key group 0 and block 2j+1 by key
// group 1; block k lives in slot k % RING.  Step j: wait until blocks 2j and 2j+1 have landed,
// barrier (which also tells that the blocks of step j-1 have been consumed), issue the copies of
// blocks 2j+3 and 2j+4 into the two slots just freed, compute.  Three blocks (48 KiB) are in flight
// per compute unit, at no cost in registers.  Every wavefront issues the same number of copies per
// block (LPB), so that one immediate wait count fits all of them; blocks beyond the split's range
// re-read its last block (from the L2) and are never consumed.  The tree's own blocks (last split)
// follow from LDS as in k_attn_fused, without barriers.  The ring also serves as the staging
// buffer of the rotated queries (both terms end up in registers) and as the merge buffer at the
// end.  Arithmetic, masking, summation order within a wavefront and the outputs are those of
// k_attn_fused with two key groups, except that a group walks every other block instead of a
// contiguous half.
#define GOOSE_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }  // s_waitcnt vmcnt(n) only

template <int NQH, bool F16, int TS>
__global__ __launch_bounds__(128 * NQH) void k_attn_wide(
    const SegTable<TS> segs, int n_heads, int n_kv_heads, int cap, const float* part, int ks, size_t part_stride,
    size_t part_ld, const float2* cs, const typename Mma16<F16>::T* __restrict__ gq,
    const typename Mma16<F16>::T* __restrict__ gk, float eps, float* __restrict__ att_o, float* __restrict__ att_ml,
    int Bpad, unsigned short* o_out, int ldo, int oterms, int o_f16, int32_t* __restrict__ flags) {
  typedef typename Mma16<F16>::T T;
  typedef typename Mma16<F16>::v8 op8;
  typedef typename Mma16<F16>::v4 op4;
  constexpr int D = 128, NG = 2;
  const SegDev& sg = segs.s[TS == 1 ? 0 : blockIdx.z];
  const int B = sg.B, row0 = sg.row0;
  T* const kc = static_cast<T*>(sg.kc);
  T* const vc = static_cast<T*>(sg.vc);
  const uint64_t* const mask = sg.mask;
  part += (size_t)row0 * part_ld;
  cs += (size_t)row0 * (D / 2);
  o_out += (size_t)row0 * ldo;
  constexpr int NTHR = 64 * NG * NQH, NWAVES = NG * NQH;
  constexpr int NS = D / 16;               // operand pieces (1 KiB) per block, for K and for V
  constexpr int TROWS = NQH * 32;          // tree rows the LDS buffers hold
  constexpr int KROW = D * 2 + 16;         // bytes per K / Q row in LDS (padded)
  constexpr int VROW = TROWS * 2 + 16;     // bytes per V^T row in LDS (padded)
  constexpr int KV_BYTES = TROWS * KROW + D * VROW;  // the tree's keys and values
  constexpr int SLOT = 2 * NS * 1024;      // one block: its K pieces, then its V pieces
  constexpr int RING = 5;
  constexpr int RING_BYTES = RING * SLOT;
  constexpr int OREGS = (D / 32) * 16;
  constexpr int QUADS = (D / 32) * 4, QPW = QUADS / NG;
  constexpr int WFLOATS = (QPW + 1) * 256;  // what a wavefront leaves for its partner at the merge
  static_assert(2 * TROWS * KROW <= RING_BYTES, "the query staging buffer lies in the ring");
  static_assert(NWAVES * WFLOATS * 4 <= RING_BYTES, "the merge buffer lies in the ring");
  static_assert(KV_BYTES + RING_BYTES <= 160 * 1024, "LDS of one compute unit");
  // (two arrays: the compiler then knows that the copies into the ring do not touch the tree's buffers)
  __shared__ __attribute__((aligned(16))) unsigned char kv_lds[KV_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char ring[RING_BYTES];
  unsigned char* Kt = kv_lds;                 // tree keys   [i][c]  (rotated)
  unsigned char* Vt = kv_lds + TROWS * KROW;  // tree values [c][i]  (transposed)
  unsigned char* Qs = ring;                   // rotated queries [i][c]: the 16-bit value ...
  unsigned char* Ql = ring + TROWS * KROW;    // ... and the 16-bit remainder

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = wave % NG, qh = wave / NG;  // key group, query tile
  const int split = blockIdx.y, nsplit = gridDim.y;
  int h = blockIdx.x;  // head = the fast grid index, as in k_attn_fused (same XCD as the projection's columns)
  if (n_kv_heads != n_heads && (n_kv_heads & 7) == 0) {
    const int grp = (int)((unsigned)n_heads / (unsigned)n_kv_heads), xcd = h & 7, s = h >> 3;
    const int t = (int)((unsigned)s / (unsigned)grp);
    h = (xcd + 8 * t) * grp + (s - t * grp);
  }
  const int l31 = lane & 31, hh = lane >> 5;
  const int group = (int)((unsigned)n_heads / (unsigned)n_kv_heads), kvh = (int)((unsigned)h / (unsigned)group);
  const int Hq = n_heads * D, Hkv = n_kv_heads * D;
  const int kcol = Hq + kvh * D - h * D, vcol = kcol + Hkv;
  const bool tail_writer = h == kvh * group;
  int P = *sg.dP;
  const bool last = blockIdx.y == gridDim.y - 1;
  const int nbt = (B + 31) >> 5;
  const int rows = nbt * 32;
  constexpr int NIT = TROWS * (D / 8) / NTHR, UG = 2;
  static_assert(TROWS * (D / 8) % NTHR == 0 && NIT % UG == 0, "items must divide over the workgroup");
  const float* prow[UG];
  f32x4 acc[UG][6], acc1[UG][6];
  f32x4 c01[UG], c23[UG];
  bool kv[UG];
  const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
  const bool two = ks > 1;
  auto load_items = [&](int u0) {
#pragma unroll
    for (int u = 0; u < UG; ++u) {
      const int it = tid + (u0 + u) * NTHR;
      const int i = it / (D / 8), j0 = (it % (D / 8)) * 4;
      prow[u] = part + (size_t)i * part_ld + h * D + j0;  // row i < Bpad exists in the buffer
      kv[u] = last && i < B;
      const float* p1 = prow[u] + part_stride;
#pragma unroll
      for (int w = 0; w < 3; ++w) {
        const bool on = w == 0 || kv[u];
        const int col = w == 0 ? 0 : (w == 1 ? kcol : vcol);
        acc[u][2 * w] = on ? *reinterpret_cast<const f32x4*>(prow[u] + col) : zero4;
        acc[u][2 * w + 1] = on ? *reinterpret_cast<const f32x4*>(prow[u] + col + D / 2) : zero4;
        acc1[u][2 * w] = (on && two) ? *reinterpret_cast<const f32x4*>(p1 + col) : zero4;
        acc1[u][2 * w + 1] = (on && two) ? *reinterpret_cast<const f32x4*>(p1 + col + D / 2) : zero4;
      }
      c01[u] = *reinterpret_cast<const f32x4*>(cs + (size_t)i * (D / 2) + j0);
      c23[u] = *reinterpret_cast<const f32x4*>(cs + (size_t)i * (D / 2) + j0 + 2);
    }
  };
  if ((P < 0 || P > sg.P_max || P > cap - B) && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
    atomicOr(flags, GOOSE_FLAG_CAPACITY);
  if (P > cap - B) P = cap - B;
  if (P < 0) P = 0;

  // ---- prefix blocks of this split (the same division as k_attn_fused)
  const int nbp = (P + 31) >> 5;
  int b_lo, b_hi;
  if (nsplit == 1) {
    b_lo = 0; b_hi = nbp;
  } else {
    const int tc = nbt * TAIL_COST;
    const int per = (int)((unsigned)(nbp + tc + nsplit - 1) / (unsigned)nsplit);
    int pl = per - tc;
    pl = pl < 0 ? 0 : (pl > nbp ? nbp : pl);
    const int rest = nbp - pl;
    if (last) { b_lo = rest; b_hi = nbp; }
    else {
      const unsigned den = (unsigned)(nsplit - 1);
      b_lo = (int)((unsigned)(rest * split) / den);
      b_hi = (int)((unsigned)(rest * (split + 1)) / den);
    }
  }
  const bool idle = qh * 32 >= B;          // a query tile wholly beyond the tree: copies and barriers only
  const int nb_split = b_hi - b_lo;        // (the same for every wavefront of the workgroup)
  const int nsteps = (nb_split + 1) >> 1;
  const int ntail = (last && !idle) ? (nbt - g + NG - 1) / NG : 0;
  const int total = nsteps + (ntail > 0 ? ntail : 0);

  const T* kh = kc + (size_t)kvh * cap * D;
  const T* vh = vc + (size_t)kvh * cap * D;

  auto finish_items = [&](int u0) {
#pragma unroll
    for (int u = 0; u < UG; ++u)
#pragma unroll
      for (int w = 0; w < 6; ++w) acc[u][w] += acc1[u][w];
    for (int sl = 2; sl < ks; ++sl) {
#pragma unroll
      for (int u = 0; u < UG; ++u) {
        const float* p = prow[u] + sl * part_stride;
#pragma unroll
        for (int w = 0; w < 3; ++w)
          if (w == 0 || kv[u]) {
            const int col = w == 0 ? 0 : (w == 1 ? kcol : vcol);
            acc[u][2 * w] += *reinterpret_cast<const f32x4*>(p + col);
            acc[u][2 * w + 1] += *reinterpret_cast<const f32x4*>(p + col + D / 2);
          }
      }
    }
    if (gq != nullptr) {
#pragma unroll
      for (int u = 0; u < UG; ++u) {
        const int j0 = ((tid + (u0 + u) * NTHR) % (D / 8)) * 4;
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          float ss = 0.f;
#pragma unroll
          for (int e = 0; e < 4; ++e) ss += acc[u][2 * w][e] * acc[u][2 * w][e] + acc[u][2 * w + 1][e] * acc[u][2 * w + 1][e];
#pragma unroll
          for (int off = 1; off < D / 8; off <<= 1) ss += __shfl_xor(ss, off, 64);
          const float rstd = 1.0f / sqrtf(ss / (float)D + eps);
          const T* gn = w == 0 ? gq : gk;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[u][2 * w][e] *= rstd * (float)gn[j0 + e];
            acc[u][2 * w + 1][e] *= rstd * (float)gn[j0 + D / 2 + e];
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UG; ++u) {
      const int it = tid + (u0 + u) * NTHR;
      const int i = it / (D / 8), j0 = (it % (D / 8)) * 4;
      const float co[4] = {c01[u][0], c01[u][2], c23[u][0], c23[u][2]}, si[4] = {c01[u][1], c01[u][3], c23[u][1], c23[u][3]};
      op4 rl, rh, rl2, rh2;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float qlo = acc[u][0][e] * co[e] - acc[u][1][e] * si[e];
        const float qhi = acc[u][1][e] * co[e] + acc[u][0][e] * si[e];
        rl[e] = (T)qlo;
        rh[e] = (T)qhi;
        rl2[e] = (T)(qlo - (float)rl[e]);
        rh2[e] = (T)(qhi - (float)rh[e]);
      }
      *reinterpret_cast<op4*>(Qs + i * KROW + j0 * 2) = rl;
      *reinterpret_cast<op4*>(Qs + i * KROW + (j0 + D / 2) * 2) = rh;
      *reinterpret_cast<op4*>(Ql + i * KROW + j0 * 2) = rl2;
      *reinterpret_cast<op4*>(Ql + i * KROW + (j0 + D / 2) * 2) = rh2;
      if (last && i < rows) {  // rows of the tree's blocks beyond B are zero (kv false)
        op4 kl, kh4, vl, vh4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          kl[e] = (T)(acc[u][2][e] * co[e] - acc[u][3][e] * si[e]);
          kh4[e] = (T)(acc[u][3][e] * co[e] + acc[u][2][e] * si[e]);
          vl[e] = (T)acc[u][4][e];
          vh4[e] = (T)acc[u][5][e];
        }
        if (kv[u] && tail_writer) {
          T* kw = const_cast<T*>(kh);
          *reinterpret_cast<op4*>(kw + k_chunk_off<D>(P + i, j0 >> 4, (j0 >> 3) & 1) + (j0 & 7)) = kl;
          *reinterpret_cast<op4*>(kw + k_chunk_off<D>(P + i, (j0 + D / 2) >> 4, (j0 >> 3) & 1) + (j0 & 7)) = kh4;
        }
        *reinterpret_cast<op4*>(Kt + i * KROW + j0 * 2) = kl;
        *reinterpret_cast<op4*>(Kt + i * KROW + (j0 + D / 2) * 2) = kh4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          *reinterpret_cast<T*>(Vt + (j0 + e) * VROW + i * 2) = vl[e];
          *reinterpret_cast<T*>(Vt + (j0 + D / 2 + e) * VROW + i * 2) = vh4[e];
        }
      }
    }
  };
#pragma unroll 1
  for (int u0 = 0; u0 < NIT; u0 += UG) {
    load_items(u0);
    finish_items(u0);
  }
  __syncthreads();

  // ---- this wavefront's q operand, both terms, and ancestor row
  const int qi = qh * 32 + l31;
  op8 qf[NS], qf2[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    qf[s] = *reinterpret_cast<const op8*>(Qs + qi * KROW + (16 * s + 8 * hh) * 2);
    qf2[s] = *reinterpret_cast<const op8*>(Ql + qi * KROW + (16 * s + 8 * hh) * 2);
  }
  uint64_t mw0 = 0, mw1 = 0;
  if (qi < B) {
    const int W = (B + 63) >> 6;
    mw0 = mask[(size_t)qi * W];
    if (W > 1) mw1 = mask[(size_t)qi * W + 1];
  }
  // ---- the tree's values into the cache (as in k_attn_fused)
  if (last && tail_writer) {
    T* vw = const_cast<T*>(vh);
    const int g_lo = P >> 3, ngrp = ((P + B - 1) >> 3) - g_lo + 1;
    for (int it = tid; it < ngrp * D; it += NTHR) {
      const int c = it % D, G = g_lo + it / D;
      const int i0 = (G << 3) - P;
      const unsigned char* src = Vt + c * VROW;
      T* dst = vw + v_elem_off<D>(G << 3, c);
      if (i0 >= 0 && i0 + 8 <= B) {
        op8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = *reinterpret_cast<const T*>(src + (i0 + e) * 2);
        *reinterpret_cast<op8*>(dst) = v;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (i0 + e >= 0 && i0 + e < B) dst[e] = *reinterpret_cast<const T*>(src + (i0 + e) * 2);
      }
    }
  }
  // Everything this wavefront has loaded or stored so far is done (the wait counts below count the
  // ring's copies only), and every wavefront holds its queries: the staging buffer becomes the ring.
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __syncthreads();

  // ---- the ring.  Copy instruction q of a wavefront moves piece min(wave*LPB + q, 2 NS - 1) of a block.
  constexpr int LPB = (2 * NS + NWAVES - 1) / NWAVES;
  const unsigned char* csrc[LPB];
  int cdst[LPB];
#pragma unroll
  for (int q = 0; q < LPB; ++q) {
    const int p = min(wave * LPB + q, 2 * NS - 1);
    csrc[q] = reinterpret_cast<const unsigned char*>(p < NS ? kh : vh) + (size_t)b_lo * (32 * D * 2) + (p & (NS - 1)) * 1024 +
              lane * 16;
    cdst[q] = p * 1024;
  }
  auto issue = [&](int k) {  // block k of the split into slot k % RING (beyond the range: the last block again)
    const int kc_ = min(k, nb_split - 1);
    const int slot = (int)((unsigned)k % (unsigned)RING);
#pragma unroll
    for (int q = 0; q < LPB; ++q) {
      unsigned char* dst = ring + slot * SLOT + cdst[q];
#if defined(__HIP_DEVICE_COMPILE__)  // (the host pass knows no such builtin and would silently drop the kernel's stub)
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const u32x4*>(csrc[q] + (size_t)kc_ * (32 * D * 2)),
                                       GOOSE_LDS_PTR(dst), 16, 0, 0);
#else
      (void)dst;
#endif
    }
  };
  auto barrier = [&]() {  // (raw: __syncthreads would also drain every copy in flight)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  // eight operand pieces of a ring slot: the reads and the wait for them in one statement (the
  // compiler is not told about these reads, so it does not make them wait for the copies in flight,
  // and it never sees registers whose data is still on its way)
  const unsigned ring_addr = (unsigned)(uintptr_t)GOOSE_LDS_PTR(ring) + lane * 16;
  u32x4 kreg[NS];
  auto read_ring = [&](unsigned addr) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile(
        "ds_read_b128 %0, %8\n\t"
        "ds_read_b128 %1, %8 offset:1024\n\t"
        "ds_read_b128 %2, %8 offset:2048\n\t"
        "ds_read_b128 %3, %8 offset:3072\n\t"
        "ds_read_b128 %4, %8 offset:4096\n\t"
        "ds_read_b128 %5, %8 offset:5120\n\t"
        "ds_read_b128 %6, %8 offset:6144\n\t"
        "ds_read_b128 %7, %8 offset:7168\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&v"(kreg[0]), "=&v"(kreg[1]), "=&v"(kreg[2]), "=&v"(kreg[3]), "=&v"(kreg[4]), "=&v"(kreg[5]),
          "=&v"(kreg[6]), "=&v"(kreg[7])
        : "v"(addr)
        : "memory");
#else
    (void)addr;
#endif
  };
  static_assert(NS == 8, "read_ring moves eight pieces");
  if (nsteps > 0) {
    issue(0);
    issue(1);
    issue(2);
    __builtin_amdgcn_sched_barrier(0);
  }

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m_run = NEG_BIG, l_run = 0.f;
  const float scale = 1.4426950408889634f / sqrtf((float)D);  // log2(e) / sqrt(d): softmax in base 2

  for (int idx = 0; idx < total; ++idx) {
    const bool staged = idx < nsteps;
    const int kblk = 2 * idx + g;  // this wavefront's block of the split in a staged step
    unsigned slot_addr = 0;
    if (staged) {
      // blocks 2 idx and 2 idx + 1 have landed once at most the copies of block 2 idx + 2 are pending
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPB));
      barrier();
      issue(2 * idx + 3);
      issue(2 * idx + 4);
      __builtin_amdgcn_sched_barrier(0);
      if (idle || kblk >= nb_split) continue;
      slot_addr = ring_addr + ((unsigned)kblk % (unsigned)RING) * SLOT;
    }
    // visibility of this lane's 16 keys
    bool masked = false, ragged = false;
    unsigned vis = 0xFFFFu;
    if (!staged) {  // tree block: the ancestor bits of nodes j0 .. j0+15
      masked = true;
      const int j0 = (g + NG * (idx - nsteps)) * 32 + hh * 16;
      vis = (unsigned)(j0 < 64 ? mw0 >> j0 : mw1 >> (j0 - 64)) & 0xFFFFu;
      const int t = g + NG * (idx - nsteps);
      const unsigned char* kp = Kt + (t * 32 + ((l31 >> 2) & 1) * 16 + (l31 & 3) + 4 * (l31 >> 3)) * KROW + hh * 16;
#pragma unroll
      for (int s = 0; s < NS; ++s) kreg[s] = *reinterpret_cast<const u32x4*>(kp + s * 32);
    } else {
      const int nvalid = P - (b_lo + kblk) * 32;  // >= 32 except in the ragged last prefix block
      if (nvalid < 32) {
        masked = ragged = true;
        const int mine = nvalid - hh * 16;
        vis = mine >= 16 ? 0xFFFFu : (mine <= 0 ? 0u : ((1u << mine) - 1u));
      }
      read_ring(slot_addr);
    }
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s)
      sacc = Mma16<F16>::mfma(__builtin_bit_cast(op8, kreg[s]), qf[s], sacc);
#pragma unroll
    for (int s = 0; s < NS; ++s)
      sacc = Mma16<F16>::mfma(__builtin_bit_cast(op8, kreg[s]), qf2[s], sacc);
    if (masked) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = ((vis >> r) & 1u) ? sacc[r] : NEG_BIG;  // also drops NaNs of stale keys
    }
    float tmax = NEG_BIG;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      sacc[r] = fmaxf(sacc[r] * scale, NEG_BIG);
      tmax = fmaxf(tmax, sacc[r]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    const bool grew = m_new > m_run;
    m_run = m_new;
    float p[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(sacc[r] - m_new);
    if (masked) {  // a fully masked row has m_new == NEG_BIG: exp2(0) must not count
#pragma unroll
      for (int r = 0; r < 16; ++r) p[r] = ((vis >> r) & 1u) ? p[r] : 0.f;
    }
    float psum = 0.f;
    op8 pf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      psum += p[r];
      pf[r >> 3][r & 7] = (T)p[r];
    }
    l_run = l_run * alpha + psum;
    if (__builtin_amdgcn_ballot_w64(grew) != 0) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
    // the values take the registers the keys had
    if (!staged) {
      const int t = g + NG * (idx - nsteps);
      const unsigned char* vp = Vt + l31 * VROW + (t * 32 + hh * 16) * 2;
#pragma unroll
      for (int s = 0; s < NS; ++s) kreg[s] = *reinterpret_cast<const u32x4*>(vp + (s >> 1) * 32 * VROW + (s & 1) * 16);
    } else {
      read_ring(slot_addr + NS * 1024);
    }
    if (ragged) {  // stale values -> 0
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const unsigned bits = (vis >> ((s & 1) * 8)) & 0xFFu;
        u16x8 e = __builtin_bit_cast(u16x8, kreg[s]);
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (!((bits >> k) & 1u)) e[k] = 0;
        kreg[s] = __builtin_bit_cast(u32x4, e);
      }
    }
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        oacc[dt] = Mma16<F16>::mfma(__builtin_bit_cast(op8, kreg[dt * 2 + j]), pf[j], oacc[dt]);
  }

  // ---- merge the two key groups of a query tile through the ring's memory: every wavefront leaves
  // (m, l) and the accumulator quads its partner owns, then combines its own QPW quads with the
  // partner's copy of them, group 0 first, and writes them out.
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // (copies of blocks beyond the range may still be landing)
  __syncthreads();
  f32x4 res[QPW];
  float l_sum;
  {
    float* mbuf = reinterpret_cast<float*>(ring);
    float* dst = mbuf + (size_t)wave * WFLOATS + lane * 4;
    *reinterpret_cast<f32x4*>(dst) = f32x4{m_run, l_run, 0.f, 0.f};
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
      // quad q of the partner's share: group 0 gives away quads QPW .. 2 QPW - 1, group 1 quads 0 .. QPW - 1
      const int q0 = q, q1 = QPW + q;
      const f32x4 a = {oacc[q0 >> 2][(q0 & 3) * 4], oacc[q0 >> 2][(q0 & 3) * 4 + 1], oacc[q0 >> 2][(q0 & 3) * 4 + 2],
                       oacc[q0 >> 2][(q0 & 3) * 4 + 3]};
      const f32x4 b = {oacc[q1 >> 2][(q1 & 3) * 4], oacc[q1 >> 2][(q1 & 3) * 4 + 1], oacc[q1 >> 2][(q1 & 3) * 4 + 2],
                       oacc[q1 >> 2][(q1 & 3) * 4 + 3]};
      *reinterpret_cast<f32x4*>(dst + 256 * (1 + q)) = g == 0 ? b : a;
      res[q] = g == 0 ? a : b;  // (its own share, for now)
    }
    __syncthreads();
    const float* src = mbuf + (size_t)(wave ^ 1) * WFLOATS + lane * 4;  // (NG == 2: the partner is wave ^ 1)
    const f32x4 ml = *reinterpret_cast<const f32x4*>(src);
    const float m0 = g == 0 ? m_run : ml[0], m1 = g == 0 ? ml[0] : m_run;
    const float l0 = g == 0 ? l_run : ml[1], l1 = g == 0 ? ml[1] : l_run;
    const float m_all = fmaxf(m0, m1);
    const float w0 = __builtin_amdgcn_exp2f(m0 - m_all), w1 = __builtin_amdgcn_exp2f(m1 - m_all);
    l_sum = w0 * l0 + w1 * l1;
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
      const f32x4 other = *reinterpret_cast<const f32x4*>(src + 256 * (1 + q));
      res[q] = g == 0 ? w0 * res[q] + w1 * other : w0 * other + w1 * res[q];
    }
    m_run = m_all;
  }

  // ---- output (as in k_attn_fused)
  const float l_tot = l_sum + __shfl_xor(l_sum, 32, 64);
  if (qi >= B) return;
  if (nsplit == 1) {
    const float inv = 1.0f / l_tot;
    unsigned short* orow = o_out + (size_t)qi * ldo;
#pragma unroll
    for (int q = 0; q < QPW; ++q) {
      const int quad = g * QPW + q;
      u16x4 v, v2;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float f = res[q][e] * inv;
        v[e] = out_bits16(f, o_f16);
        v2[e] = out_bits16(f - out_back16(v[e], o_f16), o_f16);
      }
      unsigned short* dst = orow + term_pos(oterms, h * D + quad * 8 + hh * 4);
      *reinterpret_cast<u16x4*>(dst) = v;
      if (oterms == 2) *reinterpret_cast<u16x4*>(dst + 8) = v2;
    }
  } else {
    const size_t base = ((size_t)h * nsplit + split) * Bpad + row0 + qi;
    if (hh == 0 && g == 0) {
      att_ml[base * 2] = m_run;
      att_ml[base * 2 + 1] = l_tot;
    }
    float* orow = att_o + base * D;
#pragma unroll
    for (int q = 0; q < QPW; ++q) *reinterpret_cast<f32x4*>(orow + (g * QPW + q) * 8 + hh * 4) = res[q];
  }
}

// o[q][h*D + c] = sum_s 2^(m_s - m) O_s[c] / sum_s 2^(m_s - m) l_s, splits taken in index order.
// A workgroup of 256 threads merges 1024 / D rows of one head, four columns per thread; the loads of
// up to eight splits are issued together (one load per loop round would make every split a trip to
// memory of its own).
template <bool F16, int TS>
__global__ __launch_bounds__(256) void k_attn_merge(const float* __restrict__ att_o, const float* __restrict__ att_ml,
                                                    int nsplit, int Bpad, int D, unsigned short* __restrict__ o, int ldo,
                                                    int oterms, int o_f16, const SegTable<TS> segs) {
  const SegDev& sg = segs.s[TS == 1 ? 0 : blockIdx.z];
  const int tpr = D >> 2;  // threads per row
  const int r = blockIdx.y * (256 / tpr) + threadIdx.x / tpr, c = (threadIdx.x % tpr) * 4;
  if (r >= sg.B) return;
  // head = the fast grid index: the workgroup runs on the XCD whose L2 holds that head's partials
  const int qi = sg.row0 + r, h = blockIdx.x;
  const size_t base0 = (size_t)h * nsplit * Bpad + qi, step = Bpad;  // split s at base0 + s * step
  constexpr int CH = 8;
  float mmax = NEG_BIG;
  for (int s0 = 0; s0 < nsplit; s0 += CH) {
    float m[CH];
#pragma unroll
    for (int k = 0; k < CH; ++k) m[k] = att_ml[(base0 + (size_t)min(s0 + k, nsplit - 1) * step) * 2];
#pragma unroll
    for (int k = 0; k < CH; ++k) mmax = fmaxf(mmax, m[k]);
  }
  f32x4 num = {0.f, 0.f, 0.f, 0.f};
  float den = 0.f;
  for (int s0 = 0; s0 < nsplit; s0 += CH) {
    float2 ml[CH];
    f32x4 ov[CH];
#pragma unroll
    for (int k = 0; k < CH; ++k) {
      const size_t base = base0 + (size_t)min(s0 + k, nsplit - 1) * step;
      ml[k] = *reinterpret_cast<const float2*>(att_ml + base * 2);
      ov[k] = *reinterpret_cast<const f32x4*>(att_o + base * D + c);
    }
#pragma unroll
    for (int k = 0; k < CH; ++k) {
      const float w = (s0 + k < nsplit) ? exp2f(ml[k].x - mmax) : 0.f;
      den += w * ml[k].y;
      num += w * ov[k];
    }
  }
  u16x4 v, v2;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float f = num[e] / den;
    v[e] = out_bits16(f, o_f16);
    v2[e] = out_bits16(f - out_back16(v[e], o_f16), o_f16);
  }
  unsigned short* dst = o + (size_t)qi * ldo + term_pos(oterms, h * D + c);  // four columns inside one group of eight
  *reinterpret_cast<u16x4*>(dst) = v;
  if (oterms == 2) *reinterpret_cast<u16x4*>(dst + 8) = v2;
}

// (cos, sin) of pos[m] * base^(-2j/d) for every node m and pair j: the angle is reduced in double,
// then evaluated in float (|error| ~ 1e-7 rad at any position).
__global__ void k_rope_table(const int32_t* __restrict__ pos, const double* __restrict__ inv_freq, int half,
                             float2* __restrict__ cs) {
  const int m = blockIdx.x, j = threadIdx.x;
  double ang = (double)pos[m] * inv_freq[j];
  const double two_pi = 6.283185307179586476925286766559;
  ang -= two_pi * rint(ang / two_pi);
  float sn, c;
  sincosf((float)ang, &sn, &c);
  cs[(size_t)m * half + j] = make_float2(c, sn);
}

struct AttnArgs {
  const float* part; int ks; size_t part_stride, part_ld; int n_heads, n_kv;
  const float2* cs; int cap; const void* gq; const void* gk; float eps;
  float* att_o; float* att_ml; int Bpad; void* o; int ldo; int oterms; int o_f16; bool f16; int32_t* flags;
};

template <int D, int NG, int NQH, bool F16>
int launch_t(dim3 grid, hipStream_t st, const AttnArgs& a, const SegTable<ATTN_MAX_SEGS>& t) {
  typedef typename Mma16<F16>::T T;
  if (grid.z == 1) {
    const SegTable<1> t1{{t.s[0]}};
    hipLaunchKernelGGL((k_attn_fused<D, NG, NQH, F16, 1>), grid, dim3(64 * NG * NQH), 0, st, t1, a.n_heads, a.n_kv,
                       a.cap, a.part, a.ks, a.part_stride, a.part_ld, a.cs, (const T*)a.gq, (const T*)a.gk, a.eps,
                       a.att_o, a.att_ml, a.Bpad, (unsigned short*)a.o, a.ldo, a.oterms, a.o_f16, a.flags);
  } else {
    hipLaunchKernelGGL((k_attn_fused<D, NG, NQH, F16, ATTN_MAX_SEGS>), grid, dim3(64 * NG * NQH), 0, st, t, a.n_heads,
                       a.n_kv, a.cap, a.part, a.ks, a.part_stride, a.part_ld, a.cs, (const T*)a.gq, (const T*)a.gk,
                       a.eps, a.att_o, a.att_ml, a.Bpad, (unsigned short*)a.o, a.ldo, a.oterms, a.o_f16, a.flags);
  }
  return goose_launch_status();
}

template <int D, int NG, int NQH>
int launch_cfg(dim3 grid, hipStream_t st, const AttnArgs& a, const SegTable<ATTN_MAX_SEGS>& t) {
  return a.f16 ? launch_t<D, NG, NQH, true>(grid, st, a, t) : launch_t<D, NG, NQH, false>(grid, st, a, t);
}

template <int NQH, bool F16>
int launch_wide_t(dim3 grid, hipStream_t st, const AttnArgs& a, const SegTable<ATTN_MAX_SEGS>& t) {
  typedef typename Mma16<F16>::T T;
  if (grid.z == 1) {
    const SegTable<1> t1{{t.s[0]}};
    hipLaunchKernelGGL((k_attn_wide<NQH, F16, 1>), grid, dim3(128 * NQH), 0, st, t1, a.n_heads, a.n_kv, a.cap, a.part,
                       a.ks, a.part_stride, a.part_ld, a.cs, (const T*)a.gq, (const T*)a.gk, a.eps, a.att_o, a.att_ml,
                       a.Bpad, (unsigned short*)a.o, a.ldo, a.oterms, a.o_f16, a.flags);
  } else {
    hipLaunchKernelGGL((k_attn_wide<NQH, F16, ATTN_MAX_SEGS>), grid, dim3(128 * NQH), 0, st, t, a.n_heads, a.n_kv,
                       a.cap, a.part, a.ks, a.part_stride, a.part_ld, a.cs, (const T*)a.gq, (const T*)a.gk, a.eps,
                       a.att_o, a.att_ml, a.Bpad, (unsigned short*)a.o, a.ldo, a.oterms, a.o_f16, a.flags);
  }
  return goose_launch_status();
}
template <int NQH>
int launch_wide(dim3 grid, hipStream_t st, const AttnArgs& a, const SegTable<ATTN_MAX_SEGS>& t) {
  return a.f16 ? launch_wide_t<NQH, true>(grid, st, a, t) : launch_wide_t<NQH, false>(grid, st, a, t);
}

template <int D>
int launch_d(int QT, int ng, dim3 grid, hipStream_t st, const AttnArgs& a, const SegTable<ATTN_MAX_SEGS>& t) {
  // one wavefront per (query tile, key group); at most 8 wavefronts per workgroup
  if (QT == 1) return ng == 4 ? launch_cfg<D, 4, 1>(grid, st, a, t) : launch_cfg<D, 2, 1>(grid, st, a, t);
  if (QT == 2) return ng == 4 ? launch_cfg<D, 4, 2>(grid, st, a, t) : launch_cfg<D, 2, 2>(grid, st, a, t);
  // three and four tiles: the kernel that stages the key blocks through LDS (head size 128)
  if constexpr (D == 128) {
    if (QT == 3) return launch_wide<3>(grid, st, a, t);
    return launch_wide<4>(grid, st, a, t);
  }
  if (QT == 3) return launch_cfg<D, 2, 3>(grid, st, a, t);
  return launch_cfg<D, 2, 4>(grid, st, a, t);
}

template <bool F16>
int launch_merge(dim3 grid, int head_dim, hipStream_t st, const AttnArgs& a, int splits,
                 const SegTable<ATTN_MAX_SEGS>& t) {
  typedef typename Mma16<F16>::T T;
  if (grid.z == 1) {
    const SegTable<1> t1{{t.s[0]}};
    hipLaunchKernelGGL((k_attn_merge<F16, 1>), grid, dim3(256), 0, st, a.att_o, a.att_ml, splits, a.Bpad, head_dim,
                       (unsigned short*)a.o, a.ldo, a.oterms, a.o_f16, t1);
  } else {
    hipLaunchKernelGGL((k_attn_merge<F16, ATTN_MAX_SEGS>), grid, dim3(256), 0, st, a.att_o, a.att_ml, splits, a.Bpad,
                       head_dim, (unsigned short*)a.o, a.ldo, a.oterms, a.o_f16, t);
  }
  return goose_launch_status();
}

}  // namespace

int launch_rope_table(const int32_t* pos, const double* inv_freq, int B, int head_dim, void* cs, hipStream_t st) {
  hipLaunchKernelGGL(k_rope_table, dim3(B), dim3(head_dim / 2), 0, st, pos, inv_freq, head_dim / 2, (float2*)cs);
  return goose_launch_status();
}

// Key splits per head for a pass over `keys_max` keys: about two 32-key blocks per wavefront
// (4 key groups per workgroup), but never more workgroups than compute units.  Measured: a
// workgroup's fixed cost (projection slices, rotation, merge) and its LDS footprint (one or two
// workgroups per compute unit) make a second round of workgroups cost more than longer splits
// -- 7B P=16384 B=128: 93 us at 8 splits, 143 us at 32; 33B P=4096: 56 us at 4, 88 us at 17.
int pick_attn_splits(int n_heads, int keys_max, int max_splits) {
  const int blocks = (keys_max + 31) / 32;
  int s = (blocks + 7) / 8;
  const int fit = 256 / n_heads;
  if (s > fit) s = fit;
  if (s > max_splits) s = max_splits;
  if (s < 1) s = 1;
  return s;
}

int launch_attn_16(int dtype, const float* part, int ks, size_t part_stride, size_t part_ld, const void* cs,
                   int n_heads, int n_kv_heads, int head_dim, int cap, const AttnSeg* segs, int nseg, int splits_or_0,
                   int max_splits, int key_groups, const void* gq, const void* gk, float eps, float* att_o,
                   float* att_ml, int Bpad, void* o, int ldo, int oterms, int o_dtype, int32_t* flags, hipStream_t st) {
  if (dtype != GOOSE_DTYPE_BF16 && dtype != GOOSE_DTYPE_F16) return GOOSE_ERR_ARG;
  if (n_kv_heads < 1 || n_heads % n_kv_heads != 0 || (gq == nullptr) != (gk == nullptr)) return GOOSE_ERR_ARG;
  if (nseg < 1 || nseg > ATTN_MAX_SEGS || max_splits < 1 || (key_groups != 2 && key_groups != 4) || (cap & 31))
    return GOOSE_ERR_ARG;
  if (head_dim != 128 && head_dim != 64) return GOOSE_ERR_SHAPE;
  if ((oterms != 1 && oterms != 2) || (o_dtype != GOOSE_DTYPE_BF16 && o_dtype != GOOSE_DTYPE_F16)) return GOOSE_ERR_ARG;
  const AttnArgs a{part, ks, part_stride, part_ld, n_heads, n_kv_heads, (const float2*)cs, cap, gq, gk, eps,
                   att_o, att_ml, Bpad, o, ldo, oterms, o_dtype == GOOSE_DTYPE_F16 ? 1 : 0, dtype == GOOSE_DTYPE_F16, flags};
  auto tiles_of = [](int B) { return (B + 31) / 32; };
  for (int r = 0; r < nseg; ++r) {
    const AttnSeg& g = segs[r];
    if (g.B < 1 || g.B > GOOSE_MAX_B || g.row0 < 0 || (g.row0 & 31) || g.row0 + tiles_of(g.B) * 32 > Bpad ||
        g.P_max < 0 || g.P_max + g.B > cap || !g.kc || !g.vc || !g.dP || !g.mask)
      return GOOSE_ERR_ARG;
  }
  // one launch per class of tree size (1 to 4 query tiles): the class fixes the workgroup shape
  for (int cls : {1, 2, 3, 4}) {
    SegTable<ATTN_MAX_SEGS> t{};
    int n = 0, keys_max = 0, b_max = 0;
    for (int r = 0; r < nseg; ++r) {
      const AttnSeg& g = segs[r];
      if (tiles_of(g.B) != cls) continue;
      t.s[n++] = SegDev{g.row0, g.B, g.P_max, g.kc, g.vc, g.dP, g.mask};
      keys_max = g.P_max + g.B > keys_max ? g.P_max + g.B : keys_max;
      b_max = g.B > b_max ? g.B : b_max;
    }
    if (n == 0) continue;
    int splits = splits_or_0 > 0 ? splits_or_0 : pick_attn_splits(n_heads * n, keys_max, max_splits);
    if (splits > max_splits) splits = max_splits;
    const dim3 grid(n_heads, splits, n);
    int rc = head_dim == 128 ? launch_d<128>(cls, key_groups, grid, st, a, t) : launch_d<64>(cls, key_groups, grid, st, a, t);
    if (rc != GOOSE_OK) return rc;
    if (splits == 1) continue;
    const int rows_per_wg = 1024 / head_dim;
    const dim3 mgrid(n_heads, (b_max + rows_per_wg - 1) / rows_per_wg, n);
    rc = a.f16 ? launch_merge<true>(mgrid, head_dim, st, a, splits, t)
               : launch_merge<false>(mgrid, head_dim, st, a, splits, t);
    if (rc != GOOSE_OK) return rc;
  }
  return GOOSE_OK;
}
