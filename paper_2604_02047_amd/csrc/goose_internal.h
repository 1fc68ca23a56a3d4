// Internal declarations shared by the library's translation units (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "goose.h"

typedef __bf16 bf16_t;

// Remembers the most recent failing HIP call for goose_last_hip_error() (goose_api.hip).
void goose_note_hip_error(hipError_t e, const char* what, int line);

#define GOOSE_HIP_TRY(expr)                         \
  do {                                              \
    hipError_t e_ = (expr);                         \
    if (e_ != hipSuccess) {                         \
      goose_note_hip_error(e_, #expr, __LINE__);    \
      return GOOSE_ERR_HIP;                         \
    }                                               \
  } while (0)

static inline int goose_launch_status() {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return GOOSE_OK;
  goose_note_hip_error(e, "kernel launch", 0);
  return GOOSE_ERR_HIP;
}

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
static inline size_t round_up_sz(size_t x, size_t m) { return (x + m - 1) / m * m; }

// Byte offsets of the pieces of a packed layer / packed head blob.
struct PackedLayout {
  size_t g1, g2, gq, gk, wqkv, wo, wgu, wd, total;
};
struct PackedHeadLayout {
  size_t gf, wlm, total;
};

struct goose_prof;

struct goose_ctx {
  goose_model_desc d;
  int max_B;     // nodes of one tree, as requested
  int max_rows;  // stacked rows of one pass (a multiple of 32; round_up(max_B, 32) unless created for batches)
  int Bpad;      // 32, 64 or a multiple of 128: row count of every activation buffer
  int cap;     // cache slots per head
  int Hq;      // n_heads * head_dim
  int n_kv;    // key/value heads
  int Hkv;     // n_kv * head_dim
  int Fpad;    // ffn rounded up to 128 -- the K extent of the down projection
  int Kh;      // hidden rounded up to 128
  int Kq;      // Hq rounded up to 128
  int Vpad;    // vocab rounded up to 32
  int max_splits;  // attention key splits the workspace is sized for
  int max_ksplit;  // split-K factor the partial buffer is sized for
  int act_dtype;   // type of the projections' activation operands (xn, o, h): fp16 unless two-term bf16 / fp32
  int terms;       // terms of those operands: 2 in GOOSE_ACT_TWO_TERM mode (hi + lo), else 1
  int w_exp;       // 16-bit weights were packed as fp16 values w * 2^w_exp (0: packed as stored)
  float out_scale; // 2^-w_exp
  PackedLayout pl;
  PackedHeadLayout ph;

  // device workspace
  void* xn;        // T [Bpad][Kh]   normalised activations (GEMM operand)
  float* part;     // f32 [max_ksplit][Bpad][part_ld]   GEMM outputs / split-K partials
  size_t part_ld;  // row length of `part`
  void* q;         // T [Bpad][Kq]   rotated queries
  void* o;         // T [Bpad][Kq]   attention output (GEMM operand)
  void* h;         // T [Bpad][Fpad] SwiGLU output (GEMM operand)
  float* att_o;    // f32 [n_heads][max_splits][Bpad][head_dim]
  float* att_ml;   // f32 [n_heads][max_splits][Bpad][2]
  float* logits;   // f32 [Bpad][Vpad]  (fp32 models; vocabularies that are no multiple of 32)
  void* top2;      // float4 [Bpad][Vpad/64]  per-workgroup reductions of the LM head
  double* inv_freq;  // f64 [head_dim/2]
  void* rope_cs;     // float2 [128][head_dim/2]  (cos, sin) of the current tree's positions
  // scratch for goose_verify_step
  uint64_t* s_mask;  // [128][2]
  int32_t* s_depth;  // [128]
  int32_t* s_pos;    // [128]
  float* s_x;        // [Bpad][hidden]
  int32_t* flags;    // [1]
  int32_t* s_P;      // [1] holds a host-supplied P for kernels that read it from memory
  goose_prof* prof;  // optional per-kernel event timing
};

// ---- small kernels (kernels_small.hip)
int launch_set_int(int32_t* dst, int v, hipStream_t st);
// flags: GOOSE_FLAG_BAD_PARENT for a parent array that is no topological tree, GOOSE_FLAG_CAPACITY
// for a cache length *dP outside [0, P_max] or with *dP + B > cap
int launch_build_mask(const int32_t* parent, int B, const int32_t* dP, uint64_t* mask, int32_t* depth, int32_t* pos,
                      int32_t* flags, int cap, int P_max, hipStream_t st);
int launch_embed(int dtype, const void* E, const int32_t* tokens, int B, int H, int V, float* x, hipStream_t st);
// x[m][:] += sum_s part[s][m][:H] (S may be 0); xn[m][:] = Ta(rmsnorm(x[m]) * g) if xn != NULL, in `terms`
// terms (two: hi + lo in groups of eight columns, the operand layout of the projections; 16-bit types only).
// gain_dtype: type of g; act_dtype: type Ta of xn (equal, or fp16 activations under bf16 gains).
int launch_resid_norm(int gain_dtype, int act_dtype, float* x, int H, const float* part, int S, size_t part_stride,
                      size_t part_ld, const void* g, float eps, void* xn, int ldxn, int terms, int B, hipStream_t st);
// qkv = sum_s part[s][m][0:3Hq]; rotary on q,k; q -> qout, k/v -> cache slots P+m
int launch_rope_kv(int dtype, const float* part, int S, size_t part_stride, size_t part_ld, int B, int n_heads,
                   int head_dim, const int32_t* pos, const double* inv_freq, const int32_t* dP, int cap, void* qout,
                   int ldq, void* kcache, void* vcache, int32_t* flags, hipStream_t st);
int launch_swiglu_f32(const float* gu, size_t ld, int F, float* h, int ldh, int B, hipStream_t st);
int launch_argmax(const float* logits, size_t ld, int V, int B, int32_t* argmax, float* margin, hipStream_t st);
int launch_accept(const int32_t* parent, const int32_t* tokens, const uint8_t* is_spine, const int32_t* argmax, int B,
                  int32_t* accept_len, int32_t* path, int32_t* bonus, int32_t* next_root, hipStream_t st);
// One request of a batched pass as the per-request kernels see it (16-bit storage only).
struct BatchReq {
  const int32_t* tokens;
  const int32_t* parent;
  const uint8_t* is_spine;  // or null
  int32_t B, row0;          // its rows [row0, row0 + B) of the stacked buffers
  int32_t P_max;            // host upper bound of *dP the launches are sized for
  void* kall;               // its caches, all layers
  void* vall;
  int32_t* dP;              // cache length, in/out
  int32_t* accept_len;
  int32_t* path;
  int32_t* bonus;
  int32_t* next_root;       // or null
};
// mask/depth/positions and embedding rows of all requests (2 launches); E: embedding table.
int launch_batch_begin(int dtype, const BatchReq* reqs, int n, int max_B, const void* E, int H, int V,
                       uint64_t* mask, int32_t* depth, int32_t* pos, float* x, int32_t* flags, int cap, hipStream_t st);
// walk, compaction and new cache length of all requests (3 launches)
int launch_batch_end(const BatchReq* reqs, int n, const int32_t* argmax_all, int n_layers, int n_kv_heads, int cap,
                     int head_dim, int32_t* flags, hipStream_t st);
int launch_compact(int elem_bytes, void* kall, void* vall, int n_layers, int n_heads, int cap, int head_dim,
                   const int32_t* dP, const int32_t* path, const int32_t* accept_len, int32_t* new_P, int32_t* flags,
                   hipStream_t st);

// ---- fp32 path (f32_path.hip)
// out[m][n] = sum_k A[m][k] * W[n][k]
int launch_gemm_f32(const float* A, int lda, const float* W, int N, int K, int M, float* out, size_t ldo,
                    hipStream_t st);
int launch_attn_f32(const float* q, int ldq, const float* kc, const float* vc, int n_heads, int head_dim, int cap,
                    const int32_t* dP, int B, const uint64_t* mask, float* o, int ldo, int P_max, int32_t* flags,
                    hipStream_t st);

// ---- the MFMA path: 16-bit storage, dtype = GOOSE_DTYPE_BF16 or GOOSE_DTYPE_F16
// (gemm_bf16.hip, gemm_rows_bf16.hip, attn_bf16.hip: the files are named for the first type built)
enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATE_UP = 2 };
// Re-tiles raw [rows][K] matrices of 16-bit elements into MFMA-operand order; Npad x Kpad zero padded.
// rows_each: rows of s0 (and of s1, s2 unless rows_kv > 0: then s1 and s2 have rows_kv rows each)
// cvt_exp > 0 (bf16 sources only): re-encode every weight as the fp16 value w * 2^cvt_exp (exact for
// 2^(-24-cvt_exp) <= |w| < 65504 / 2^cvt_exp; anything else raises GOOSE_FLAG_WEIGHT_RANGE in *flags)
int launch_pack_16(int mode, const void* s0, const void* s1, const void* s2, int rows_each, int K, int Npad,
                   int Kpad, void* dst, hipStream_t st, int rows_kv = 0, int cvt_exp = 0, int32_t* flags = nullptr);
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_TOP2 = 2 };
// Activation operands come in `terms` = 1 or 2 terms (gemm_bf16.hip): two terms carry a value as hi + lo,
// stored in groups of eight inputs, 8 hi values then their 8 lo values; lda = elements per row = terms * K at least.
// Element offset of input column c in such a row:
static inline __host__ __device__ size_t term_pos(int terms, int c) { return terms == 1 ? (size_t)c : (size_t)(c >> 3) * 16 + (c & 7); }
// silu(g) * u = g / (1 + exp(-g)) * u with the hardware exponential and reciprocal (about one ulp each,
// far inside the 16-bit rounding of the result).  Both projection kernels use this one function, so that
// a request gets the same bits from either.
static __device__ __forceinline__ float swiglu_f32(float g, float u) {
  return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}
// out partials f32 [ksplit][Bpad][ldo] (EPI_PARTIAL) or 16-bit h [Bpad][ldo] in `terms` terms (EPI_SWIGLU, ksplit must be 1).
// out_scale: an exact power of two applied to every sum before the epilogue uses it (1, or the inverse of
// the scale of weights re-encoded by launch_pack_16).  flags (or null): GOOSE_FLAG_RANGE is raised when
// an fp16 SwiGLU result had to be clamped.
int launch_gemm_16(int dtype, int epi, const void* A, int lda, int terms, const void* Wp, int Npad, int Kpad, int B,
                   int nw, int ksplit, void* out, size_t ldo, size_t out_split_stride, float out_scale, int32_t* flags,
                   hipStream_t st);
// The same products for 128 < B <= GOOSE_MAX_ROWS stacked rows, blocked for the matrix cores
// (gemm_rows_bf16.hip); A must hold whole chunks of 128 readable rows.
int launch_gemm_rows_16(int dtype, int epi, const void* A, int lda, int terms, const void* Wp, int Npad, int Kpad, int B,
                        int ksplit, void* out, size_t ldo, size_t out_split_stride, float out_scale, int32_t* flags,
                        hipStream_t st);
// Projection whose workgroups (nw column tiles each) also emit per-row (max, second max, index of
// max) over their valid columns (< n_valid): top2 is float4 [B][ceil(Npad/32/nw)], index bits in .z.
// `out` (f32 [B][ldo]) may be null when only the reduction is wanted.
int launch_gemm_top2_16(int dtype, const void* A, int lda, int terms, const void* Wp, int Npad, int Kpad, int B, int nw,
                        float* out, size_t ldo, void* top2, int n_valid, float out_scale, hipStream_t st);
int launch_harvest_topk(const float* logits, size_t ld, int V, const int32_t* tokens, int B, int K, int table_rows,
                        int32_t* succ_ids, float* succ_scores, hipStream_t st);
int launch_split_operand(int dtype, const float* src, int rows, int cols, int ld_src, void* dst, int ld_dst,
                         hipStream_t st);
int launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st);
int launch_argmax_top2(const void* top2, int n_groups, int B, int32_t* argmax, float* margin, hipStream_t st);
void pick_gemm_config(int Npad, int Kpad, int max_ksplit, int max_rows, int* nw_out, int* ksplit_out);
// (cos, sin) of every node's rotary angles: cs is float2 [B][head_dim/2].
int launch_rope_table(const int32_t* pos, const double* inv_freq, int B, int head_dim, void* cs, hipStream_t st);
// One request's share of an attention launch: its rows [row0, row0 + B) of the stacked projections,
// this layer's operand-ordered caches, its cache length and its ancestor bitmask (words per row =
// ceil(B/64)); P_max bounds *dP and sizes the launch.
struct AttnSeg {
  int32_t row0, B, P_max;
  void* kc;
  void* vc;
  const int32_t* dP;
  const uint64_t* mask;
};
enum { ATTN_MAX_SEGS = 16 };
// Fused rotary embedding + KV-tail write + tree attention of `nseg` requests.  part: the q|k|v
// projection as `ks` split-K slices of f32 [Bpad][part_ld]; cs: rotary table of all rows;
// o: 16-bit [Bpad][ldo] of type o_dtype (which may differ from the caches' type `dtype`) in `oterms` terms
// (the operand layout of the O projection, see launch_gemm_16).
// Requests with the same number of 32-row query tiles share one launch
// (grid z = request).  splits_or_0: key splits per head, 0 = chosen here (at most max_splits).
int launch_attn_16(int dtype, const float* part, int ks, size_t part_stride, size_t part_ld, const void* cs,
                   int n_heads, int n_kv_heads, int head_dim, int cap, const AttnSeg* segs, int nseg, int splits_or_0,
                   int max_splits, int key_groups, const void* gq, const void* gk, float eps, float* att_o,
                   float* att_ml, int Bpad, void* o, int ldo, int oterms, int o_dtype, int32_t* flags, hipStream_t st);
int pick_attn_splits(int n_heads, int keys_max, int max_splits);
