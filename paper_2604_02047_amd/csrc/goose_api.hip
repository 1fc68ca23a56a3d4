// C ABI of the tree-verification library: argument checks, workspace, kernel sequencing.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include <stdio.h>

#include "goose_internal.h"

static char g_last_hip_error[256] = "";

void goose_note_hip_error(hipError_t e, const char* what, int line) {
  snprintf(g_last_hip_error, sizeof(g_last_hip_error), "%s (%d) at %s:%d", hipGetErrorString(e), (int)e, what, line);
}

namespace {

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline bool is16(int dtype) { return dtype == GOOSE_DTYPE_BF16 || dtype == GOOSE_DTYPE_F16; }  // the MFMA path
inline size_t elem_size(int dtype) { return is16(dtype) ? 2 : 4; }

// Launch-shape overrides from the environment exist only in builds made with -DGOOSE_TUNING (a
// development aid: they change split counts, hence summation orders); the library proper reads none.
int env_int(const char* name, int dflt) {
#ifdef GOOSE_TUNING
  const char* v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
#else
  (void)name;
  return dflt;
#endif
}

// ---- optional per-kernel timing with HIP events on the caller's stream -----------------------
enum ProfKind { PK_NORM = 0, PK_GEMM_QKV, PK_ROPE, PK_ATTN, PK_GEMM_O, PK_GEMM_GATE_UP, PK_GEMM_DOWN, PK_LM_HEAD,
                PK_ARGMAX, PK_HARVEST, PK_MISC, PK_COUNT };
const char* const kProfNames[PK_COUNT] = {"rmsnorm_residual", "gemm_qkv", "rope_table", "tree_attention", "gemm_o",
                                          "gemm_gate_up_swiglu", "gemm_down", "gemm_lm_head", "argmax",
                                          "harvest_topk", "mask_embed_accept_compact"};
}  // namespace
enum { GOOSE_PROFILE_POOL = 16384 };  // launches that can be timed between two goose_profile_read calls
struct goose_prof {
  bool on = false;
  std::vector<hipEvent_t> ev;   // pairs: ev[2i] start, ev[2i+1] end
  std::vector<int> kind;        // kind of pair i
  size_t used = 0;              // pairs used since the last read
};
namespace {
struct ProfScope {
  goose_prof* p;
  hipStream_t st;
  ProfScope(goose_ctx* c, int kind, hipStream_t s) : p(c->prof && c->prof->on ? c->prof : nullptr), st(s) {
    if (!p) return;
    if (p->used * 2 >= p->ev.size()) { p = nullptr; return; }  // the pool is used up: not timed (nothing is created here)
    p->kind[p->used] = kind;
    (void)hipEventRecord(p->ev[2 * p->used], st);
  }
  ~ProfScope() {
    if (!p) return;
    (void)hipEventRecord(p->ev[2 * p->used + 1], st);
    ++p->used;
  }
};
#define PROF(kind) ProfScope prof_scope_(c, kind, st)

void compute_layouts(goose_ctx* c) {
  const goose_model_desc& d = c->d;
  const size_t es = elem_size(d.dtype);
  const size_t A = 256;
  size_t off = 0;
  PackedLayout& p = c->pl;
  p.g1 = off; off = round_up_sz(off + (size_t)d.hidden * es, A);
  p.g2 = off; off = round_up_sz(off + (size_t)d.hidden * es, A);
  p.gq = off; off = round_up_sz(off + (size_t)d.head_dim * es, A);
  p.gk = off; off = round_up_sz(off + (size_t)d.head_dim * es, A);
  if (is16(d.dtype)) {
    const size_t f32r = (size_t)round_up(d.ffn, 32);
    p.wqkv = off; off = round_up_sz(off + (size_t)round_up(c->Hq + 2 * c->Hkv, 32) * c->Kh * 2, A);
    p.wo = off;   off = round_up_sz(off + (size_t)round_up(d.hidden, 32) * c->Kq * 2, A);
    p.wgu = off;  off = round_up_sz(off + 2 * f32r * c->Kh * 2, A);
    p.wd = off;   off = round_up_sz(off + (size_t)round_up(d.hidden, 32) * c->Fpad * 2, A);
  } else {
    p.wqkv = off; off = round_up_sz(off + (size_t)3 * c->Hq * d.hidden * 4, A);
    p.wo = off;   off = round_up_sz(off + (size_t)d.hidden * c->Hq * 4, A);
    p.wgu = off;  off = round_up_sz(off + (size_t)2 * d.ffn * d.hidden * 4, A);
    p.wd = off;   off = round_up_sz(off + (size_t)d.hidden * d.ffn * 4, A);
  }
  p.total = off;
  PackedHeadLayout& hl = c->ph;
  hl.gf = 0;
  hl.wlm = round_up_sz((size_t)d.hidden * es, A);
  hl.total = round_up_sz(hl.wlm + (is16(d.dtype) ? (size_t)c->Vpad * c->Kh * 2
                                                               : (size_t)d.vocab * d.hidden * 4), A);
}

int dev_alloc(void** p, size_t bytes) {
  GOOSE_HIP_TRY(hipMalloc(p, bytes));
  GOOSE_HIP_TRY(hipMemset(*p, 0, bytes));
  return GOOSE_OK;
}

int check_tree_args(const goose_ctx* ctx, int B, int P) {
  if (!ctx) return GOOSE_ERR_ARG;
  if (B < 1 || P < 0) return GOOSE_ERR_ARG;
  if (B > ctx->max_B || B > GOOSE_MAX_B) return GOOSE_ERR_CAPACITY;
  if ((long)P + B > ctx->cap) return GOOSE_ERR_CAPACITY;
  return GOOSE_OK;
}

// Workgroup width / split-K of one projection: heuristic, or "nw,ksplit" from the environment (tuning aid).
struct GemmCfg { int nw, ks; };
GemmCfg gemm_cfg(const goose_ctx* c, const char* env_name, int Npad, int Kpad) {
  GemmCfg g;
  pick_gemm_config(Npad, Kpad, c->max_ksplit, c->Bpad, &g.nw, &g.ks);
#ifdef GOOSE_TUNING
  const char* v = getenv(env_name);
  if (v && *v) {
    int nw = 0, ks = 0;
    const int nstages = Kpad / 128;
    if (sscanf(v, "%d,%d", &nw, &ks) == 2 && (nw == 2 || nw == 4) && ks >= 1 && ks <= c->max_ksplit &&
        ks <= nstages && ((nstages + ks - 1) / ks) * (ks - 1) < nstages) {  // no empty split
      g.nw = nw;
      g.ks = ks;
    }
  }
#else
  (void)env_name;
#endif
  return g;
}

// Resolves "P from memory if given, else the host value" to a device pointer.
int resolve_P(goose_ctx* ctx, int P, const int32_t* d_P, hipStream_t st, const int32_t** out) {
  if (d_P) { *out = d_P; return GOOSE_OK; }
  int rc = launch_set_int(ctx->s_P, P, st);
  *out = ctx->s_P;
  return rc;
}

}  // namespace

extern "C" {

const char* goose_last_hip_error(void) { return g_last_hip_error; }

const char* goose_strerror(int status) {
  switch (status) {
    case GOOSE_OK: return "ok";
    case GOOSE_ERR_ARG: return "invalid argument";
    case GOOSE_ERR_SHAPE: return "unsupported model shape";
    case GOOSE_ERR_CAPACITY: return "tree or cache capacity exceeded";
    case GOOSE_ERR_NOT_TOPOLOGICAL: return "parent array is not a tree in topological order";
    case GOOSE_ERR_HIP: return "HIP runtime error";
    case GOOSE_ERR_UNSUPPORTED: return "unsupported";
  }
  return "unknown status";
}

int goose_create(const goose_model_desc* desc, int max_B, int cap, goose_ctx** out) {
  return goose_create_batched(desc, max_B, round_up(max_B, 32), cap, out);
}

int goose_create_batched(const goose_model_desc* desc, int max_B, int max_rows, int cap, goose_ctx** out) {
  if (!desc || !out) return GOOSE_ERR_ARG;
  *out = nullptr;
  if (max_B < 1 || max_B > GOOSE_MAX_B || cap < max_B || (cap % 64) != 0) return GOOSE_ERR_ARG;
  if (max_rows < max_B || max_rows > GOOSE_MAX_ROWS || (max_rows & 31)) return GOOSE_ERR_ARG;
  const goose_model_desc& d = *desc;
  if (d.n_layers < 1 || d.hidden < 1 || d.n_heads < 1 || d.head_dim < 2 || d.ffn < 1 || d.vocab < 1)
    return GOOSE_ERR_ARG;
  if (!is16(d.dtype) && d.dtype != GOOSE_DTYPE_F32) return GOOSE_ERR_ARG;
  if (d.act_mode != GOOSE_ACT_F16 && d.act_mode != GOOSE_ACT_TWO_TERM) return GOOSE_ERR_ARG;
  if (!(d.rope_base > 1.0f) || !(d.rms_eps >= 0.0f)) return GOOSE_ERR_ARG;
  if (d.head_dim % 8 != 0 || d.head_dim > 256) return GOOSE_ERR_SHAPE;
  const int n_kv = d.n_kv_heads > 0 ? d.n_kv_heads : d.n_heads;
  if (n_kv > d.n_heads || d.n_heads % n_kv != 0) return GOOSE_ERR_SHAPE;
  if (is16(d.dtype)) {
    // MFMA kernels: 16-byte vector access to rows, two head sizes
    if (d.head_dim != 64 && d.head_dim != 128) return GOOSE_ERR_SHAPE;
    if (d.hidden % 8 != 0 || d.ffn % 8 != 0) return GOOSE_ERR_SHAPE;
  } else if (n_kv != d.n_heads || d.qk_norm) {
    return GOOSE_ERR_SHAPE;  // the fp32 path is the plain multi-head model only
  }
  goose_ctx* c = new (std::nothrow) goose_ctx();
  if (!c) return GOOSE_ERR_ARG;
  memset(c, 0, sizeof(*c));
  c->d = d;
  c->max_B = max_B;
  c->max_rows = max_rows;
  c->Bpad = max_rows <= 32 ? 32 : (max_rows <= 64 ? 64 : round_up(max_rows, 128));
  c->cap = cap;
  c->Hq = d.n_heads * d.head_dim;
  c->n_kv = n_kv;
  c->Hkv = n_kv * d.head_dim;
  c->Kh = round_up(d.hidden, 128);
  c->Kq = round_up(c->Hq, 128);
  c->Fpad = round_up(d.ffn, 128);
  c->Vpad = round_up(d.vocab, 32);
  c->max_splits = 32;
  c->max_ksplit = 16;
  // 16-bit storage: how the projections carry their activation operands (goose.h, GOOSE_ACT_*)
  c->act_dtype = d.dtype;
  c->terms = 1;
  c->w_exp = 0;
  c->out_scale = 1.0f;
  if (is16(d.dtype)) {
    if (d.act_mode == GOOSE_ACT_TWO_TERM) {
      c->terms = 2;
    } else {
      c->act_dtype = GOOSE_DTYPE_F16;
      if (d.dtype == GOOSE_DTYPE_BF16) { c->w_exp = 8; c->out_scale = 1.0f / 256.0f; }
    }
  }
  compute_layouts(c);

  const size_t es = elem_size(d.dtype);
  size_t widest = (size_t)round_up(c->Hq + 2 * c->Hkv, 32);
  if ((size_t)2 * c->Fpad > widest) widest = (size_t)2 * c->Fpad;
  if ((size_t)c->Kh > widest) widest = c->Kh;
  c->part_ld = widest;
  int rc = GOOSE_OK;
  auto A = [&](void** p, size_t bytes) { if (rc == GOOSE_OK) rc = dev_alloc(p, bytes); };
  A(&c->xn, (size_t)c->Bpad * c->Kh * es * c->terms);
  A((void**)&c->part, (size_t)c->max_ksplit * c->Bpad * c->part_ld * sizeof(float));
  A(&c->q, (size_t)c->Bpad * c->Kq * es);
  A(&c->o, (size_t)c->Bpad * c->Kq * es * c->terms);
  A(&c->h, (size_t)c->Bpad * c->Fpad * es * c->terms);
  A((void**)&c->att_o, (size_t)d.n_heads * c->max_splits * c->Bpad * d.head_dim * sizeof(float));
  A((void**)&c->att_ml, (size_t)d.n_heads * c->max_splits * c->Bpad * 2 * sizeof(float));
  A((void**)&c->logits, (size_t)c->Bpad * c->Vpad * sizeof(float));
  A(&c->top2, (size_t)c->Bpad * (c->Vpad / 64 + 1) * 16);
  A((void**)&c->inv_freq, (size_t)(d.head_dim / 2) * sizeof(double));
  A(&c->rope_cs, (size_t)c->Bpad * (d.head_dim / 2) * 2 * sizeof(float));
  A((void**)&c->s_mask, (size_t)c->Bpad * 2 * sizeof(uint64_t));
  A((void**)&c->s_depth, (size_t)c->Bpad * sizeof(int32_t));
  A((void**)&c->s_pos, (size_t)c->Bpad * sizeof(int32_t));
  A((void**)&c->s_x, (size_t)c->Bpad * d.hidden * sizeof(float));
  A((void**)&c->flags, sizeof(int32_t));
  A((void**)&c->s_P, sizeof(int32_t));
  if (rc == GOOSE_OK) {
    std::vector<double> f(d.head_dim / 2);
    for (int j = 0; j < d.head_dim / 2; ++j) f[j] = pow((double)d.rope_base, -2.0 * j / d.head_dim);
    hipError_t e = hipMemcpy(c->inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice);
    if (e != hipSuccess) { goose_note_hip_error(e, "hipMemcpy(inv_freq)", __LINE__); rc = GOOSE_ERR_HIP; }
  }
  // the zero fills above ran on the null stream; callers use their own streams
  if (rc == GOOSE_OK) {
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) { goose_note_hip_error(e, "hipDeviceSynchronize", __LINE__); rc = GOOSE_ERR_HIP; }
  }
  if (rc != GOOSE_OK) { goose_destroy(c); return rc; }
  *out = c;
  return GOOSE_OK;
}

void goose_destroy(goose_ctx* c) {
  if (!c) return;
  void* ptrs[] = {c->xn, c->part, c->q, c->o, c->h, c->att_o, c->att_ml, c->logits, c->top2, c->inv_freq, c->rope_cs,
                  c->s_mask, c->s_depth, c->s_pos, c->s_x, c->flags, c->s_P};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  if (c->prof) {
    for (hipEvent_t e : c->prof->ev) (void)hipEventDestroy(e);
    delete c->prof;
  }
  delete c;
}

size_t goose_packed_layer_bytes(const goose_ctx* ctx) { return ctx ? ctx->pl.total : 0; }
size_t goose_packed_lm_head_bytes(const goose_ctx* ctx) { return ctx ? ctx->ph.total : 0; }

int goose_pack_layer(goose_ctx* c, const goose_layer_weights* w, void* d_packed, void* stream) {
  if (!c || !w || !d_packed) return GOOSE_ERR_ARG;
  if (!w->wq || !w->wk || !w->wv || !w->wo || !w->wg || !w->wu || !w->wd || !w->g1 || !w->g2) return GOOSE_ERR_ARG;
  hipStream_t st = as_stream(stream);
  const goose_model_desc& d = c->d;
  char* base = (char*)d_packed;
  const size_t es = elem_size(d.dtype);
  const hipMemcpyKind D2D = hipMemcpyDeviceToDevice;
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.g1, w->g1, d.hidden * es, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.g2, w->g2, d.hidden * es, D2D, st));
  if (is16(d.dtype)) {
    if (d.qk_norm) {
      if (!w->gq || !w->gk) return GOOSE_ERR_ARG;
      GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.gq, w->gq, d.head_dim * elem_size(d.dtype), hipMemcpyDeviceToDevice, st));
      GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.gk, w->gk, d.head_dim * elem_size(d.dtype), hipMemcpyDeviceToDevice, st));
    }
    int rc = launch_pack_16(PACK_QKV, w->wq, w->wk, w->wv, c->Hq, d.hidden, round_up(c->Hq + 2 * c->Hkv, 32), c->Kh,
                            base + c->pl.wqkv, st, c->Hkv, c->w_exp, c->flags);
    if (rc) return rc;
    rc = launch_pack_16(PACK_PLAIN, w->wo, nullptr, nullptr, d.hidden, c->Hq, round_up(d.hidden, 32), c->Kq,
                        base + c->pl.wo, st, 0, c->w_exp, c->flags);
    if (rc) return rc;
    rc = launch_pack_16(PACK_GATE_UP, w->wg, w->wu, nullptr, d.ffn, d.hidden, 2 * round_up(d.ffn, 32), c->Kh,
                        base + c->pl.wgu, st, 0, c->w_exp, c->flags);
    if (rc) return rc;
    return launch_pack_16(PACK_PLAIN, w->wd, nullptr, nullptr, d.hidden, d.ffn, round_up(d.hidden, 32), c->Fpad,
                          base + c->pl.wd, st, 0, c->w_exp, c->flags);
  }
  const size_t qb = (size_t)c->Hq * d.hidden * 4, fb = (size_t)d.ffn * d.hidden * 4;
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wqkv, w->wq, qb, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wqkv + qb, w->wk, qb, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wqkv + 2 * qb, w->wv, qb, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wo, w->wo, qb, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wgu, w->wg, fb, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wgu + fb, w->wu, fb, D2D, st));
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->pl.wd, w->wd, fb, D2D, st));
  return GOOSE_OK;
}

int goose_pack_lm_head(goose_ctx* c, const void* d_gf, const void* d_wlm, void* d_packed, void* stream) {
  if (!c || !d_gf || !d_wlm || !d_packed) return GOOSE_ERR_ARG;
  hipStream_t st = as_stream(stream);
  const goose_model_desc& d = c->d;
  char* base = (char*)d_packed;
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->ph.gf, d_gf, d.hidden * elem_size(d.dtype), hipMemcpyDeviceToDevice, st));
  if (is16(d.dtype))
    return launch_pack_16(PACK_PLAIN, d_wlm, nullptr, nullptr, d.vocab, d.hidden, c->Vpad, c->Kh,
                          base + c->ph.wlm, st, 0, c->w_exp, c->flags);
  GOOSE_HIP_TRY(hipMemcpyAsync(base + c->ph.wlm, d_wlm, (size_t)d.vocab * d.hidden * 4, hipMemcpyDeviceToDevice, st));
  return GOOSE_OK;
}

int goose_build_mask(goose_ctx* c, const int32_t* d_parent, int B, int P, const int32_t* d_P, uint64_t* d_mask,
                     int32_t* d_depth, int32_t* d_pos, void* stream) {
  int rc = check_tree_args(c, B, P);
  if (rc) return rc;
  if (!d_parent || !d_mask || !d_depth || !d_pos) return GOOSE_ERR_ARG;
  hipStream_t st = as_stream(stream);
  const int32_t* dP;
  rc = resolve_P(c, P, d_P, st, &dP);
  if (rc) return rc;
  return launch_build_mask(d_parent, B, dP, d_mask, d_depth, d_pos, c->flags, c->cap, d_P ? c->cap - B : P, st);
}

int goose_embed(goose_ctx* c, const void* d_embed, const int32_t* d_tokens, int B, float* d_x, void* stream) {
  if (!c || !d_embed || !d_tokens || !d_x) return GOOSE_ERR_ARG;
  if (B < 1) return GOOSE_ERR_ARG;
  if (B > c->max_B) return GOOSE_ERR_CAPACITY;
  return launch_embed(c->d.dtype, d_embed, d_tokens, B, c->d.hidden, c->d.vocab, d_x, as_stream(stream));
}

// One decoder layer.  `xhat_ready`: the operand buffer already holds RMSNorm(x)*g1 (the previous
// layer's closing kernel wrote it).  `g_next`: gain of the normalisation that follows this layer
// (the next layer's g1 or the final norm), folded into the closing residual add; null to skip.
// A batch of requests shares every projection (their rows are stacked, each request starting at a
// multiple of 32 rows); in the attention every request is a slice of the grid with its own caches,
// mask and length (`segs`; none = the single request given by the plain arguments).
static_assert(GOOSE_MAX_REQUESTS <= ATTN_MAX_SEGS, "a batch must fit the attention's request table");
static int layer_impl(goose_ctx* c, const char* w, float* d_x, void* d_kcache, void* d_vcache, int P,
                      const int32_t* dP, int B, const uint64_t* d_mask, const int32_t* d_pos, hipStream_t st,
                      bool xhat_ready, const void* g_next, const AttnSeg* segs = nullptr, int nseg = 0) {
  int rc = GOOSE_OK;
  const goose_model_desc& d = c->d;
  const size_t pstride = (size_t)c->Bpad * c->part_ld;
  const int H = d.hidden, Hq = c->Hq;

  // x_hat = RMSNorm(x) * g1
  if (!xhat_ready) {
    PROF(PK_NORM);
    rc = launch_resid_norm(d.dtype, c->act_dtype, d_x, H, nullptr, 0, 0, 0, w + c->pl.g1, d.rms_eps, c->xn,
                           c->Kh * c->terms, c->terms, B, st);
  }
  if (rc) return rc;

  if (is16(d.dtype)) {
    const int T = c->terms;
    const int Nqkv = round_up(Hq + 2 * c->Hkv, 32), Nh = round_up(H, 32), Ngu = 2 * round_up(d.ffn, 32);
    static const int splits_env = env_int("GOOSE_ATTN_SPLITS", 0);
    const GemmCfg cq = gemm_cfg(c, "GOOSE_CFG_QKV", Nqkv, c->Kh);
    int ks = cq.ks;
    { PROF(PK_GEMM_QKV);
      rc = launch_gemm_16(c->act_dtype, EPI_PARTIAL, c->xn, c->Kh * T, T, w + c->pl.wqkv, Nqkv, c->Kh, B, cq.nw, ks,
                          c->part, c->part_ld, pstride, c->out_scale, c->flags, st); }
    if (rc) return rc;
    // rotary embedding of q and k, KV rows of the tree into the cache, tree attention: one kernel
    static const int ng_env = env_int("GOOSE_ATTN_NG", 4) == 2 ? 2 : 4;
    const AttnSeg whole{0, B, P, d_kcache, d_vcache, dP, d_mask};
    if (nseg == 0) { segs = &whole; nseg = 1; }
    { PROF(PK_ATTN);
      rc = launch_attn_16(d.dtype, c->part, ks, pstride, c->part_ld, c->rope_cs, d.n_heads, c->n_kv, d.head_dim, c->cap, segs,
                            nseg, splits_env, c->max_splits, ng_env, d.qk_norm ? w + c->pl.gq : nullptr,
                            d.qk_norm ? w + c->pl.gk : nullptr, d.rms_eps, c->att_o, c->att_ml, c->Bpad, c->o, c->Kq * T,
                            T, c->act_dtype, c->flags, st); }
    if (rc) return rc;
    const GemmCfg co = gemm_cfg(c, "GOOSE_CFG_O", Nh, c->Kq);
    ks = co.ks;
    { PROF(PK_GEMM_O);
      rc = launch_gemm_16(c->act_dtype, EPI_PARTIAL, c->o, c->Kq * T, T, w + c->pl.wo, Nh, c->Kq, B, co.nw, ks, c->part,
                          c->part_ld, pstride, c->out_scale, c->flags, st); }
    if (rc) return rc;
    // x += attention projection; x_hat = RMSNorm(x) * g2
    { PROF(PK_NORM);
      rc = launch_resid_norm(d.dtype, c->act_dtype, d_x, H, c->part, ks, pstride, c->part_ld, w + c->pl.g2, d.rms_eps,
                             c->xn, c->Kh * T, T, B, st); }
    if (rc) return rc;
    static const int gu_nw = env_int("GOOSE_GU_NW", 4) == 2 ? 2 : 4;
    { PROF(PK_GEMM_GATE_UP);
      rc = launch_gemm_16(c->act_dtype, EPI_SWIGLU, c->xn, c->Kh * T, T, w + c->pl.wgu, Ngu, c->Kh, B, gu_nw, 1, c->h,
                          (size_t)c->Fpad * T, 0, c->out_scale, c->flags, st); }
    if (rc) return rc;
    const GemmCfg cd = gemm_cfg(c, "GOOSE_CFG_DOWN", Nh, c->Fpad);
    ks = cd.ks;
    { PROF(PK_GEMM_DOWN);
      rc = launch_gemm_16(c->act_dtype, EPI_PARTIAL, c->h, c->Fpad * T, T, w + c->pl.wd, Nh, c->Fpad, B, cd.nw, ks,
                          c->part, c->part_ld, pstride, c->out_scale, c->flags, st); }
    if (rc) return rc;
    // x += MLP output (and the following normalisation when its gain is known)
    PROF(PK_NORM);
    return launch_resid_norm(d.dtype, c->act_dtype, d_x, H, c->part, ks, pstride, c->part_ld, g_next, d.rms_eps,
                             g_next ? c->xn : nullptr, g_next ? c->Kh * T : 0, T, B, st);
  }

  // fp32 storage: plain kernels (one request)
  if (nseg > 1) return GOOSE_ERR_SHAPE;
  const float* xn = (const float*)c->xn;
  rc = launch_gemm_f32(xn, c->Kh, (const float*)(w + c->pl.wqkv), 3 * Hq, H, B, c->part, c->part_ld, st);
  if (rc) return rc;
  rc = launch_rope_kv(d.dtype, c->part, 1, pstride, c->part_ld, B, d.n_heads, d.head_dim, d_pos, c->inv_freq, dP,
                      c->cap, c->q, c->Kq, d_kcache, d_vcache, c->flags, st);
  if (rc) return rc;
  rc = launch_attn_f32((const float*)c->q, c->Kq, (const float*)d_kcache, (const float*)d_vcache, d.n_heads,
                       d.head_dim, c->cap, dP, B, d_mask, (float*)c->o, c->Kq, P, c->flags, st);
  if (rc) return rc;
  rc = launch_gemm_f32((const float*)c->o, c->Kq, (const float*)(w + c->pl.wo), H, Hq, B, c->part, c->part_ld, st);
  if (rc) return rc;
  rc = launch_resid_norm(d.dtype, d.dtype, d_x, H, c->part, 1, pstride, c->part_ld, w + c->pl.g2, d.rms_eps, c->xn, c->Kh,
                         1, B, st);
  if (rc) return rc;
  rc = launch_gemm_f32(xn, c->Kh, (const float*)(w + c->pl.wgu), 2 * d.ffn, H, B, c->part, c->part_ld, st);
  if (rc) return rc;
  rc = launch_swiglu_f32(c->part, c->part_ld, d.ffn, (float*)c->h, c->Fpad, B, st);
  if (rc) return rc;
  rc = launch_gemm_f32((const float*)c->h, c->Fpad, (const float*)(w + c->pl.wd), H, d.ffn, B, c->part, c->part_ld,
                       st);
  if (rc) return rc;
  return launch_resid_norm(d.dtype, d.dtype, d_x, H, c->part, 1, pstride, c->part_ld, g_next, d.rms_eps,
                           g_next ? c->xn : nullptr, g_next ? c->Kh : 0, 1, B, st);
}

int goose_verify_layer(goose_ctx* c, const void* d_packed_layer, float* d_x, void* d_kcache, void* d_vcache, int P,
                       const int32_t* d_P, int B, const uint64_t* d_mask, const int32_t* d_pos, void* stream) {
  int rc = check_tree_args(c, B, P);
  if (rc) return rc;
  if (!d_packed_layer || !d_x || !d_kcache || !d_vcache || !d_mask || !d_pos) return GOOSE_ERR_ARG;
  hipStream_t st = as_stream(stream);
  const int32_t* dP;
  rc = resolve_P(c, P, d_P, st, &dP);
  if (rc) return rc;
  if (is16(c->d.dtype)) {
    PROF(PK_ROPE);
    rc = launch_rope_table(d_pos, c->inv_freq, B, c->d.head_dim, c->rope_cs, st);
    if (rc) return rc;
  }
  return layer_impl(c, (const char*)d_packed_layer, d_x, d_kcache, d_vcache, P, dP, B, d_mask, d_pos, st, false,
                    nullptr);
}

struct HarvestArgs {  // optional harvest of the logits into the successor tables
  const int32_t* tokens = nullptr;
  int K = 0;
  int32_t* ids = nullptr;
  float* scores = nullptr;
  bool keep_logits = false;  // write the logits to the workspace even though nothing is harvested here
};
static int lm_head_impl(goose_ctx* c, const void* d_packed_head, const float* d_x, int B, int32_t* d_argmax,
                        float* d_logits_or_null, float* d_margin_or_null, hipStream_t st, bool xhat_ready,
                        const HarvestArgs& hv);

int goose_lm_head_argmax(goose_ctx* c, const void* d_packed_head, const float* d_x, int B, int32_t* d_argmax,
                         float* d_logits_or_null, float* d_margin_or_null, void* stream) {
  if (!c || !d_packed_head || !d_x || !d_argmax) return GOOSE_ERR_ARG;
  if (B < 1) return GOOSE_ERR_ARG;
  if (B > c->max_B) return GOOSE_ERR_CAPACITY;
  return lm_head_impl(c, d_packed_head, d_x, B, d_argmax, d_logits_or_null, d_margin_or_null, as_stream(stream),
                      false, HarvestArgs());
}

static int lm_head_impl(goose_ctx* c, const void* d_packed_head, const float* d_x, int B, int32_t* d_argmax,
                        float* d_logits_or_null, float* d_margin_or_null, hipStream_t st, bool xhat_ready,
                        const HarvestArgs& hv) {
  const goose_model_desc& d = c->d;
  const char* w = (const char*)d_packed_head;
  // the residual stream is left untouched: normalise into the operand buffer only
  int rc = GOOSE_OK;
  if (!xhat_ready)
    rc = launch_resid_norm(d.dtype, c->act_dtype, const_cast<float*>(d_x), d.hidden, nullptr, 0, 0, 0, w + c->ph.gf,
                           d.rms_eps, c->xn, c->Kh * c->terms, c->terms, B, st);
  if (rc) return rc;
  if (is16(d.dtype)) {
    // the projection kernel reduces its own columns to (max, second, index) per row; logits are
    // written only on request (through the padded workspace when rows are no multiple of a tile)
    static const int lm_nw = env_int("GOOSE_LM_NW", 4) == 2 ? 2 : 4;
    // (the harvest needs them too: into the workspace then)
    const bool bounce = d_logits_or_null && (d.vocab % 32) != 0;
    float* out = (bounce || (!d_logits_or_null && (hv.ids || hv.keep_logits))) ? c->logits : d_logits_or_null;
    const size_t ld = out == c->logits ? (size_t)c->Vpad : (size_t)d.vocab;
    const int groups = (c->Vpad / 32 + lm_nw - 1) / lm_nw;
    { PROF(PK_LM_HEAD);
      rc = launch_gemm_top2_16(c->act_dtype, c->xn, c->Kh * c->terms, c->terms, w + c->ph.wlm, c->Vpad, c->Kh, B, lm_nw, out,
                               ld, c->top2, d.vocab, c->out_scale, st); }
    if (rc) return rc;
    if (bounce)
      GOOSE_HIP_TRY(hipMemcpy2DAsync(d_logits_or_null, (size_t)d.vocab * 4, c->logits, (size_t)c->Vpad * 4,
                                     (size_t)d.vocab * 4, B, hipMemcpyDeviceToDevice, st));
    { PROF(PK_ARGMAX);
      rc = launch_argmax_top2(c->top2, groups, B, d_argmax, d_margin_or_null, st); }
    if (rc || !hv.ids) return rc;
    PROF(PK_HARVEST);
    return launch_harvest_topk(out, ld, d.vocab, hv.tokens, B, hv.K, d.vocab, hv.ids, hv.scores, st);
  }
  float* logits = d_logits_or_null ? d_logits_or_null : c->logits;
  const size_t ld = d_logits_or_null ? (size_t)d.vocab : (size_t)c->Vpad;
  rc = launch_gemm_f32((const float*)c->xn, c->Kh, (const float*)(w + c->ph.wlm), d.vocab, d.hidden, B, logits, ld, st);
  if (rc) return rc;
  rc = launch_argmax(logits, ld, d.vocab, B, d_argmax, d_margin_or_null, st);
  if (rc || !hv.ids) return rc;
  return launch_harvest_topk(logits, ld, d.vocab, hv.tokens, B, hv.K, d.vocab, hv.ids, hv.scores, st);
}

int goose_harvest_topk(goose_ctx* c, const float* d_logits, size_t ld, const int32_t* d_tokens, int B, int K,
                       int32_t* d_succ_ids, float* d_succ_scores, void* stream) {
  if (!c || !d_logits || !d_tokens || !d_succ_ids || !d_succ_scores) return GOOSE_ERR_ARG;
  if (B < 1 || K < 1 || K > 16 || ld < (size_t)c->d.vocab) return GOOSE_ERR_ARG;
  if (B > GOOSE_MAX_B) return GOOSE_ERR_CAPACITY;
  return launch_harvest_topk(d_logits, ld, c->d.vocab, d_tokens, B, K, c->d.vocab, d_succ_ids, d_succ_scores,
                             as_stream(stream));
}

int goose_accept(goose_ctx* c, const int32_t* d_parent, const int32_t* d_tokens, const uint8_t* d_is_spine_or_null,
                 const int32_t* d_argmax, int B, int32_t* d_accept_len, int32_t* d_path, int32_t* d_bonus,
                 void* stream) {
  if (!c || !d_parent || !d_tokens || !d_argmax || !d_accept_len || !d_path || !d_bonus) return GOOSE_ERR_ARG;
  if (B < 1) return GOOSE_ERR_ARG;
  if (B > GOOSE_MAX_B) return GOOSE_ERR_CAPACITY;
  return launch_accept(d_parent, d_tokens, d_is_spine_or_null, d_argmax, B, d_accept_len, d_path, d_bonus, nullptr,
                       as_stream(stream));
}

int goose_compact_kv(goose_ctx* c, void* d_kcache_all, void* d_vcache_all, int P, const int32_t* d_P,
                     const int32_t* d_path, const int32_t* d_accept_len, int32_t* d_new_P_or_null, void* stream) {
  if (!c || !d_kcache_all || !d_vcache_all || !d_path || !d_accept_len) return GOOSE_ERR_ARG;
  if (P < 0 || P >= c->cap) return GOOSE_ERR_CAPACITY;
  hipStream_t st = as_stream(stream);
  const int32_t* dP;
  int rc = resolve_P(c, P, d_P, st, &dP);
  if (rc) return rc;
  const goose_model_desc& d = c->d;
  return launch_compact((int)elem_size(d.dtype), d_kcache_all, d_vcache_all, d.n_layers, c->n_kv, c->cap,
                        d.head_dim, dP, d_path, d_accept_len, d_new_P_or_null, c->flags, st);
}

int goose_verify_step(goose_ctx* c, const goose_model_ptrs* m, const goose_step_io* io, int B, int P_max,
                      void* stream) {
  if (!c || !m || !io) return GOOSE_ERR_ARG;
  int rc = check_tree_args(c, B, P_max);
  if (rc) return rc;
  if (!m->d_embed || !m->d_packed_layers || !m->d_packed_head || !m->d_kcache_all || !m->d_vcache_all)
    return GOOSE_ERR_ARG;
  if (!io->d_tokens || !io->d_parent || !io->d_P || !io->d_argmax || !io->d_accept_len || !io->d_path || !io->d_bonus)
    return GOOSE_ERR_ARG;
  hipStream_t st = as_stream(stream);
  const goose_model_desc& d = c->d;
  rc = launch_build_mask(io->d_parent, B, io->d_P, c->s_mask, c->s_depth, c->s_pos, c->flags, c->cap, P_max, st);
  if (rc) return rc;
  rc = launch_embed(d.dtype, m->d_embed, io->d_tokens, B, d.hidden, d.vocab, c->s_x, st);
  if (rc) return rc;
  if (is16(d.dtype)) {  // the tree's rotary angles, once for all layers
    PROF(PK_ROPE);
    rc = launch_rope_table(c->s_pos, c->inv_freq, B, d.head_dim, c->rope_cs, st);
    if (rc) return rc;
  }
  const size_t layer_cache = (size_t)c->n_kv * c->cap * d.head_dim * elem_size(d.dtype);
  // each layer's closing residual add also writes the next normalisation's output
  for (int l = 0; l < d.n_layers; ++l) {
    const char* w = (const char*)m->d_packed_layers + (size_t)l * c->pl.total;
    const void* g_next = (l + 1 < d.n_layers) ? (const void*)(w + c->pl.total + c->pl.g1)
                                              : (const void*)((const char*)m->d_packed_head + c->ph.gf);
    rc = layer_impl(c, w, c->s_x, (char*)m->d_kcache_all + l * layer_cache, (char*)m->d_vcache_all + l * layer_cache,
                    P_max, io->d_P, B, c->s_mask, c->s_pos, st, l > 0, g_next);
    if (rc) return rc;
  }
  HarvestArgs hv;
  if (io->d_succ_ids_or_null) {
    if (!io->d_succ_scores_or_null || io->harvest_k < 1 || io->harvest_k > 16) return GOOSE_ERR_ARG;
    hv.tokens = io->d_tokens;
    hv.K = io->harvest_k;
    hv.ids = io->d_succ_ids_or_null;
    hv.scores = io->d_succ_scores_or_null;
  }
  rc = lm_head_impl(c, m->d_packed_head, c->s_x, B, io->d_argmax, io->d_logits_or_null, io->d_margin_or_null, st,
                    true, hv);
  if (rc) return rc;
  rc = launch_accept(io->d_parent, io->d_tokens, io->d_is_spine, io->d_argmax, B, io->d_accept_len, io->d_path,
                     io->d_bonus, io->d_next_root_or_null, st);
  if (rc) return rc;
  return launch_compact((int)elem_size(d.dtype), m->d_kcache_all, m->d_vcache_all, d.n_layers, c->n_kv, c->cap,
                        d.head_dim, io->d_P, io->d_path, io->d_accept_len, io->d_P, c->flags, st);
}

int goose_verify_step_batched(goose_ctx* c, const goose_model_ptrs* m, const goose_request* reqs, int n_req,
                              int32_t* d_argmax_all, void* stream) {
  if (!c || !m || !reqs || !d_argmax_all || n_req < 1 || n_req > GOOSE_MAX_REQUESTS) return GOOSE_ERR_ARG;
  if (!m->d_embed || !m->d_packed_layers || !m->d_packed_head) return GOOSE_ERR_ARG;
  const goose_model_desc& d = c->d;
  if (!is16(d.dtype)) return GOOSE_ERR_SHAPE;
  hipStream_t st = as_stream(stream);
  AttnSeg segs[GOOSE_MAX_REQUESTS];
  int rows = 0;
  bool any_harvest = false;
  for (int r = 0; r < n_req; ++r) {
    const goose_request& q = reqs[r];
    int rc = check_tree_args(c, q.B, q.P_max);
    if (rc) return rc;
    if (!q.d_tokens || !q.d_parent || !q.d_P || !q.d_kcache_all || !q.d_vcache_all || !q.d_accept_len || !q.d_path ||
        !q.d_bonus)
      return GOOSE_ERR_ARG;
    if ((q.d_succ_ids_or_null == nullptr) != (q.d_succ_scores_or_null == nullptr)) return GOOSE_ERR_ARG;
    if (q.d_succ_ids_or_null && (q.harvest_k < 1 || q.harvest_k > 16)) return GOOSE_ERR_ARG;
    any_harvest = any_harvest || q.d_succ_ids_or_null != nullptr;
    segs[r] = AttnSeg{rows, q.B, q.P_max, nullptr, nullptr, q.d_P, c->s_mask + (size_t)rows * 2};
    rows += round_up(q.B, 32);
  }
  if (rows > c->max_rows) return GOOSE_ERR_CAPACITY;
  BatchReq br[GOOSE_MAX_REQUESTS];
  int b_max = 0;
  for (int r = 0; r < n_req; ++r) {
    const goose_request& q = reqs[r];
    br[r] = BatchReq{q.d_tokens, q.d_parent, q.d_is_spine, q.B, segs[r].row0, q.P_max, q.d_kcache_all, q.d_vcache_all, q.d_P,
                     q.d_accept_len, q.d_path, q.d_bonus, q.d_next_root_or_null};
    b_max = q.B > b_max ? q.B : b_max;
  }
  int rc = launch_batch_begin(d.dtype, br, n_req, b_max, m->d_embed, d.hidden, d.vocab, c->s_mask, c->s_depth, c->s_pos,
                              c->s_x, c->flags, c->cap, st);
  if (rc) return rc;
  // rows between requests keep stale (finite) values: they ride through the projections unused
  rc = launch_rope_table(c->s_pos, c->inv_freq, rows, d.head_dim, c->rope_cs, st);
  if (rc) return rc;
  const size_t layer_cache = (size_t)c->n_kv * c->cap * d.head_dim * elem_size(d.dtype);
  for (int l = 0; l < d.n_layers; ++l) {
    const char* w = (const char*)m->d_packed_layers + (size_t)l * c->pl.total;
    const void* g_next = (l + 1 < d.n_layers) ? (const void*)(w + c->pl.total + c->pl.g1)
                                              : (const void*)((const char*)m->d_packed_head + c->ph.gf);
    for (int r = 0; r < n_req; ++r) {
      segs[r].kc = (char*)reqs[r].d_kcache_all + l * layer_cache;
      segs[r].vc = (char*)reqs[r].d_vcache_all + l * layer_cache;
    }
    rc = layer_impl(c, w, c->s_x, nullptr, nullptr, 0, nullptr, rows, nullptr, c->s_pos, st, l > 0, g_next, segs, n_req);
    if (rc) return rc;
  }
  HarvestArgs hv;
  hv.keep_logits = any_harvest;
  rc = lm_head_impl(c, m->d_packed_head, c->s_x, rows, d_argmax_all, nullptr, nullptr, st, true, hv);
  if (rc) return rc;
  for (int r = 0; r < n_req && any_harvest; ++r) {  // every request into its own tables, from its rows of the logits
    const goose_request& q = reqs[r];
    if (!q.d_succ_ids_or_null) continue;
    rc = launch_harvest_topk(c->logits + (size_t)segs[r].row0 * c->Vpad, (size_t)c->Vpad, d.vocab, q.d_tokens, q.B,
                             q.harvest_k, d.vocab, q.d_succ_ids_or_null, q.d_succ_scores_or_null, st);
    if (rc) return rc;
  }
  return launch_batch_end(br, n_req, d_argmax_all, d.n_layers, c->n_kv, c->cap, d.head_dim, c->flags, st);
}

// ---- the LM head without a context: its workspace is a static device array --------------------
// For callers that cannot allocate (stream capture, serving loops that forbid it): the operand rows
// and the per-workgroup reductions of goose_lm_head_argmax live in `scratch`, a file-scope device
// array that every GPU this library runs on holds until the process ends.  Its address is looked up
// once per device; calls on one device share the array, so calls that overlap there race.
enum {
  STATIC_MAX_B = 128,
  STATIC_MAX_HIDDEN = 8192,
  STATIC_MAX_VOCAB = 262144,
  STATIC_XN_BYTES = STATIC_MAX_B * STATIC_MAX_HIDDEN * 2 * 2,              // 16-bit rows, up to two terms
  STATIC_TOP2_BYTES = STATIC_MAX_B * (STATIC_MAX_VOCAB / 128) * 16,        // one float4 per row and 128-column group
  STATIC_SCRATCH_BYTES = STATIC_XN_BYTES + STATIC_TOP2_BYTES               // 8 MiB
};
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {
enum { STATIC_MAX_DEVICES = 64 };
void* g_scratch_ptr[STATIC_MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// the current device's copy of `scratch` (each GPU holds its own, at its own address)
int scratch_for_current_device(unsigned char** out) {
  int dev = -1;
  GOOSE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return GOOSE_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    GOOSE_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
  return GOOSE_OK;
}
}  // namespace

int goose_lm_head_argmax_static(const goose_model_desc* desc, const void* d_packed_head, const float* d_x, int B,
                                int32_t* d_argmax, float* d_margin_or_null, void* stream) {
  if (!desc || !d_packed_head || !d_x || !d_argmax) return GOOSE_ERR_ARG;
  const goose_model_desc& d = *desc;
  if (!is16(d.dtype)) return GOOSE_ERR_SHAPE;
  if (d.hidden < 8 || (d.hidden % 8) != 0 || d.vocab < 1 || !(d.rms_eps >= 0.0f)) return GOOSE_ERR_ARG;
  if (d.act_mode != GOOSE_ACT_F16 && d.act_mode != GOOSE_ACT_TWO_TERM) return GOOSE_ERR_ARG;
  if (B < 1) return GOOSE_ERR_ARG;
  if (B > STATIC_MAX_B || d.hidden > STATIC_MAX_HIDDEN || d.vocab > STATIC_MAX_VOCAB) return GOOSE_ERR_CAPACITY;
  // the layout of the packed head and the operand mode, as a context of this description has them (no allocation)
  goose_ctx t;
  memset(&t, 0, sizeof(t));
  t.d = d;
  t.Kh = round_up(d.hidden, 128);
  t.Vpad = round_up(d.vocab, 32);
  t.Hq = d.n_heads * d.head_dim;
  t.n_kv = d.n_kv_heads > 0 ? d.n_kv_heads : d.n_heads;
  t.Hkv = t.n_kv * d.head_dim;
  t.Kq = round_up(t.Hq, 128);
  t.Fpad = round_up(d.ffn, 128);
  compute_layouts(&t);
  const bool two_term = d.act_mode == GOOSE_ACT_TWO_TERM;
  const int terms = two_term ? 2 : 1;
  const int act_dtype = two_term ? d.dtype : GOOSE_DTYPE_F16;
  const float out_scale = (!two_term && d.dtype == GOOSE_DTYPE_BF16) ? 1.0f / 256.0f : 1.0f;
  if (t.Kh > STATIC_MAX_HIDDEN) return GOOSE_ERR_CAPACITY;
  unsigned char* base = nullptr;
  int rc = scratch_for_current_device(&base);
  if (rc) return rc;
  void* xn = base;                       // [round_up(B,32) <= 128][Kh * terms] 16-bit
  void* top2 = base + STATIC_XN_BYTES;   // float4 [B][groups]
  hipStream_t st = as_stream(stream);
  const char* w = (const char*)d_packed_head;
  rc = launch_resid_norm(d.dtype, act_dtype, const_cast<float*>(d_x), d.hidden, nullptr, 0, 0, 0, w + t.ph.gf, d.rms_eps,
                         xn, t.Kh * terms, terms, B, st);
  if (rc) return rc;
  const int lm_nw = 4, groups = (t.Vpad / 32 + lm_nw - 1) / lm_nw;
  rc = launch_gemm_top2_16(act_dtype, xn, t.Kh * terms, terms, w + t.ph.wlm, t.Vpad, t.Kh, B, lm_nw, nullptr, 0, top2,
                           d.vocab, out_scale, st);
  if (rc) return rc;
  return launch_argmax_top2(top2, groups, B, d_argmax, d_margin_or_null, st);
}

int goose_device_flags(goose_ctx* c, void* stream, int32_t* h_flags_out) {
  if (!c || !h_flags_out) return GOOSE_ERR_ARG;
  hipStream_t st = as_stream(stream);
  GOOSE_HIP_TRY(hipMemcpyAsync(h_flags_out, c->flags, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  GOOSE_HIP_TRY(hipStreamSynchronize(st));
  GOOSE_HIP_TRY(hipMemsetAsync(c->flags, 0, sizeof(int32_t), st));
  return GOOSE_OK;
}

// ---- the projection kernel on its own (unit tests, tuning) -----------------------------------
size_t goose_packed_matrix_bytes(int N, int K) {
  if (N < 1 || K < 1) return 0;
  return (size_t)round_up(N, 32) * round_up(K, 128) * 2;
}

int goose_pack_matrix(const void* d_w, int N, int K, void* d_packed, void* stream) {
  if (!d_w || !d_packed || N < 1 || K < 1) return GOOSE_ERR_ARG;
  return launch_pack_16(PACK_PLAIN, d_w, nullptr, nullptr, N, K, round_up(N, 32), round_up(K, 128), d_packed,
                        as_stream(stream));
}

int goose_split_operand(int dtype, const float* d_src, int rows, int cols, int ld_src, void* d_dst, int ld_dst,
                        void* stream) {
  if (!d_src || !d_dst || rows < 1 || cols < 1 || ld_src < cols || !is16(dtype)) return GOOSE_ERR_ARG;
  if (ld_dst < 2 * round_up(cols, 8) || (ld_dst % 16) != 0) return GOOSE_ERR_ARG;
  return launch_split_operand(dtype, d_src, rows, cols, ld_src, d_dst, ld_dst, as_stream(stream));
}

int goose_gemm_swiglu_packed_ex(int dtype, const void* d_a, int lda, int terms, const void* d_packed, int N, int K,
                                int B, int nw, float out_scale, void* d_h, int ldh, void* stream) {
  if (!d_a || !d_packed || !d_h || N < 32 || (N % 32) != 0 || K < 1) return GOOSE_ERR_ARG;
  if (!is16(dtype) || B < 1 || B > GOOSE_MAX_ROWS || (nw != 2 && nw != 4)) return GOOSE_ERR_ARG;
  if (terms != 1 && terms != 2) return GOOSE_ERR_ARG;
  const int Kpad = round_up(K, 128);
  if (lda < Kpad * terms || (lda % 8) != 0 || ldh < N / 2 * terms || (ldh % 2) != 0) return GOOSE_ERR_ARG;
  return launch_gemm_16(dtype, EPI_SWIGLU, d_a, lda, terms, d_packed, N, Kpad, B, nw, 1, d_h, (size_t)ldh, 0, out_scale,
                        nullptr, as_stream(stream));
}

int goose_gemm_swiglu_packed(int dtype, const void* d_a, int lda, const void* d_packed, int N, int K, int B, int nw,
                             void* d_h, int ldh, void* stream) {
  return goose_gemm_swiglu_packed_ex(dtype, d_a, lda, 1, d_packed, N, K, B, nw, 1.0f, d_h, ldh, stream);
}

int goose_gemm_packed_ex(int dtype, const void* d_a, int lda, int terms, const void* d_packed, int N, int K, int B,
                         int nw, int ksplit, float out_scale, float* d_partials, void* stream) {
  if (!d_a || !d_packed || !d_partials || N < 1 || K < 1) return GOOSE_ERR_ARG;
  if (!is16(dtype) || B < 1 || B > GOOSE_MAX_ROWS || (nw != 2 && nw != 4) || ksplit < 1) return GOOSE_ERR_ARG;
  if (terms != 1 && terms != 2) return GOOSE_ERR_ARG;
  const int Npad = round_up(N, 32), Kpad = round_up(K, 128);
  if (lda < Kpad * terms || (lda % 8) != 0) return GOOSE_ERR_ARG;
  const int nstages = Kpad / 128;
  if (ksplit > nstages || ((nstages + ksplit - 1) / ksplit) * (ksplit - 1) >= nstages) return GOOSE_ERR_ARG;
  const int rows = round_up(B, 32);
  return launch_gemm_16(dtype, EPI_PARTIAL, d_a, lda, terms, d_packed, Npad, Kpad, B, nw, ksplit, d_partials,
                        (size_t)Npad, (size_t)rows * Npad, out_scale, nullptr, as_stream(stream));
}

int goose_gemm_packed(int dtype, const void* d_a, int lda, const void* d_packed, int N, int K, int B, int nw, int ksplit,
                      float* d_partials, void* stream) {
  return goose_gemm_packed_ex(dtype, d_a, lda, 1, d_packed, N, K, B, nw, ksplit, 1.0f, d_partials, stream);
}

int goose_copy_probe(const void* d_src, void* d_dst, size_t bytes, void* stream) {
  if (!d_src || !d_dst || bytes < 16 || (bytes % 16) != 0) return GOOSE_ERR_ARG;
  return launch_copy_probe(d_src, d_dst, bytes, as_stream(stream));
}

int goose_profile_enable(goose_ctx* c, int enable) {
  if (!c) return GOOSE_ERR_ARG;
  if (!c->prof) c->prof = new (std::nothrow) goose_prof();
  if (!c->prof) return GOOSE_ERR_ARG;
  // all events are created here, so that the timed entry points themselves create nothing
  if (enable && c->prof->ev.empty()) {
    c->prof->ev.reserve(2 * GOOSE_PROFILE_POOL);
    c->prof->kind.assign(GOOSE_PROFILE_POOL, 0);
    for (int i = 0; i < 2 * GOOSE_PROFILE_POOL; ++i) {
      hipEvent_t e;
      GOOSE_HIP_TRY(hipEventCreate(&e));
      c->prof->ev.push_back(e);
    }
  }
  c->prof->on = enable != 0;
  return GOOSE_OK;
}

int goose_profile_kinds(void) { return PK_COUNT; }

const char* goose_profile_kind_name(int kind) { return (kind >= 0 && kind < PK_COUNT) ? kProfNames[kind] : ""; }

int goose_profile_read(goose_ctx* c, void* stream, double* h_ms_sum, int32_t* h_count) {
  if (!c || !h_ms_sum || !h_count) return GOOSE_ERR_ARG;
  for (int k = 0; k < PK_COUNT; ++k) { h_ms_sum[k] = 0.0; h_count[k] = 0; }
  if (!c->prof) return GOOSE_OK;
  GOOSE_HIP_TRY(hipStreamSynchronize(as_stream(stream)));
  for (size_t i = 0; i < c->prof->used; ++i) {
    float ms = 0.f;
    GOOSE_HIP_TRY(hipEventElapsedTime(&ms, c->prof->ev[2 * i], c->prof->ev[2 * i + 1]));
    h_ms_sum[c->prof->kind[i]] += ms;
    ++h_count[c->prof->kind[i]];
  }
  c->prof->used = 0;
  return GOOSE_OK;
}

}  // extern "C"
