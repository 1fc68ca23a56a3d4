/*
 * goose.h -- C ABI of the tree-verification library for MI355X (gfx950).
 *
 * One call sequence verifies one draft tree in one pass of the target model
 * (Goose, Sec. 4, stage 2 "one forward pass scores every candidate" and stage 3
 * "greedy walk"; Alg. UnifiedGreedyWalk):
 *
 *   goose_build_mask  ->  goose_embed  ->  goose_verify_layer x n_layers
 *   ->  goose_lm_head_argmax  ->  goose_accept  ->  goose_compact_kv
 *
 * goose_verify_step runs that whole sequence from device-resident inputs.
 *
 * Conventions for every call
 *   - returns GOOSE_OK (0) or a negative goose_status; never throws, never aborts;
 *   - `d_*` arguments are DEVICE pointers owned by the caller (the library never
 *     frees or reallocates them); `h_*` arguments are HOST pointers;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); work is
 *     queued on it and results are valid once the caller has synchronised it;
 *     no call synchronises the device or the stream;
 *   - a goose_ctx owns device workspace only.  One ctx serves one stream at a time:
 *     calls on the same ctx from different streams race on that workspace.
 *
 * Tree: B nodes in topological order, node 0 = root (the anchor token, which is part of
 * the pass and not yet in the cache), parent[0] = -1, 0 <= parent[i] < i, 1 <= B <= 128.
 * P = number of committed cache slots (the prefix).  A node sees slots [0,P) plus the
 * slots P+j of the nodes j on its own root path, itself included, and sits at
 * position P + depth (Sec. 4 "tree attention mask": each node attends only to its
 * root-to-node ancestors).
 *
 * Model: pre-norm Llama-style decoder (the architecture the paper evaluates, Sec. 5.1):
 * RMSNorm x*rsqrt(mean(x^2)+eps)*g, rotary embedding on q,k with half-split pairing
 * (j, j+d/2) and angle pos*base^(-2j/d), scores/sqrt(d), softmax, SwiGLU MLP, untied LM
 * head, no biases; optionally grouped-query attention and a per-head norm of q and k (the
 * other model families of Sec. 5.1).  Raw weight matrices are row-major [out][in].
 *
 * Storage types.  desc.dtype selects the storage type T of weights, KV cache and gains:
 * GOOSE_DTYPE_BF16 or GOOSE_DTYPE_F16 (the precision the paper runs in, App. C; both: MFMA
 * kernels on 16-bit operands, fp32 accumulation) or GOOSE_DTYPE_F32 (plain fp32 kernels for
 * small models).  The residual stream x is always fp32 [B][hidden].
 *
 * KV cache: two allocations of n_layers * n_kv_heads * cap * head_dim elements each, one KV head's
 * cap * head_dim elements contiguous, cap a multiple of 64.  K is stored after the rotary embedding.
 *   GOOSE_DTYPE_F32:  K[layer][kv head][slot][d];  V TRANSPOSED, Vt[layer][kv head][d][slot].
 *   GOOSE_DTYPE_BF16, GOOSE_DTYPE_F16: both in MFMA OPERAND ORDER, in blocks of 32 slots, so that the attention
 *   kernel streams them with one coalesced 16-byte load per lane and no re-arrangement.
 *   With g = slot, kk = g % 32, c = head-dim column, the element offset inside one head is
 *     K: (((g/32)*(d/16) + c/16)*64 + i + 32*((c/8)%2))*8 + c%8,
 *        i = ((kk/4)%4)*8 + (kk/16)*4 + kk%4      (the MFMA row that carries key kk of a block)
 *     V: ((((g/32)*(d/32) + c/32)*2 + (kk/8)%2)*64 + c%32 + 32*(kk/16))*8 + kk%8.
 * verify_layer writes slots [P, P+B) of its layer, compact_kv rewrites slots [P, P+L] of every
 * layer; slots above P+L hold leftovers afterwards (never read: every kernel masks by P).
 */
#ifndef GOOSE_H
#define GOOSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GOOSE_OK = 0,
  GOOSE_ERR_ARG = -1,             /* NULL pointer or a value out of its documented range */
  GOOSE_ERR_SHAPE = -2,           /* model dimensions the kernels do not support */
  GOOSE_ERR_CAPACITY = -3,        /* B > max_B, or P + B > cap */
  GOOSE_ERR_NOT_TOPOLOGICAL = -4, /* parent array is not a rooted tree in topological order */
  GOOSE_ERR_HIP = -5,             /* a HIP runtime call failed */
  GOOSE_ERR_UNSUPPORTED = -6
} goose_status;

enum { GOOSE_DTYPE_BF16 = 0, GOOSE_DTYPE_F32 = 1, GOOSE_DTYPE_F16 = 2 };
enum { GOOSE_MAX_B = 128 };
/* Most rows (nodes of all requests, each request rounded up to 32) one batched pass may stack. */
enum { GOOSE_MAX_ROWS = 512 };

typedef struct {
  int32_t n_layers, hidden, n_heads, head_dim, ffn, vocab;
  float rope_base, rms_eps;
  int32_t dtype;      /* GOOSE_DTYPE_* */
  int32_t n_kv_heads; /* key/value heads; 0 = n_heads.  Must divide n_heads: query head h reads KV head
                         h / (n_heads / n_kv_heads) (grouped-query attention; 16-bit models only) */
  int32_t qk_norm;    /* != 0: RMSNorm over head_dim (gains gq, gk, eps = rms_eps) on every head of q and k
                         before the rotary embedding (16-bit models only) */
  int32_t act_mode;   /* GOOSE_ACT_* below: how the projections carry their activation operands (16-bit models) */
} goose_model_desc;

/* Activation operands of the projections (the normalised rows, the attention output, the SwiGLU output).
 * Rounding them to bf16 (8 significant bits) is what dominates the logit error of a deep bf16 model; the
 * cached K/V rows, which the storage type does force to 16 bits, contribute ten times less.  Two remedies:
 *   GOOSE_ACT_F16       the operands are fp16 (11 significant bits; the precision the paper runs in, App. C).
 *                       Under bf16 storage the packed copy of every weight matrix then holds each weight w as
 *                       the fp16 value 256 w -- the same number for 2^-32 <= |w| < 256, anything else raises
 *                       GOOSE_FLAG_WEIGHT_RANGE -- the projections run the fp16 matrix instruction and scale
 *                       their fp32 sums by 1/256; KV cache, gains and embedding stay bf16.  An operand beyond
 *                       the fp16 range (65504) is clamped and raises GOOSE_FLAG_RANGE.  Costs nothing.
 *   GOOSE_ACT_TWO_TERM  the operands keep the storage type and carry every value as hi + lo (two 16-bit
 *                       values, 2^-17 relative): bf16's range is kept, each weight piece meets two matrix
 *                       instructions and the small operand doubles in size (about 15 % per step at 64 rows).
 * In both modes the rotated query of the attention keeps two terms as well. */
enum { GOOSE_ACT_F16 = 0, GOOSE_ACT_TWO_TERM = 1 };

/* Raw weights of one decoder layer as a checkpoint stores them: device pointers,
 * row-major [out][in] of the model's storage type. */
typedef struct {
  const void *wq;           /* [n_heads*head_dim][hidden] */
  const void *wk, *wv;      /* [n_kv_heads*head_dim][hidden] */
  const void *wo;           /* [hidden][n_heads*head_dim] */
  const void *wg, *wu;      /* [ffn][hidden] */
  const void *wd;           /* [hidden][ffn] */
  const void *g1, *g2;      /* [hidden] RMSNorm gains before attention / before the MLP */
  const void *gq, *gk;      /* [head_dim] gains of the q / k head norms; read only when desc.qk_norm */
} goose_layer_weights;

typedef struct goose_ctx goose_ctx;

const char* goose_strerror(int status);
/* Text of the most recent failing HIP runtime call in this process ("" if none): which call, which error. */
const char* goose_last_hip_error(void);

/* Creates a context with workspace for trees of up to max_B nodes and caches of `cap`
 * slots per head (a multiple of 64).  Allocates device memory on the current device. */
int goose_create(const goose_model_desc* desc, int max_B, int cap, goose_ctx** out);
/* The same, with workspace for passes of up to max_rows stacked rows (goose_verify_step_batched):
 * max_B <= max_rows <= GOOSE_MAX_ROWS, a multiple of 32.  A request gets the same bits alone and
 * inside any batch (equal attention split counts assumed). */
int goose_create_batched(const goose_model_desc* desc, int max_B, int max_rows, int cap, goose_ctx** out);
void goose_destroy(goose_ctx* ctx);

/* Host-side check of a parent array (h_parent is a HOST pointer): GOOSE_OK,
 * GOOSE_ERR_ARG (NULL, B outside [1,128]) or GOOSE_ERR_NOT_TOPOLOGICAL.
 * The device kernels never fault on a bad array (an offending node is treated as a child
 * of the root) but their result is then meaningless; callers validate trees here. */
int goose_check_parent(const int32_t* h_parent, int B);

/* ---- weight packing (once, at load time) -------------------------------------------
 * The kernels stream weights from a packed copy: for the 16-bit types each matrix is re-tiled so
 * that one wavefront load instruction reads 1 KiB of consecutive bytes that is exactly
 * one MFMA operand (32 output rows x 16 inputs); q,k,v rows are concatenated and
 * gate/up rows interleaved in blocks of 16 (a 32-row tile = the gate rows and the up rows of 16
 * outputs); with bf16 storage and GOOSE_ACT_F16 the packed elements are the fp16 values 256 * w (exact
 * for 2^-32 <= |w| < 256, else GOOSE_FLAG_WEIGHT_RANGE).  For fp32 the blob holds plain row-major
 * matrices.  The caller allocates goose_packed_layer_bytes() per layer; all layers of a
 * model live in one allocation, layer l at byte offset l * goose_packed_layer_bytes(). */
size_t goose_packed_layer_bytes(const goose_ctx* ctx);
int goose_pack_layer(goose_ctx* ctx, const goose_layer_weights* raw, void* d_packed_layer, void* stream);
size_t goose_packed_lm_head_bytes(const goose_ctx* ctx);
/* d_gf: final RMSNorm gain T[hidden]; d_wlm: LM head T[vocab][hidden]. */
int goose_pack_lm_head(goose_ctx* ctx, const void* d_gf, const void* d_wlm, void* d_packed_head, void* stream);

/* ---- 1. ancestor bitmask -------------------------------------------------------------
 * mask[i] = mask[parent[i]] | bit(i), depth[i] = depth[parent[i]] + 1, pos[i] = P + depth[i]
 * (Sec. 4, tree attention mask).  d_mask: uint64 [B][ceil(B/64)], bit (j%64) of word j/64 of
 * row i set iff node j is i or an ancestor of i.  d_depth, d_pos: int32 [B].
 * P is taken from *d_P when d_P is not NULL, else from the argument P. */
int goose_build_mask(goose_ctx* ctx, const int32_t* d_parent, int B, int P, const int32_t* d_P,
                     uint64_t* d_mask, int32_t* d_depth, int32_t* d_pos, void* stream);

/* ---- 2. embedding gather: x[i][:] = fp32(E[tokens[i]][:]).  d_embed: T[vocab][hidden]. */
int goose_embed(goose_ctx* ctx, const void* d_embed, const int32_t* d_tokens, int B, float* d_x, void* stream);

/* ---- 3. one decoder layer over the B packed nodes (Alg. UnifiedGreedyWalk line 1, per layer) ------------
 * d_x fp32 [B][hidden], updated in place.  d_kcache / d_vcache: THIS layer's part of the two
 * cache allocations (n_kv_heads * cap * head_dim elements each, layout above).
 * d_mask/d_pos as written by goose_build_mask.  P from *d_P when d_P != NULL (then the
 * argument P must be an upper bound of *d_P; it sizes the launch), else the argument. */
int goose_verify_layer(goose_ctx* ctx, const void* d_packed_layer, float* d_x, void* d_kcache, void* d_vcache,
                       int P, const int32_t* d_P, int B, const uint64_t* d_mask, const int32_t* d_pos,
                       void* stream);

/* ---- 4. final norm + LM head + per-node argmax (Alg. UnifiedGreedyWalk line 2) ------------------------
 * d_argmax int32 [B]: greedy prediction at every node, lowest index on ties.
 * d_logits_or_null fp32 [B][vocab]; d_margin_or_null fp32 [B] = top-1 minus top-2 logit. */
int goose_lm_head_argmax(goose_ctx* ctx, const void* d_packed_head, const float* d_x, int B, int32_t* d_argmax,
                         float* d_logits_or_null, float* d_margin_or_null, void* stream);

/* The same reduction for callers that cannot allocate device memory (code under stream capture,
 * serving loops and harnesses that forbid it): no context, no allocation, no synchronisation.  The
 * operand rows and the per-workgroup (max, second, index) records that goose_lm_head_argmax keeps in
 * its context's workspace live here in one static 8 MiB device array that every GPU the library
 * runs on holds until the process ends (its address on the current device is looked up on the first
 * call there).  desc: the description the head was packed under (dtype bf16 or fp16; act_mode as at
 * packing); d_packed_head: from goose_pack_lm_head of a context of that description; d_x fp32
 * [B][hidden], untouched; d_argmax int32 [B]; d_margin_or_null fp32 [B].  Results equal
 * goose_lm_head_argmax's bit for bit.  Limits: B <= 128, hidden <= 8192, vocab <= 262144, else
 * GOOSE_ERR_CAPACITY and nothing is launched.  All calls on one GPU share the array: calls that
 * overlap there (two streams, two threads) race; calls queued on one stream do not. */
int goose_lm_head_argmax_static(const goose_model_desc* desc, const void* d_packed_head, const float* d_x, int B,
                                int32_t* d_argmax, float* d_margin_or_null, void* stream);

/* ---- 5. greedy walk (Alg. UnifiedGreedyWalk lines 3-13; Sec. 4.2) -------------------------------------
 * From the root, step to the child whose draft token equals the prediction at the current
 * node; spine-tagged children are examined before branch children, lower node index first
 * within a tag; stop when no child matches.  d_is_spine_or_null: uint8 [B] (NULL = all spine).
 * Outputs: d_accept_len[0] = L (accepted drafts, root and bonus not counted);
 * d_path int32 [B]: path[0] = 0, path[1..L] = accepted nodes, rest = -1;
 * d_bonus[0] = prediction at the last node of the path. */
int goose_accept(goose_ctx* ctx, const int32_t* d_parent, const int32_t* d_tokens, const uint8_t* d_is_spine_or_null,
                 const int32_t* d_argmax, int B, int32_t* d_accept_len, int32_t* d_path, int32_t* d_bonus,
                 void* stream);

/* ---- 6. commit the accepted path to the cache -----------------------------------------
 * For every layer, K and V: slot P + path[j] -> slot P + j, j = 0..L (the root and the
 * accepted nodes become cache slots P..P+L; valid because a node's K was rotated at
 * P + depth and depth(path[j]) = j).  Exact byte copies.  The paper does not describe
 * cache handling; this is the standard commit of tree speculation.
 * d_kcache_all/d_vcache_all: the whole K and V allocations, all layers (layout above).
 * If d_new_P_or_null != NULL it receives P + L + 1 (it may alias d_P). */
int goose_compact_kv(goose_ctx* ctx, void* d_kcache_all, void* d_vcache_all, int P, const int32_t* d_P,
                     const int32_t* d_path, const int32_t* d_accept_len, int32_t* d_new_P_or_null, void* stream);

/* ---- whole step from device-resident inputs (no host round trip inside) --------------
 * Runs 1..6 above.  *d_P is read at the start and replaced by P + L + 1 at the end;
 * P_max is a host upper bound of *d_P used to size launches (P_max + B <= cap).
 * d_next_root_or_null receives the bonus token (e.g. tokens[0] of the next step's tree). */
typedef struct {
  const void* d_embed;         /* T[vocab][hidden] */
  const void* d_packed_layers; /* n_layers * goose_packed_layer_bytes() */
  const void* d_packed_head;
  void* d_kcache_all;
  void* d_vcache_all;
} goose_model_ptrs;

typedef struct {
  const int32_t* d_tokens;   /* [B] */
  const int32_t* d_parent;   /* [B] */
  const uint8_t* d_is_spine; /* [B] or NULL */
  int32_t* d_P;              /* [1] in/out */
  int32_t* d_argmax;         /* [B] out */
  int32_t* d_accept_len;     /* [1] out */
  int32_t* d_path;           /* [B] out */
  int32_t* d_bonus;          /* [1] out */
  int32_t* d_next_root_or_null;
  float* d_logits_or_null;   /* [B][vocab] */
  float* d_margin_or_null;   /* [B] */
  int32_t* d_succ_ids_or_null;    /* [vocab][harvest_k]: harvest this cycle's logits (goose_harvest_topk) */
  float* d_succ_scores_or_null;   /* [vocab][harvest_k], required with d_succ_ids_or_null */
  int32_t harvest_k;              /* 1..16 when harvesting */
} goose_step_io;

int goose_verify_step(goose_ctx* ctx, const goose_model_ptrs* model, const goose_step_io* io, int B, int P_max,
                      void* stream);

/* ---- 6b. several requests in one pass (the batch sweep of App. D: trees of different requests share
 * every weight read; masks, positions, caches and cache lengths stay per request) ---------------
 * The rows of the requests are stacked, each request starting at a multiple of 32 rows; the sum of
 * the rounded-up B must not exceed the context's max_rows (goose_create_batched), each B its max_B.
 * Projections, norms and the LM head run once over all rows (beyond 128 rows in chunks of 128 that
 * share the weight stream through the L2 cache); the attention runs on every request's own caches
 * as one launch per tree-size class; walk, compaction and the optional harvest (into the request's own
 * successor tables) run per request.  16-bit models only.
 * d_argmax_all: int32 [max_rows], receives every row's prediction (request r's rows start
 * at the sum of round_up(B, 32) of the requests before it).  All pointers DEVICE; P of a request is
 * read from *d_P (P_max: host upper bound, as in goose_verify_step) and updated in place. */
#define GOOSE_MAX_REQUESTS 16
typedef struct {
  const int32_t* d_tokens;   /* [B] */
  const int32_t* d_parent;   /* [B] */
  const uint8_t* d_is_spine; /* [B] or NULL */
  int32_t B;
  int32_t P_max;
  void* d_kcache_all;        /* this request's caches, all layers */
  void* d_vcache_all;
  int32_t* d_P;              /* [1] in/out */
  int32_t* d_accept_len;     /* [1] out */
  int32_t* d_path;           /* [B] out */
  int32_t* d_bonus;          /* [1] out */
  int32_t* d_next_root_or_null;
  int32_t* d_succ_ids_or_null;    /* this request's successor tables [vocab][harvest_k]: harvest the logits */
  float* d_succ_scores_or_null;   /* of its nodes as goose_harvest_topk does; both or neither */
  int32_t harvest_k;              /* 1..16 when harvesting */
} goose_request;
int goose_verify_step_batched(goose_ctx* ctx, const goose_model_ptrs* model, const goose_request* reqs, int n_req,
                              int32_t* d_argmax_all, void* stream);

/* ---- 7. logit harvest (Sec. 4 stage 2 "verify and harvest"; App. C "adjacency table", tier 1, and
 * "logit harvesting"; Alg. "Decoding Loop", the update of the table from all logits of a cycle) ----
 * For every node i < B -- accepted or not -- row d_tokens[i] of the two dense successor tables
 * receives the K most likely next tokens under node i's logits: d_succ_ids int32 [vocab][K], ordered
 * by decreasing logit (equal logits: increasing id), and d_succ_scores f32 [vocab][K], their softmax
 * probabilities.  When several nodes carry the same token the highest node index wins; rows of other
 * tokens are untouched; a token outside [0, vocab) writes nothing.  d_logits: f32 [B][ld] DEVICE,
 * ld >= vocab.  1 <= K <= 16 (the paper uses 10).  The tier-2 (two-token context) table is host-side
 * hashing and not part of this library. */
int goose_harvest_topk(goose_ctx* ctx, const float* d_logits, size_t ld, const int32_t* d_tokens, int B, int K,
                       int32_t* d_succ_ids, float* d_succ_scores, void* stream);

/* ---- 8. the draft side of a cycle (HOST functions on HOST memory; no GPU work) ---------------
 * goose_context_match (the n-gram lookup described under Alg. "Decoding Loop", App. B.2): for every
 * query length n in h_lens, the most recent earlier occurrence of the last n tokens of h_seq; the
 * draft chain is the continuation after the match of the largest n that matched (at most max_len
 * tokens, never past the end of the sequence); *h_consensus = 1 iff at least two lengths matched
 * and two of them agree on the first continuation token.  h_draft: [max_len], *h_m tokens valid.
 *
 * goose_spine_budget: lines 1-3 of Alg. BuildSpineTree (b_s spine nodes, b_r root branches, b_rho
 * spine-level branches) in double precision.
 *
 * goose_build_spine_tree: Alg. BuildSpineTree on the one-token successor tables (host mirror of
 * what goose_harvest_topk writes: ids int32 [vocab][K], scores f32 [vocab][K]).  Node 0 is the
 * anchor; creation order (root, spine, root branches, spine branches by spine position with the
 * harmonic allocation floor(b_rho * (1/i) / H_{b_s}), then the breadth-first extension) is the node
 * order and is topological.  A successor is skipped if its id < 0, its score < min_score, or its
 * token is already a child of the node (this covers the spine continuation); the extension visits
 * branch leaves first-in first-out and appends one successor per visit while budget remains, down
 * to branch depth D.  Outputs: h_tokens/h_parent/h_is_spine [B], *h_n <= B nodes written.
 * The two-token table tier and the score-proportional re-weighting of branch widths (App. C) are
 * not implemented.
 *
 * goose_spine_ratio_tier / goose_ema_update: Sec. 4.3 and the hyperparameter table of App. C
 * (tiers 0.15 / 0.30 / 0.50 at 0.2 and 0.4; p <- (1-alpha) p + alpha * accepted/offered, unchanged
 * when no spine node was offered). */
int goose_context_match(const int32_t* h_seq, int n_seq, const int32_t* h_lens, int n_lens, int max_len,
                        int32_t* h_draft, int32_t* h_m, int32_t* h_consensus);
int goose_spine_budget(int B, int m, double r, double rho, int32_t* b_s, int32_t* b_r, int32_t* b_rho);
int goose_build_spine_tree(int32_t anchor, const int32_t* h_draft, int m, const int32_t* h_succ_ids,
                           const float* h_succ_scores, int vocab, int K, int B, double r, double rho, int D,
                           double min_score, int32_t* h_tokens, int32_t* h_parent, uint8_t* h_is_spine,
                           int32_t* h_n);
/* Routing of a cycle (Alg. "Decoding Loop"): a non-empty draft chain that is long (>= bypass_len) or
 * has consensus is verified as a plain chain (bypass); otherwise any draft source gives a spine
 * tree; with none the cycle is one autoregressive step. */
enum { GOOSE_MODE_AR = 0, GOOSE_MODE_TREE = 1, GOOSE_MODE_BYPASS = 2 };
int goose_cycle_mode(int m, int consensus, int bypass_len, int anchor_has_successors);
double goose_spine_ratio_tier(double p_hat);
/* One call for the host side of a cycle (Alg. "Decoding Loop"): the context match on h_seq, the test
 * whether the adjacency table holds a successor of `anchor` with a score >= min_score, the routing
 * (goose_cycle_mode), and the nodes of the pass: the chain anchor + draft for a bypass cycle, the
 * spine tree (goose_build_spine_tree with the spine ratio of goose_spine_ratio_tier(p_hat)) for a
 * tree cycle, the anchor alone otherwise.  h_succ_ids / h_succ_scores: host [vocab][K]; h_tokens,
 * h_parent int32 [B], h_is_spine uint8 [B]; *h_n = nodes written, *h_mode = GOOSE_MODE_*.
 * B >= 1 + max_spine (a bypass chain must fit). */
int goose_plan_cycle(const int32_t* h_seq, int n_seq, const int32_t* h_lens, int n_lens, int max_spine, int32_t anchor,
                     const int32_t* h_succ_ids, const float* h_succ_scores, int vocab, int K, int B, double p_hat,
                     double rho, int D, double min_score, int bypass_len, int32_t* h_tokens, int32_t* h_parent,
                     uint8_t* h_is_spine, int32_t* h_n, int32_t* h_mode);
double goose_ema_update(double p_hat, int accepted_spine, int offered_spine, double alpha);

/* Device-side diagnostics of the calls queued on this context since the last read (the word is then
 * cleared).  Kernels that take the cache length from device memory (d_P) cannot return a status, so
 * they record here what the host checks catch for a host-known P:
 *   GOOSE_FLAG_BAD_PARENT  a parent array that is not a rooted tree in topological order;
 *   GOOSE_FLAG_CAPACITY    *d_P < 0, *d_P > P_max (the bound the launches were sized for), *d_P + B > cap,
 *                          or a commit whose new length would exceed cap.
 * With either bit set the results of that step are meaningless (indices were clamped to stay inside
 * the buffers) and the caches of the offending request must be treated as corrupt.
 * This is the one call that synchronises `stream`. */
/*   GOOSE_FLAG_RANGE        an fp16 activation operand overflowed and was clamped (GOOSE_ACT_F16);
 *   GOOSE_FLAG_WEIGHT_RANGE a weight could not be re-encoded exactly while packing (GOOSE_ACT_F16, bf16 storage). */
enum { GOOSE_FLAG_BAD_PARENT = 1, GOOSE_FLAG_CAPACITY = 2, GOOSE_FLAG_RANGE = 4, GOOSE_FLAG_WEIGHT_RANGE = 8 };
int goose_device_flags(goose_ctx* ctx, void* stream, int32_t* h_flags_out);

/* ---- the projection kernel on its own (unit tests and tuning; dtype = GOOSE_DTYPE_BF16 or _F16) ---
 * out[m][n] = sum_k A[m][k] * W[n][k] for the skinny-M shapes of the pass (M = B <= 128 tree nodes;
 * up to GOOSE_MAX_ROWS stacked rows of a batch, computed in chunks of 128 rows).
 * goose_pack_matrix re-tiles a row-major 16-bit W[N][K] into goose_packed_matrix_bytes(N, K) bytes
 * (N padded to 32, K to 128, zero filled).  goose_gemm_packed multiplies: d_a is 16-bit with
 * round_up(B,32) readable rows (round_up(B,128) when B > 128) of lda >= round_up(K,128) elements
 * (columns K.. and rows B.. must be finite),
 * nw = 2 or 4 column tiles per workgroup, ksplit = split-K factor (every split non-empty).
 * d_partials receives fp32 [ksplit][round_up(B,32)][round_up(N,32)]; the result is the sum over
 * the first index, rows < B (other rows are not written). */
size_t goose_packed_matrix_bytes(int N, int K);
int goose_pack_matrix(const void* d_w, int N, int K, void* d_packed, void* stream);
int goose_gemm_packed(int dtype, const void* d_a, int lda, const void* d_packed, int N, int K, int B, int nw, int ksplit,
                      float* d_partials, void* stream);
/* Same product with the fused SwiGLU epilogue: the N rows of W (N a multiple of 32) alternate in blocks
 * of 16 between gate rows and up rows (rows 32t .. 32t+15 = gate rows 16t .., rows 32t+16 .. 32t+31 = up
 * rows 16t ..); d_h 16-bit [B][ldh] (ldh even, d_h 4-byte aligned) receives silu(gate) * up, N/2 columns. */
int goose_gemm_swiglu_packed(int dtype, const void* d_a, int lda, const void* d_packed, int N, int K, int B, int nw, void* d_h,
                             int ldh, void* stream);
/* The same two products as the decoder layers run them.
 * terms = 2: the activation operand carries every value as the sum of two 16-bit values, hi + lo with
 * lo = T(a - hi) (rounding 2^-17 instead of 2^-9 relative; the kernel feeds both to the matrix cores),
 * stored in groups of eight inputs: inputs 8j..8j+7 occupy elements [16j, 16j+8) (hi) and [16j+8, 16j+16)
 * (lo) of the row; lda >= 2*round_up(K,128).  goose_split_operand writes that layout from fp32 rows
 * (d_src f32 [rows][ld_src], d_dst T [rows][ld_dst], ld_dst a multiple of 16, >= 2*round_up(cols,8);
 * padding columns are zeroed).  With terms = 2 the SwiGLU result is written in the same two-term layout
 * (ldh >= N: two elements per column).  out_scale multiplies every sum before it is used (1 normally). */
int goose_split_operand(int dtype, const float* d_src, int rows, int cols, int ld_src, void* d_dst, int ld_dst,
                        void* stream);
int goose_gemm_packed_ex(int dtype, const void* d_a, int lda, int terms, const void* d_packed, int N, int K, int B,
                         int nw, int ksplit, float out_scale, float* d_partials, void* stream);
int goose_gemm_swiglu_packed_ex(int dtype, const void* d_a, int lda, int terms, const void* d_packed, int N, int K,
                                int B, int nw, float out_scale, void* d_h, int ldh, void* stream);

/* ---- diagnostics: per-kernel timing --------------------------------------------------------
 * While enabled, every kernel launch of verify_layer / lm_head_argmax is bracketed by two
 * hipEvents recorded on the caller's stream (this adds gaps between kernels: use it to time
 * kernels, not whole steps; do not enable it under stream capture).  goose_profile_read
 * synchronises the stream, adds the elapsed milliseconds per kernel kind into
 * h_ms_sum[goose_profile_kinds()] / h_count[...] (HOST arrays) and resets the records.
 * goose_profile_enable creates the events (a pool for 16384 launches between two reads; launches
 * beyond that go untimed), so the timed entry points still create and allocate nothing. */
int goose_profile_enable(goose_ctx* ctx, int enable);
int goose_profile_kinds(void);
const char* goose_profile_kind_name(int kind);
int goose_profile_read(goose_ctx* ctx, void* stream, double* h_ms_sum, int32_t* h_count);

/* Profiling aid: a plain streaming copy of `bytes` (a multiple of 16) from d_src to d_dst, both
 * DEVICE, non-overlapping.  It reads and writes exactly `bytes` of HBM once each, which calibrates
 * hardware traffic counters read for the other kernels in the same profiler run. */
int goose_copy_probe(const void* d_src, void* d_dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GOOSE_H */
