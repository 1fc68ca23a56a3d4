"""CPU oracle for tree verification (Goose, Sec. 4 and Alg. UnifiedGreedyWalk).  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the verification step computes.
It shares no code with the HIP library and must never be imported by the
product path; only tests, the smoke check and the benchmark's CPU-baseline
leg call it.

What is verified (Sec. 1 and Sec. 4, "tree attention mask"; Alg. UnifiedGreedyWalk):
  * the target model scores every node i of a draft tree as if the plain
    sequence  prefix + tokens on the root->i path  had been fed causally;
  * x_hat[i] = argmax of node i's logits (Alg. UnifiedGreedyWalk, greedy prediction per node);
  * a walk from the root follows the child whose draft token equals x_hat of
    the current node (spine child checked before branch children), stops when
    no child matches, and returns the accepted nodes plus the bonus token
    x_hat[last node] (Alg. UnifiedGreedyWalk; Sec. 4.2);
  * the accepted path (root included) becomes the new end of the KV cache.

Two routes to the per-node logits are kept on purpose:
  path_logits_bruteforce : the definition itself, one causal run per node;
  tree_logits            : one packed pass with an ancestor mask and
                           positions P + depth (the method).

The model is a pre-norm Llama-style decoder (the paper runs stock Llama /
Vicuna checkpoints, Sec. 5.1 "Setup"; it prints no model equations, so the
conventions are those of that architecture and are pinned in the tests
against an independent library implementation of it):
RMSNorm x*rsqrt(mean(x^2)+eps)*g, rotary embedding with half-split pairing
(j, j+d/2) and angle pos*base^(-2j/d), scores scaled by 1/sqrt(d), softmax,
SwiGLU MLP  W_d(silu(W_g x) * W_u x), untied LM head, no biases, weights [out,in].
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- model pieces
class OracleModel:
    """Weights as float64 arrays.  `layers[l]` is a dict with wq wk wv wo wg wu wd g1 g2;
    it may be any sequence (also a lazy one) so that large models stream layer by layer."""

    def __init__(self, n_heads, head_dim, rope_base, rms_eps, layers, embed, lm_head, final_norm,
                 n_kv_heads=None, qk_norm=False):
        self.n_heads = int(n_heads)
        self.n_kv_heads = int(n_kv_heads or n_heads)   # grouped-query attention: query head h reads KV head h // group
        self.qk_norm = bool(qk_norm)                   # RMSNorm over head_dim on q and k (gains gq, gk) before RoPE
        self.head_dim = int(head_dim)
        self.rope_base = float(rope_base)
        self.rms_eps = float(rms_eps)
        self.layers = layers
        self.embed = embed
        self.lm_head = lm_head
        self.final_norm = final_norm

    @property
    def n_layers(self):
        return len(self.layers)


def rmsnorm(x, g, eps):
    x = np.asarray(x, F64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def rope(x, pos, base):
    """x [T, n_h, d], pos [T] -> rotated copy.  Pair (j, j+d/2) turns by pos*base^(-2j/d)."""
    T, n_h, d = x.shape
    half = d // 2
    j = np.arange(half, dtype=F64)
    inv_freq = base ** (-2.0 * j / d)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]        # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax_rows(s):
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention(q, K, V, allow):
    """q [T,n_h,d]; K,V [n_kv,S,d] with n_kv dividing n_h (query head h uses KV head h // (n_h/n_kv));
    allow bool [T,S] (True = query t may see slot s) -> [T,n_h,d]."""
    T, n_h, d = q.shape
    group = n_h // K.shape[0]
    out = np.empty_like(q)
    for h in range(n_h):
        s = q[:, h, :] @ K[h // group].T / np.sqrt(F64(d))
        s = np.where(allow, s, -np.inf)
        out[:, h, :] = softmax_rows(s) @ V[h // group]
    return out


def decoder_layer(model, w, x, Kc, Vc, pos, allow):
    """One pre-norm block over T new rows.
    x [T,H]; Kc,Vc [n_kv,P,d] cached (K already rotated); pos [T]; allow [T,P+T].
    Returns (x_out [T,H], k_new [n_kv,T,d] rotated, v_new [n_kv,T,d])."""
    T = x.shape[0]
    n_h, n_kv, d = model.n_heads, model.n_kv_heads, model.head_dim
    xn = rmsnorm(x, w["g1"], model.rms_eps)
    q = (xn @ w["wq"].T).reshape(T, n_h, d)
    k = (xn @ w["wk"].T).reshape(T, n_kv, d)
    v = (xn @ w["wv"].T).reshape(T, n_kv, d)
    if model.qk_norm:                                   # per head, over head_dim, before the rotation
        q = rmsnorm(q, w["gq"], model.rms_eps)
        k = rmsnorm(k, w["gk"], model.rms_eps)
    q = rope(q, pos, model.rope_base)
    k = rope(k, pos, model.rope_base)
    k_new = np.ascontiguousarray(k.transpose(1, 0, 2))
    v_new = np.ascontiguousarray(v.transpose(1, 0, 2))
    K = np.concatenate([Kc, k_new], axis=1)
    V = np.concatenate([Vc, v_new], axis=1)
    o = attention(q, K, V, allow).reshape(T, n_h * d)
    x = x + o @ w["wo"].T
    xn2 = rmsnorm(x, w["g2"], model.rms_eps)
    x = x + (silu(xn2 @ w["wg"].T) * (xn2 @ w["wu"].T)) @ w["wd"].T
    return x, k_new, v_new


def final_logits(model, x):
    return rmsnorm(x, model.final_norm, model.rms_eps) @ model.lm_head.T


def empty_cache(model):
    z = np.zeros((model.n_kv_heads, 0, model.head_dim), F64)
    return [(z.copy(), z.copy()) for _ in range(model.n_layers)]


def masked_forward(model, cache, tokens, pos, allow, return_hidden=False):
    """Rows `tokens` at positions `pos` on top of `cache`; allow [T, P+T].
    Returns (logits [T,V], new_kv = [(k_new,v_new)] per layer[, hidden per layer])."""
    x = np.asarray(model.embed, F64)[np.asarray(tokens, np.int64)]
    new_kv, hidden = [], []
    for l in range(model.n_layers):
        Kc, Vc = cache[l]
        x, k_new, v_new = decoder_layer(model, model.layers[l], x, Kc, Vc, pos, allow)
        new_kv.append((k_new, v_new))
        if return_hidden:
            hidden.append(x.copy())
    logits = final_logits(model, x)
    if return_hidden:
        return logits, new_kv, hidden
    return logits, new_kv


# --------------------------------------------------------------------------- plain causal model
def causal_logits(model, tokens):
    """Textbook causal LM over a plain sequence, no cache: logits [T,V] and its KV."""
    T = len(tokens)
    allow = np.tril(np.ones((T, T), dtype=bool))
    return masked_forward(model, empty_cache(model), tokens, np.arange(T), allow)


def prefill(model, tokens):
    """KV cache of a committed prefix (what a plain causal run of it leaves behind)."""
    if len(tokens) == 0:
        return empty_cache(model)
    _, kv = causal_logits(model, tokens)
    return kv


def greedy_decode(model, prefix, n_new):
    """Plain greedy autoregressive decoding, one token per full causal run."""
    seq = [int(t) for t in prefix]
    out = []
    for _ in range(n_new):
        logits, _ = causal_logits(model, seq)
        t = int(np.argmax(logits[-1]))
        out.append(t)
        seq.append(t)
    return out


# --------------------------------------------------------------------------- tree side
def ancestor_mask(parent):
    """anc[i, j] = True iff j is i or an ancestor of i; depth[i] = edges from the root.
    (Sec. 4: each node attends only to the nodes on its root-to-node path.)"""
    B = len(parent)
    anc = np.zeros((B, B), dtype=bool)
    depth = np.zeros(B, dtype=np.int32)
    for i in range(B):
        v = i
        while v >= 0:
            anc[i, v] = True
            v = int(parent[v])
        depth[i] = int(anc[i].sum()) - 1
    return anc, depth


def mask_words(anc):
    """The B x B ancestor relation as bit words: bit (j % 64) of word j // 64 of row i."""
    B = anc.shape[0]
    W = (B + 63) // 64
    words = np.zeros((B, W), dtype=np.uint64)
    for i in range(B):
        for j in range(B):
            if anc[i, j]:
                words[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return words


def root_path(parent, i):
    p = []
    v = int(i)
    while v >= 0:
        p.append(v)
        v = int(parent[v])
    return p[::-1]


def tree_logits(model, cache, tokens, parent, return_hidden=False):
    """One packed pass over the B nodes: every node sees the whole prefix plus its
    own root path, and sits at position P + depth."""
    P = cache[0][0].shape[1]
    anc, depth = ancestor_mask(parent)
    B = len(parent)
    allow = np.concatenate([np.ones((B, P), dtype=bool), anc], axis=1)
    return masked_forward(model, cache, tokens, P + depth.astype(np.int64), allow, return_hidden)


def path_logits_bruteforce(model, prefix, tokens, parent):
    """The definition: node i's logits are the last-position logits of a plain causal
    run over prefix + (tokens on the root->i path)."""
    B = len(parent)
    rows = []
    for i in range(B):
        seq = [int(t) for t in prefix] + [int(tokens[v]) for v in root_path(parent, i)]
        logits, _ = causal_logits(model, seq)
        rows.append(logits[-1])
    return np.stack(rows)


def argmax_lowest(logits):
    """Per-row argmax; the lowest index wins ties (np.argmax's rule)."""
    return np.argmax(logits, axis=-1).astype(np.int32)


def top2_margin(logits):
    part = np.partition(logits, -2, axis=-1)
    return part[:, -1] - part[:, -2]


def harvest_topk(logits, tokens, K, table_ids=None, table_scores=None, vocab=None):
    """Harvest of a cycle's logits into the unigram successor tables (Sec. 4 stage 2; App. C,
    "adjacency table", tier 1, and "logit harvesting"): for every tree node i -- accepted or not --
    row tokens[i] of the two dense [vocab, K] tables receives the K most likely successors of that
    token according to node i's distribution: their ids, and as scores their softmax probabilities.

    Readings where the paper is silent: entries are ordered by decreasing logit, equal logits by
    increasing token id; when several nodes of the tree carry the same token, the node with the
    highest index writes last and wins; rows of other tokens are left as they were.
    Returns (ids int32 [vocab, K], scores float64 [vocab, K]); fresh tables hold id -1, score 0."""
    logits = np.asarray(logits, F64)
    B, V = logits.shape
    vocab = V if vocab is None else vocab
    ids = np.full((vocab, K), -1, np.int32) if table_ids is None else np.array(table_ids, np.int32)
    scores = np.zeros((vocab, K), F64) if table_scores is None else np.array(table_scores, F64)
    prob = softmax_rows(logits)
    for i in range(B):
        t = int(tokens[i])
        # decreasing logit, then increasing id: sort ids by the pair (-logit, id)
        order = sorted(range(V), key=lambda v: (-logits[i, v], v))[:K]
        ids[t, :] = order
        scores[t, :] = prob[i, order]
    return ids, scores


def greedy_walk(parent, tokens, is_spine, x_hat):
    """The accepted path of a verification pass (Sec. 4.2; what Alg. UnifiedGreedyWalk computes), from its
    definition rather than as a walk:

      * an edge (p -> c) MATCHES when the draft token at c equals the model's greedy prediction at p;
      * among the matching children of a node exactly one is ELECTED: spine-tagged children rank before
        branch children, lower node index first within a tag;
      * a node is ACCEPTED when it is elected and its parent is accepted (the root is accepted by
        definition), so the accepted nodes form one chain from the root;
      * the bonus token is the prediction at the chain's last node.

    Nodes are numbered in topological order (parent[i] < i), so one pass in index order settles every
    node after its parent.  Returns (accepted nodes without the root, in root-to-leaf order; bonus token)."""
    B = len(parent)
    tag = np.ones(B, np.uint8) if is_spine is None else np.asarray(is_spine)
    matches = [i > 0 and int(tokens[i]) == int(x_hat[int(parent[i])]) for i in range(B)]
    rank = [(0 if tag[i] else 1, i) for i in range(B)]                       # spine first, then index
    elected = [matches[i] and all(not matches[j] or rank[i] < rank[j]
                                  for j in range(1, B) if j != i and int(parent[j]) == int(parent[i]))
               for i in range(B)]
    accepted = [True] + [False] * (B - 1)
    for i in range(1, B):
        accepted[i] = elected[i] and accepted[int(parent[i])]
    chain = [i for i in range(1, B) if accepted[i]]                          # index order = depth order on a chain
    last = chain[-1] if chain else 0
    return chain, int(x_hat[last])


def accepted_nodes_bruteforce(parent, tokens, x_hat):
    """All nodes whose every edge from the root matches the model's prediction."""
    B = len(parent)
    ok = np.zeros(B, dtype=bool)
    ok[0] = True
    for i in range(1, B):
        p = int(parent[i])
        ok[i] = ok[p] and int(tokens[i]) == int(x_hat[p])
    return ok


def commit_path(cache, new_kv, path):
    """New cache = old cache followed by the K/V rows of the path nodes, in path order."""
    out = []
    idx = np.asarray(path, dtype=np.int64)
    for (Kc, Vc), (k_new, v_new) in zip(cache, new_kv):
        out.append((np.concatenate([Kc, k_new[:, idx, :]], axis=1),
                    np.concatenate([Vc, v_new[:, idx, :]], axis=1)))
    return out


def verify_step(model, cache, tokens, parent, is_spine, return_hidden=False):
    """One verification cycle.  Returns a dict with everything the GPU path is compared on."""
    res = tree_logits(model, cache, tokens, parent, return_hidden)
    logits, new_kv = res[0], res[1]
    x_hat = argmax_lowest(logits)
    accepted, bonus = greedy_walk(parent, tokens, is_spine, x_hat)
    path = [0] + accepted
    anc, depth = ancestor_mask(parent)
    out = {
        "logits": logits,
        "x_hat": x_hat,
        "margin": top2_margin(logits),
        "accepted": accepted,
        "path": path,
        "bonus": bonus,
        "new_kv": new_kv,
        "cache": commit_path(cache, new_kv, path),
        "anc": anc,
        "depth": depth,
    }
    if return_hidden:
        out["hidden"] = res[2]
    return out
