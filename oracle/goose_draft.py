"""CPU oracle for the draft side of Goose and its decoding loop.  TEST INFRASTRUCTURE ONLY.

Plain Python statements of: the context n-gram match (App. B.2, text after Alg. "Decoding Loop"),
the budget split and the spine tree (Sec. 4.1, Alg. BuildSpineTree), the spine-ratio tiers and
their moving average (Sec. 4.3; App. C hyperparameter table), and the loop that ties them to
verification and harvest (Alg. "Decoding Loop").  Shares no code with the C++ implementation; the
product never imports it.

Only tier 1 of the adjacency table (one-token context, dense [vocab][K] ids and scores) is
modelled; the two-token hash tier and the score-proportional re-weighting of branch widths
(App. C) are not.

Readings where the paper leaves room:
  * context match: for every n in the query lengths, the MOST RECENT earlier occurrence of the
    sequence's last n tokens; the draft chain is the continuation after the match of the largest
    n that matched, at most `max_len` tokens, never running past the end of the sequence;
    consensus = at least two of the n's matched and two of them agree on the first continuation
    token;
  * successors of a token = its table row in stored order, entries with id < 0 or score below
    the minimum score dropped;
  * attachment skips a successor that is already a child of the node (this covers the spine
    continuation d_{i+1}); fewer successors than allocated simply leave budget over;
  * step 4: leaves are visited breadth-first in creation order; each visit appends the leaf's
    best not-yet-present successor as its only child while budget remains; a branch node attached
    to the root or the spine has branch depth 1 and nothing is appended below branch depth D;
  * node order = creation order: root, spine, root branches, spine branches by spine position,
    then step-4 nodes (this is a topological order);
  * moving average: p <- (1 - alpha) * p + alpha * (accepted spine nodes / spine nodes offered),
    on every cycle that offered spine nodes (tree or bypass).
"""
from __future__ import annotations

import math

import numpy as np

from . import goose_oracle as orc


# --------------------------------------------------------------------------- context match
def context_match(seq, lens=(3, 4, 5), max_len=20):
    """Returns (draft chain as a list, consensus flag)."""
    seq = [int(t) for t in seq]
    L = len(seq)
    found = {}
    for n in lens:
        if L < n + 1:
            continue
        tail = seq[L - n:]
        for j in range(L - n - 1, -1, -1):          # most recent earlier occurrence first
            if seq[j:j + n] == tail:
                cont = seq[j + n:j + n + max_len]
                if cont:
                    found[n] = cont
                break
    if not found:
        return [], False
    firsts = [c[0] for c in found.values()]
    consensus = any(firsts.count(f) >= 2 for f in firsts)
    return found[max(found)], consensus


# --------------------------------------------------------------------------- tree
def spine_budget(B, m, r, rho):
    """(b_s, b_r, b_rho) of Alg. BuildSpineTree: spine nodes, root-level and spine-level branch counts."""
    b_s = min(int(m), int(math.floor(B * r)))
    b_r = int(math.floor((B - 1 - b_s) * (1.0 - rho)))
    b_rho = B - 1 - b_s - b_r
    return b_s, b_r, b_rho


def harmonic_allocation(b_rho, b_s):
    """a_i = floor(b_rho * (1/i) / H_{b_s}), i = 1..b_s (step 3 of Alg. BuildSpineTree)."""
    H = sum(1.0 / j for j in range(1, b_s + 1))
    return [int(math.floor(b_rho * (1.0 / i) / H)) for i in range(1, b_s + 1)]


def successors(table_ids, table_scores, token, min_score):
    return [int(s) for s, p in zip(table_ids[token], table_scores[token]) if s >= 0 and p >= min_score]


def build_spine_tree(anchor, draft, table_ids, table_scores, B, r, rho=0.5, D=6, min_score=0.01):
    """Returns (tokens, parent, is_spine) as lists; node 0 is the anchor."""
    b_s, b_r, b_rho = spine_budget(B, len(draft), r, rho)
    tokens, parent, is_spine = [int(anchor)], [-1], [1]
    bdepth = [0]                                     # branch depth; 0 on the spine
    children = [[]]

    def add(p, tok, spine, bd):
        tokens.append(int(tok)); parent.append(p); is_spine.append(spine); bdepth.append(bd)
        children.append([])
        children[p].append(int(tok))
        return len(tokens) - 1

    def attach(p, count, bd):
        new = []
        for s in successors(table_ids, table_scores, tokens[p], min_score):
            if len(new) == count or len(tokens) == B:
                break
            if s in children[p]:
                continue
            new.append(add(p, s, 0, bd))
        return new

    for i in range(b_s):                             # step 1: the spine
        add(i, draft[i], 1, 0)
    leaves = attach(0, b_r, 1)                       # step 2: root branches
    if b_s:
        alloc = harmonic_allocation(b_rho, b_s)
        for i in range(1, b_s + 1):                  # step 3: spine branches
            leaves += attach(i, alloc[i - 1], 1)
    queue = list(leaves)                             # step 4: breadth-first extension
    while queue and len(tokens) < B:
        v = queue.pop(0)
        if bdepth[v] >= D:
            continue
        queue += attach(v, 1, bdepth[v] + 1)
    return tokens, parent, is_spine


# --------------------------------------------------------------------------- adaptation
def spine_ratio_tier(p):
    return 0.15 if p < 0.2 else (0.30 if p < 0.4 else 0.50)


def ema_update(p, accepted_spine, offered_spine, alpha=0.3):
    if offered_spine <= 0:
        return p
    return (1.0 - alpha) * p + alpha * (accepted_spine / offered_spine)


# --------------------------------------------------------------------------- decoding loop
def goose_decode(model, prompt, n_new, B=60, K=10, rho=0.5, D=6, min_score=0.01, bypass_len=8,
                 lens=(3, 4, 5), max_spine=20, trace=None):
    """Alg. "Decoding Loop" on the oracle model.  Returns the generated tokens (at least n_new).
    `trace`, if a list, receives one dict per cycle (mode, tree, accepted, bonus, p_hat)."""
    V = model.lm_head.shape[0]
    ids = np.full((V, K), -1, np.int32)
    scores = np.zeros((V, K))
    prompt = [int(t) for t in prompt]
    logits, new_kv = orc.masked_forward(model, orc.empty_cache(model), prompt, np.arange(len(prompt)),
                                        np.tril(np.ones((len(prompt), len(prompt)), bool)))
    cache = new_kv
    ids, scores = orc.harvest_topk(logits, prompt, K, ids, scores)
    anchor = int(orc.argmax_lowest(logits[-1:])[0])
    y = [anchor]
    p_hat = 0.3
    while len(y) < n_new:
        draft, consensus = context_match(prompt + y, lens, max_spine)
        if draft and (len(draft) >= bypass_len or consensus):
            mode = "bypass"
            tokens = [anchor] + draft
            parent = list(range(-1, len(draft)))
            is_spine = [1] * len(tokens)
        elif draft or successors(ids, scores, anchor, min_score):
            mode = "tree"
            tokens, parent, is_spine = build_spine_tree(anchor, draft, ids, scores, B, spine_ratio_tier(p_hat), rho,
                                                        D, min_score)
        else:
            mode = "ar"
            tokens, parent, is_spine = [anchor], [-1], [1]
        out = orc.verify_step(model, cache, np.asarray(tokens), np.asarray(parent), np.asarray(is_spine))
        ids, scores = orc.harvest_topk(out["logits"], tokens, K, ids, scores)
        offered = sum(is_spine) - 1
        acc_spine = sum(1 for v in out["accepted"] if is_spine[v])
        p_hat = ema_update(p_hat, acc_spine, offered)
        cache = out["cache"]
        y += [int(tokens[v]) for v in out["accepted"]] + [int(out["bonus"])]
        anchor = int(out["bonus"])
        if trace is not None:
            trace.append({"mode": mode, "tokens": tokens, "parent": parent, "is_spine": is_spine,
                          "accepted": list(out["accepted"]), "bonus": anchor, "p_hat": p_hat})
    return y
