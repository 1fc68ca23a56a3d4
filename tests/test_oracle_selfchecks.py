"""The oracle's pins: what the method must equal by the paper's own statements.

  1. a chain tree is ordinary causal attention (also the bypass mode, Sec. 4.3);
  2. in a star tree a node sees the prefix, the root and itself, never a sibling;
  3. the packed tree pass equals one plain causal run per root-to-node path
     (Sec. 1: every path is scored in one forward pass) -- brute force;
  4. accepted tokens + bonus over several cycles equal plain greedy decoding
     (the lossless property, Sec. 1 and Sec. 5.2 "identical output").
Plus cheap structural checks on the mask, the walk (Alg. UnifiedGreedyWalk) and the KV commit.
"""
import json
import os

import numpy as np
import pytest

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import oracle_model, torch_model

TOL = 1e-9  # fp64 runs of the same sums in a different order


@pytest.fixture(scope="module")
def tiny():
    shape = gi.SHAPES["tiny"]
    om = oracle_model(shape, torch_model(shape, seed=0, gain_jitter=0.1))
    prefix = gi.prefix_tokens(0, 24, shape.vocab)
    return shape, om, prefix, orc.prefill(om, prefix)


# ------------------------------------------------------------------ 1. chain == causal
def test_chain_tree_is_causal_attention(tiny):
    shape, om, prefix, cache = tiny
    tree = gi.tree_chain(9)
    toks = gi.draft_tokens_uniform(1, tree.parent, shape.vocab, 5)
    got, new_kv = orc.tree_logits(om, cache, toks, tree.parent)
    ref, ref_kv = orc.causal_logits(om, np.concatenate([prefix, toks]))
    np.testing.assert_allclose(got, ref[len(prefix):], atol=TOL)
    for (k, v), (rk, rv) in zip(new_kv, ref_kv):
        np.testing.assert_allclose(k, rk[:, len(prefix):], atol=TOL)
        np.testing.assert_allclose(v, rv[:, len(prefix):], atol=TOL)


# ------------------------------------------------------------------ 2. star
def test_star_tree_sees_prefix_root_and_self_only(tiny):
    shape, om, prefix, cache = tiny
    tree = gi.tree_star(7)
    toks = gi.draft_tokens_uniform(2, tree.parent, shape.vocab, 5)
    got, _ = orc.tree_logits(om, cache, toks, tree.parent)
    for i in range(1, tree.B):
        ref, _ = orc.causal_logits(om, np.concatenate([prefix, [toks[0], toks[i]]]))
        np.testing.assert_allclose(got[i], ref[-1], atol=TOL)
    # changing one sibling's token leaves every other node's logits untouched
    toks2 = toks.copy()
    toks2[3] = (toks2[3] + 17) % shape.vocab
    got2, _ = orc.tree_logits(om, cache, toks2, tree.parent)
    keep = [i for i in range(tree.B) if i != 3]
    np.testing.assert_array_equal(got[keep], got2[keep])
    assert np.abs(got[3] - got2[3]).max() > 1e-3


def test_single_node_is_one_decoding_step(tiny):
    shape, om, prefix, cache = tiny
    got, _ = orc.tree_logits(om, cache, np.array([77]), gi.tree_single().parent)
    ref, _ = orc.causal_logits(om, np.concatenate([prefix, [77]]))
    np.testing.assert_allclose(got[0], ref[-1], atol=TOL)


# ------------------------------------------------------------------ 3. brute force
@pytest.mark.parametrize("tree", [gi.tree_tiny_spine(), gi.tree_random(12, 1), gi.tree_random(10, 2, spine_len=4),
                                  gi.tree_balanced(14, (3, 2, 2))], ids=["spine16", "rand12", "rand10", "bal14"])
def test_tree_pass_equals_one_causal_run_per_path(tiny, tree):
    shape, om, prefix, cache = tiny
    toks = gi.draft_tokens_uniform(3, tree.parent, shape.vocab, 9)
    got, _ = orc.tree_logits(om, cache, toks, tree.parent)
    ref = orc.path_logits_bruteforce(om, prefix, toks, tree.parent)
    assert np.abs(ref).max() > 0.05
    np.testing.assert_allclose(got, ref, atol=TOL)


def test_tree_pass_with_empty_prefix(tiny):
    shape, om, _, _ = tiny
    tree = gi.tree_random(8, 5)
    toks = gi.draft_tokens_uniform(4, tree.parent, shape.vocab, 9)
    got, _ = orc.tree_logits(om, orc.empty_cache(om), toks, tree.parent)
    np.testing.assert_allclose(got, orc.path_logits_bruteforce(om, [], toks, tree.parent), atol=TOL)


def test_relabelling_the_tree_permutes_logits(tiny):
    shape, om, prefix, cache = tiny
    tree = gi.tree_random(12, 7, spine_len=3)
    toks = gi.draft_tokens_uniform(5, tree.parent, shape.vocab, 9)
    tree2, perm = gi.relabel_topological(tree, 1)
    assert not np.array_equal(perm, np.arange(tree.B))
    a, _ = orc.tree_logits(om, cache, toks, tree.parent)
    b, _ = orc.tree_logits(om, cache, toks[perm], tree2.parent)
    np.testing.assert_allclose(b, a[perm], atol=TOL)


# ------------------------------------------------------------------ 4. lossless
@pytest.mark.parametrize("planted", [False, True], ids=["random_drafts", "planted_drafts"])
def test_cycles_reproduce_plain_greedy_decoding(tiny, planted):
    shape, om, prefix, cache = tiny
    n_cycles = 5
    greedy = orc.greedy_decode(om, prefix, 1 + n_cycles * 9)
    root = greedy[0]          # the anchor: the prediction after the prefix, not yet in the cache
    emitted = [root]
    P = len(prefix)
    accepted_total = 0
    for cyc in range(n_cycles):
        tree = gi.tree_tiny_spine() if cyc % 2 == 0 else gi.tree_random(16, cyc, spine_len=5)
        toks = gi.draft_tokens_uniform(100 + cyc, tree.parent, shape.vocab, root)
        if planted:
            cont = np.array(greedy[len(emitted):len(emitted) + 8])
            toks = gi.plant_drafts(200 + cyc, tree.parent, tree.is_spine, toks, cont, shape.vocab,
                                   p_spine=0.8, p_branch=0.9, p_grand=0.9)
        r = orc.verify_step(om, cache, toks, tree.parent, tree.is_spine)
        emitted += [int(toks[v]) for v in r["accepted"]] + [r["bonus"]]
        accepted_total += len(r["accepted"])
        cache, root = r["cache"], r["bonus"]
        P += 1 + len(r["accepted"])
        assert cache[0][0].shape[1] == P
    assert emitted == greedy[:len(emitted)]
    if planted:
        assert accepted_total >= 5  # the planted runs really exercise multi-node acceptance
    # the cache the cycles built is the cache of the plain sequence
    ref = orc.prefill(om, list(prefix) + emitted[:-1])
    for (k, v), (rk, rv) in zip(cache, ref):
        np.testing.assert_allclose(k, rk, atol=TOL)
        np.testing.assert_allclose(v, rv, atol=TOL)


# ------------------------------------------------------------------ mask structure
@pytest.mark.parametrize("tree", [gi.tree_tiny_spine(), gi.tree_spine_7b(0), gi.tree_spine_stress(),
                                  gi.tree_balanced(), gi.tree_random(100, 3)],
                         ids=["tiny", "7b", "stress", "balanced", "rand100"])
def test_mask_structure(tree):
    anc, depth = orc.ancestor_mask(tree.parent)
    B = tree.B
    assert np.array_equal(anc & np.triu(np.ones((B, B), bool), 1), np.zeros((B, B), bool))  # sub-mask of causal
    assert anc.diagonal().all() and anc[:, 0].all()
    assert np.array_equal(anc.sum(1) - 1, depth)
    for i in range(1, B):
        p = tree.parent[i]
        assert depth[i] == depth[p] + 1
        only_self = anc[i] & ~anc[p]
        assert only_self.sum() == 1 and only_self[i]
    words = orc.mask_words(anc)
    assert words.shape == (B, (B + 63) // 64)
    for i in range(B):
        bits = [(int(words[i, j // 64]) >> (j % 64)) & 1 for j in range(B)]
        assert bits == anc[i].astype(int).tolist()
        assert sum(bin(int(w)).count("1") for w in words[i]) == depth[i] + 1


def test_chain_and_star_masks_are_the_textbook_ones():
    anc, depth = orc.ancestor_mask(gi.tree_chain(6).parent)
    assert np.array_equal(anc, np.tril(np.ones((6, 6), bool))) and depth.tolist() == [0, 1, 2, 3, 4, 5]
    anc, depth = orc.ancestor_mask(gi.tree_star(5).parent)
    want = np.eye(5, dtype=bool)
    want[:, 0] = True
    assert np.array_equal(anc, want) and depth.tolist() == [0, 1, 1, 1, 1]
    assert orc.mask_words(anc)[:, 0].tolist() == [1, 3, 5, 9, 17]


# ------------------------------------------------------------------ walk
def test_walk_golden_cases():
    with open(os.path.join(os.path.dirname(__file__), "golden", "walk_cases.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        acc, bonus = orc.greedy_walk(np.array(c["parent"]), np.array(c["tokens"]),
                                     np.array(c["is_spine"], np.uint8), np.array(c["x_hat"]))
        assert (acc, bonus) == (c["accepted"], c["bonus"]), c["name"]


def test_walk_equals_deepest_fully_matching_node():
    rng = np.random.default_rng(0)
    hit = 0
    for trial in range(300):
        tree = gi.tree_random(int(rng.integers(1, 40)), trial, spine_len=int(rng.integers(0, 6)))
        vocab = 6  # a small vocabulary makes matches frequent
        B = tree.B
        if max(np.bincount(tree.parent[1:], minlength=B)) > vocab:
            continue
        toks = gi.draft_tokens_uniform(trial, tree.parent, vocab, 0)
        x_hat = rng.integers(0, vocab, B)
        acc, bonus = orc.greedy_walk(tree.parent, toks, tree.is_spine, x_hat)
        ok = orc.accepted_nodes_bruteforce(tree.parent, toks, x_hat)
        _, depth = orc.ancestor_mask(tree.parent)
        deepest = max(np.flatnonzero(ok), key=lambda i: depth[i])
        assert sum(depth[ok] == depth[deepest]) == 1       # distinct siblings: the path is unique
        assert ([0] + acc) == orc.root_path(tree.parent, deepest)
        assert bonus == x_hat[deepest]
        assert [depth[v] for v in acc] == list(range(1, len(acc) + 1))
        # visiting order of children cannot matter when siblings are distinct
        acc2, bonus2 = orc.greedy_walk(tree.parent, toks, 1 - tree.is_spine, x_hat)
        assert (acc2, bonus2) == (acc, bonus)
        hit += len(acc) > 1
    assert hit > 20


# ------------------------------------------------------------------ KV commit
def test_commit_keeps_prefix_and_appends_path_rows(tiny):
    shape, om, prefix, cache = tiny
    tree = gi.tree_tiny_spine()
    toks = gi.draft_tokens_uniform(9, tree.parent, shape.vocab, 3)
    _, new_kv = orc.tree_logits(om, cache, toks, tree.parent)
    path = [0, 1, 2, 10]
    out = orc.commit_path(cache, new_kv, path)
    P = len(prefix)
    for (k, v), (k0, v0), (kn, vn) in zip(out, cache, new_kv):
        assert k.shape[1] == P + 4
        np.testing.assert_array_equal(k[:, :P], k0)
        for j, node in enumerate(path):
            np.testing.assert_array_equal(k[:, P + j], kn[:, node])
            np.testing.assert_array_equal(v[:, P + j], vn[:, node])
    # the committed rows are those of the plain sequence prefix + path tokens
    ref = orc.prefill(om, list(prefix) + [int(toks[n]) for n in path])
    for (k, v), (rk, rv) in zip(out, ref):
        np.testing.assert_allclose(k, rk, atol=TOL)
        np.testing.assert_allclose(v, rv, atol=TOL)
