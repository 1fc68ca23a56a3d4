"""Plausible mistakes planted in the oracle (on the CPU) must trip one of its pins."""
import numpy as np
import pytest

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import oracle_model, torch_model

import test_oracle_primitives as prim
import test_oracle_selfchecks as chk


@pytest.fixture(scope="module")
def tiny():
    shape = gi.SHAPES["tiny"]
    om = oracle_model(shape, torch_model(shape, seed=0, gain_jitter=0.1))
    prefix = gi.prefix_tokens(0, 24, shape.vocab)
    return shape, om, prefix, orc.prefill(om, prefix)


def _expect_failure(fn, *args):
    with pytest.raises(AssertionError):
        fn(*args)


def test_mask_without_self_is_caught(tiny, monkeypatch):
    real = orc.ancestor_mask
    # drop the diagonal but keep the root visible to itself so softmax stays defined
    def bad2(parent):
        anc, depth = real(parent)
        anc = anc.copy()
        for i in range(1, len(parent)):
            anc[i, i] = False
        return anc, depth
    monkeypatch.setattr(orc, "ancestor_mask", bad2)
    _expect_failure(chk.test_chain_tree_is_causal_attention, tiny)


def test_position_by_node_index_is_caught(tiny, monkeypatch):
    real = orc.ancestor_mask
    monkeypatch.setattr(orc, "ancestor_mask",
                        lambda parent: (real(parent)[0], np.arange(len(parent), dtype=np.int32)))
    _expect_failure(chk.test_tree_pass_equals_one_causal_run_per_path, tiny, gi.tree_tiny_spine())


def test_sibling_leak_is_caught(tiny, monkeypatch):
    real = orc.ancestor_mask
    monkeypatch.setattr(orc, "ancestor_mask",
                        lambda parent: (np.tril(np.ones((len(parent),) * 2, bool)), real(parent)[1]))
    _expect_failure(chk.test_star_tree_sees_prefix_root_and_self_only, tiny)


def test_interleaved_rope_pairing_is_caught(monkeypatch):
    def bad(x, pos, base):
        T, n_h, d = x.shape
        y = orc_rope(x.reshape(T, n_h, d // 2, 2).transpose(0, 1, 3, 2).reshape(T, n_h, d), pos, base)
        return y.reshape(T, n_h, 2, d // 2).transpose(0, 1, 3, 2).reshape(T, n_h, d)
    orc_rope = orc.rope
    monkeypatch.setattr(orc, "rope", bad)
    _expect_failure(prim.test_rope_closed_form_complex_rotation)


def test_missing_score_scale_is_caught(monkeypatch):
    real = orc.attention
    monkeypatch.setattr(orc, "attention",
                        lambda q, K, V, allow: real(q * np.sqrt(q.shape[-1]), K, V, allow))
    _expect_failure(prim.test_attention_matches_library_with_mask)


def test_walk_past_a_mismatch_is_caught(monkeypatch):
    def bad(parent, tokens, is_spine, x_hat):
        ok = orc.accepted_nodes_bruteforce(parent, tokens, x_hat)
        # wrong: accept every node whose own edge matches, ignoring its ancestors
        acc = [i for i in range(1, len(parent)) if int(tokens[i]) == int(x_hat[int(parent[i])])]
        chain, v = [], 0
        for i in acc:
            if int(parent[i]) == v or not ok[int(parent[i])]:
                chain.append(i)
                v = i
        return chain, int(x_hat[v])
    monkeypatch.setattr(orc, "greedy_walk", bad)
    _expect_failure(chk.test_walk_golden_cases)


def test_commit_in_node_order_is_caught(tiny, monkeypatch):
    real = orc.commit_path
    monkeypatch.setattr(orc, "commit_path", lambda cache, new_kv, path: real(cache, new_kv, list(range(len(path)))))
    _expect_failure(chk.test_commit_keeps_prefix_and_appends_path_rows, tiny)


def test_root_left_out_of_the_cache_breaks_losslessness(tiny, monkeypatch):
    real = orc.commit_path
    # wrong reading: commit only the accepted drafts, not the root (anchor) itself
    def bad(cache, new_kv, path):
        out = real(cache, new_kv, path)
        return [(k[:, [*range(k.shape[1] - len(path)), *range(k.shape[1] - len(path) + 1, k.shape[1])]],
                 v[:, [*range(v.shape[1] - len(path)), *range(v.shape[1] - len(path) + 1, v.shape[1])]])
                for k, v in out]
    monkeypatch.setattr(orc, "commit_path", bad)
    _expect_failure(chk.test_cycles_reproduce_plain_greedy_decoding, tiny, True)
