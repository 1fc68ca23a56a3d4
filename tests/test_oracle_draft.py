"""Pins of the draft-side oracle: printed values of the paper, hand-worked cases, invariants, and the
lossless property of the whole loop (Alg. "Decoding Loop": output identical to autoregressive decoding)."""
import json
import math
import os

import numpy as np

import goose_inputs as gi
from oracle import goose_draft as dr
from oracle import goose_oracle as orc
from util import oracle_model, torch_model

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "draft_cases.json")))


def test_budget_split_printed_and_hand_cases():
    for c in G["budget_cases"]:
        assert dr.spine_budget(c["B"], c["m"], c["r"], c["rho"]) == (c["b_s"], c["b_r"], c["b_rho"])
        assert c["b_s"] + c["b_r"] + c["b_rho"] == c["B"] - 1
    bs = G["branch_share"]
    for r, share in zip(bs["r"], bs["share"]):
        b_s, b_r, b_rho = dr.spine_budget(bs["B"], 10 ** 6, r, 0.5)
        assert bs["B"] - b_s == share                     # branches incl. the root's own slot, as the paper counts


def test_harmonic_schedule_matches_the_printed_table():
    h = G["harmonic_30_12"]
    a = dr.harmonic_allocation(30, 12)
    assert a[:7] == [math.floor(x) for x in h["printed_first7"]]
    assert all(math.floor(h["printed_rest_range"][0]) <= x <= math.floor(h["printed_rest_range"][1]) for x in a[7:])
    assert a == sorted(a, reverse=True) and sum(a) <= 30   # wider near the root, never over budget


def test_tiers_and_moving_average():
    for p, r in G["tiers"]:
        assert dr.spine_ratio_tier(p) == r
    p = 0.3
    for _ in range(5):
        p = dr.ema_update(p, 9, 9)
    assert dr.spine_ratio_tier(p) == 0.50                  # settles within a few cycles (Sec. 4.3)
    p = 0.3
    for _ in range(5):
        p = dr.ema_update(p, 0, 9)
    assert dr.spine_ratio_tier(p) == 0.15
    assert dr.ema_update(0.3, 0, 0) == 0.3
    assert abs(dr.ema_update(0.3, 1, 2) - (0.7 * 0.3 + 0.3 * 0.5)) < 1e-15


def test_context_match_hand_cases():
    #           0  1  2  3  4  5  6  7  8  9 10 11 12
    seq = [7, 1, 2, 3, 9, 8, 5, 1, 2, 3, 4, 1, 2, 3]
    # suffix (1,2,3) occurred at 1 (-> 9 8 5 ...) and at 7 (-> 4 1 2 3): the most recent wins
    d, c = dr.context_match(seq, lens=(3,), max_len=20)
    assert d == [4, 1, 2, 3] and c is False
    assert dr.context_match(seq, lens=(3,), max_len=2)[0] == [4, 1]
    # 4-gram (4,1,2,3)? it never occurred before; 5-gram neither -> the 3-gram match stands, no consensus
    assert dr.context_match(seq, lens=(3, 4, 5)) == ([4, 1, 2, 3], False)
    # a sequence repeating with period 4: all three lengths match and agree -> consensus, longest n gives the chain
    rep = [5, 6, 7, 8] * 4
    d, c = dr.context_match(rep, lens=(3, 4, 5), max_len=20)
    assert c is True and d == [5, 6, 7, 8]                # most recent occurrence: only 4 tokens follow it
    assert dr.context_match([1, 2, 3], lens=(3, 4, 5)) == ([], False)
    assert dr.context_match([1, 2, 3, 4, 5, 6], lens=(3, 4, 5)) == ([], False)
    # two lengths match at different places and disagree on the first token: no consensus
    s2 = [9, 2, 3, 4, 50,   1, 2, 3, 4, 60,   1, 2, 3, 4]
    d, c = dr.context_match(s2, lens=(3, 4), max_len=3)
    assert d == [60, 1, 2] and c is True                  # both lengths find position 6 first: same continuation
    s3 = [1, 2, 3, 4, 60, 0, 9, 2, 3, 4, 50, 0, 1, 2, 3, 4]
    d, c = dr.context_match(s3, lens=(3, 4), max_len=3)
    assert d == [60, 0, 9] and c is False                 # n=3 finds (2,3,4)->50, n=4 finds (1,2,3,4)->60


def _tables(V, K, rows):
    ids = np.full((V, K), -1, np.int32)
    sc = np.zeros((V, K))
    for t, succ in rows.items():
        for j, (s, p) in enumerate(succ):
            ids[t, j], sc[t, j] = s, p
    return ids, sc


def test_build_spine_tree_hand_case():
    V, K = 40, 4
    ids, sc = _tables(V, K, {
        10: [(11, 0.5), (20, 0.3), (21, 0.1), (22, 0.005)],       # anchor: 11 is the spine child, 22 below threshold
        11: [(12, 0.6), (23, 0.2)],
        12: [(24, 0.4)],
        20: [(30, 0.9)], 21: [(31, 0.9)], 23: [(32, 0.9)], 30: [(33, 0.9)],
    })
    # B=12, r=0.25, m=3 -> b_s = min(3, 3) = 3; b_r = floor(8*0.5) = 4; b_rho = 4;
    # a_i = floor(4*(1/i)/(11/6)) = 2, 1, 0.  Root: 11 is the spine child, 22 is below the threshold -> 20, 21.
    # Spine node 11: 12 is its spine child -> 23.  Spine node 12: 24.  Spine node 13: nothing allotted.
    # Step 4, D=2: 20->30, 21->31, 23->32, 24 has no row; the new nodes are at branch depth 2 and stay leaves.
    tok, par, sp = dr.build_spine_tree(10, [11, 12, 13], ids, sc, B=12, r=0.25, rho=0.5, D=2, min_score=0.01)
    assert tok == [10, 11, 12, 13, 20, 21, 23, 24, 30, 31, 32]
    assert par == [-1, 0, 1, 2, 0, 0, 1, 2, 4, 5, 6]
    assert sp == [1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0]
    # with D=3 node 30 is extended by 33, which fills the budget of 12
    tok3, par3, _ = dr.build_spine_tree(10, [11, 12, 13], ids, sc, B=12, r=0.25, rho=0.5, D=3, min_score=0.01)
    assert tok3 == tok + [33] and par3 == par + [8]
    # the budget is a hard cap
    tok5, _, _ = dr.build_spine_tree(10, [11, 12, 13], ids, sc, B=5, r=0.25, rho=0.5, D=3, min_score=0.01)
    assert len(tok5) <= 5 and tok5[:2] == [10, 11]


def test_build_spine_tree_invariants_on_random_tables():
    rng = np.random.default_rng(0)
    V, K = 300, 10
    for trial in range(30):
        ids = rng.integers(-1, V, size=(V, K)).astype(np.int32)
        sc = rng.random(size=(V, K)) * (rng.random(size=(V, K)) < 0.8)
        m = int(rng.integers(0, 25))
        draft = rng.integers(0, V, size=m).tolist()
        B = int(rng.integers(2, 129))
        r = [0.15, 0.30, 0.50][trial % 3]
        D = int(rng.integers(1, 7))
        tok, par, sp = dr.build_spine_tree(5, draft, ids, sc, B, r, 0.5, D, 0.01)
        n = len(tok)
        b_s, _, _ = dr.spine_budget(B, m, r, 0.5)
        assert 1 + b_s <= n <= B and par[0] == -1 and all(0 <= par[i] < i for i in range(1, n))
        assert tok[1:1 + b_s] == draft[:b_s] and par[1:1 + b_s] == list(range(b_s)) and sum(sp) == 1 + b_s
        for v in range(n):                                    # branch children come from the table, distinct siblings
            kids = [i for i in range(n) if par[i] == v]
            btoks = [tok[i] for i in kids if not sp[i]]
            assert len(set(tok[i] for i in kids)) == len(kids)
            assert all(t in dr.successors(ids, sc, tok[v], 0.01) for t in btoks)
        depth = [0] * n
        for i in range(1, n):
            depth[i] = 0 if sp[i] else depth[par[i]] + 1
        assert max(depth) <= D


def test_loop_is_lossless_and_uses_all_modes():
    shape = gi.SHAPES["tiny"]
    om = oracle_model(shape, torch_model(shape, seed=4, gain_jitter=0.1))
    pat = gi.prefix_tokens(3, 12, shape.vocab).tolist()
    prompt = pat * 3 + pat[:5]
    trace = []
    y = dr.goose_decode(om, prompt, 60, B=24, trace=trace)
    ref = orc.greedy_decode(om, prompt, len(y))
    assert y == list(ref)[:len(y)]
    modes = {t["mode"] for t in trace}
    assert "tree" in modes or "bypass" in modes
    assert len(trace) < len(y)                                # fewer model calls than tokens: something was accepted
