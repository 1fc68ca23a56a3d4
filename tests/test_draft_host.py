"""The library's host-side draft functions against the oracle, bit for bit (no GPU involved):
context match, budget split, spine tree, tiers and moving average."""
import numpy as np

from oracle import goose_draft as dr
from paper_2604_02047_amd import binding as gb


def test_context_match_matches_the_oracle():
    rng = np.random.default_rng(1)
    hits = 0
    for trial in range(400):
        L = int(rng.integers(0, 120))
        vocab = int(rng.choice([2, 3, 5, 50]))                 # small alphabets repeat a lot
        seq = rng.integers(0, vocab, size=L)
        if trial % 5 == 0 and L > 20:                          # periodic tails
            per = int(rng.integers(1, 9))
            seq[-3 * per:] = np.tile(seq[-per:], 3)
        lens = [(3, 4, 5), (3,), (2, 4), (5, 4, 3), (1, 2, 3, 4, 5, 6)][trial % 5]
        max_len = int(rng.integers(1, 25))
        d_ref, c_ref = dr.context_match(seq, lens, max_len)
        d, c = gb.goose_context_match(seq, lens, max_len)
        assert d.tolist() == d_ref and c == c_ref, (trial, seq.tolist(), lens, max_len)
        hits += bool(d_ref)
    assert hits > 100


def test_budget_tier_and_average_match_the_oracle():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        B, m = int(rng.integers(1, 129)), int(rng.integers(0, 40))
        r = float(rng.choice([0.15, 0.30, 0.50, rng.uniform(0.01, 0.99)]))
        rho = float(rng.choice([0.5, 0.25, rng.uniform(0.01, 0.99)]))
        ref = dr.spine_budget(B, m, r, rho)
        if ref[0] <= B - 1:                                    # the library also caps the spine at B-1 nodes
            assert gb.goose_spine_budget(B, m, r, rho) == ref
    for p in np.linspace(0, 1, 101).tolist() + [0.2, 0.4, 0.19999999, 0.39999999]:
        assert gb.goose_spine_ratio_tier(p) == dr.spine_ratio_tier(p)
    p_lib = p_ref = 0.3
    for _ in range(50):
        a, o = int(rng.integers(0, 10)), int(rng.integers(0, 10))
        a = min(a, o)
        p_lib, p_ref = gb.goose_ema_update(p_lib, a, o), dr.ema_update(p_ref, a, o)
        assert p_lib == p_ref


def test_spine_tree_matches_the_oracle():
    rng = np.random.default_rng(3)
    for trial in range(300):
        V, K = int(rng.choice([40, 300, 2000])), int(rng.choice([1, 4, 10, 16]))
        ids = rng.integers(-1, V, size=(V, K)).astype(np.int32)
        if trial % 3 == 0:
            ids[rng.random(size=V) < 0.5] = -1                  # many tokens without successors
        sc = (rng.random(size=(V, K)) * (rng.random(size=(V, K)) < 0.85)).astype(np.float32)
        m = int(rng.integers(0, 25))
        draft = rng.integers(0, V, size=m)
        if m and trial % 4 == 0:                                # the spine continuation is also the top successor
            prev = 7
            for i in range(m):
                ids[prev, 0], sc[prev, 0] = draft[i], 0.9
                prev = int(draft[i])
        B = int(rng.integers(1, 129))
        r = float(rng.choice([0.15, 0.30, 0.50]))
        rho = float(rng.choice([0.5, 0.3]))
        D = int(rng.integers(0, 7))
        thr = float(rng.choice([0.01, 0.0, 0.3]))
        if dr.spine_budget(B, m, r, rho)[0] > B - 1:
            continue
        t_ref, p_ref, s_ref = dr.build_spine_tree(7, draft.tolist(), ids, sc, B, r, rho, D, thr)
        t, p, s = gb.goose_build_spine_tree(7, draft, ids, sc, B, r, rho, D, thr)
        assert t.tolist() == t_ref and p.tolist() == p_ref and s.tolist() == s_ref, trial
        assert gb.goose_check_parent(p) == 0


def _plan_ref(seq, lens, max_spine, anchor, ids, sc, B, p_hat, rho, D, thr, bypass_len):
    """The routing of Alg. "Decoding Loop" spelled out with the oracle's pieces."""
    draft, consensus = dr.context_match(seq, lens, max_spine)
    if draft and (len(draft) >= bypass_len or consensus):
        return [anchor] + draft, list(range(-1, len(draft))), [1] * (1 + len(draft)), gb.MODE_BYPASS
    if draft or dr.successors(ids, sc, anchor, thr):
        t, p, s = dr.build_spine_tree(anchor, draft, ids, sc, B, dr.spine_ratio_tier(p_hat), rho, D, thr)
        return t, p, s, gb.MODE_TREE
    return [anchor], [-1], [1], gb.MODE_AR


def test_cycle_plan_matches_the_oracle():
    rng = np.random.default_rng(11)
    seen = set()
    for trial in range(400):
        V, K = int(rng.choice([12, 40, 300])), int(rng.choice([1, 4, 10]))
        ids = rng.integers(-1, V, size=(V, K)).astype(np.int32)
        if trial % 2 == 0:
            ids[rng.random(size=V) < 0.6] = -1                  # many tokens without successors
        sc = (rng.random(size=(V, K)) * (rng.random(size=(V, K)) < 0.7)).astype(np.float32)
        n = int(rng.integers(1, 80))
        seq = rng.integers(0, min(V, int(rng.choice([3, 6, V]))), size=n).tolist()   # small alphabets repeat n-grams
        anchor = int(seq[-1])
        lens = (3, 4, 5) if trial % 3 else (2, 3)
        max_spine = int(rng.choice([4, 20]))
        B = int(rng.integers(1 + max_spine, 129))
        p_hat = float(rng.random())
        thr = float(rng.choice([0.01, 0.0, 0.3]))
        bypass_len = int(rng.choice([3, 8]))
        t_ref, p_ref, s_ref, mode_ref = _plan_ref(seq, lens, max_spine, anchor, ids, sc, B, p_hat, 0.5, 6, thr, bypass_len)
        t, p, s, mode = gb.goose_plan_cycle(seq, lens, max_spine, anchor, ids, sc, B, p_hat, 0.5, 6, thr, bypass_len)
        assert mode == mode_ref, trial
        assert t.tolist() == list(t_ref) and p.tolist() == list(p_ref) and s.tolist() == list(s_ref), trial
        assert gb.goose_check_parent(p) == 0
        seen.add(mode)
    assert seen == {gb.MODE_AR, gb.MODE_TREE, gb.MODE_BYPASS}
