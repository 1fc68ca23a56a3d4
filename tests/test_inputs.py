"""The seeded input generators: determinism, shapes and the structure the configs ask for."""
import numpy as np
import torch

import goose_inputs as gi


def test_weights_are_deterministic_and_roughly_normal():
    a = gi.gen_normal(0, 3, (257, 129), 0.02, torch.float32)
    b = gi.gen_normal(0, 3, (257, 129), 0.02, torch.float32, chunk=1000)  # chunking is invisible
    assert torch.equal(a, b)
    assert not torch.equal(a, gi.gen_normal(1, 3, (257, 129), 0.02, torch.float32))
    assert not torch.equal(a, gi.gen_normal(0, 4, (257, 129), 0.02, torch.float32))
    assert abs(float(a.std()) - 0.02) < 5e-4 and abs(float(a.mean())) < 5e-4
    assert float(a.abs().max()) <= 0.02 * 3.47
    # a known element, so a change of the generator cannot go unnoticed
    assert gi.gen_normal(0, 0, (4,), 0.02, torch.float32).tolist() == gi.gen_normal(0, 0, (2, 2), 0.02, torch.float32).flatten().tolist()


def test_bf16_weights_are_the_rounded_fp32_values():
    a = gi.gen_normal(5, 1, (64, 64), 0.02, torch.float32)
    b = gi.gen_normal(5, 1, (64, 64), 0.02, torch.bfloat16)
    assert torch.equal(a.to(torch.bfloat16), b)


def test_hash_is_a_32_bit_permutation_sample():
    x = torch.arange(0, 1 << 16, dtype=torch.int64)
    h = gi.hash32(x)
    assert int(h.min()) >= 0 and int(h.max()) < (1 << 32)
    assert len(torch.unique(h)) == len(x)  # the mix is a bijection on 32-bit words


def test_config_trees_have_the_stated_budgets():
    t = gi.tree_tiny_spine()
    assert t.B == 16 and t.parent[8:].tolist() == list(range(8)) and t.is_spine.sum() == 8
    for seed in range(5):
        t = gi.tree_spine_7b(seed)
        assert t.B == 64 and t.is_spine.sum() == 16 and t.parent[1:16].tolist() == list(range(15))
        kids = np.bincount(t.parent[1:], minlength=64)
        assert kids[:16].max() <= 4 and kids[16:].max() <= 1
    assert not np.array_equal(gi.tree_spine_7b(0).parent, gi.tree_spine_7b(1).parent)
    assert gi.tree_spine_13b().B == 80 and gi.tree_spine_33b().B == 80 and gi.tree_spine_stress().B == 128
    bal = gi.tree_balanced()
    assert bal.B == 128
    widths = np.bincount(gi.tree_spine_33b().parent[24:], minlength=24)
    assert widths.tolist() == [4] * 4 + [3] * 4 + [2] * 12 + [1] * 4


def test_all_trees_are_topological():
    for t in [gi.tree_chain(9), gi.tree_star(9), gi.tree_single(), gi.tree_random(50, 1), gi.tree_balanced(),
              gi.relabel_topological(gi.tree_spine_7b(2), 3)[0]]:
        assert t.parent[0] == -1 and all(0 <= t.parent[i] < i for i in range(1, t.B))


def test_sibling_tokens_are_distinct():
    t = gi.tree_star(40)
    toks = gi.draft_tokens_uniform(0, t.parent, 48, root_token=7)
    assert toks[0] == 7 and len(set(toks[1:].tolist())) == 39
    prefix = gi.prefix_tokens(0, 300, 1000)
    t = gi.tree_spine_13b()
    toks = gi.draft_tokens_pld_like(1, t.parent, t.is_spine, 1000, 3, prefix)
    for p in range(t.B):
        kids = [toks[i] for i in range(1, t.B) if t.parent[i] == p]
        assert len(set(kids)) == len(kids)
    # some spine tokens continue a run of the prefix
    runs = sum(1 for i in range(2, 20) for s in range(len(prefix) - 1)
               if prefix[s] == toks[i - 1] and prefix[s + 1] == toks[i])
    assert runs >= 2
