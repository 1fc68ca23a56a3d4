"""Parity of the HIP verification path with the CPU oracle, element by element.

Tolerances (max abs error relative to the logit scale max|logit_oracle| of the step):
fp32 storage 1e-4, bf16 storage 2e-2, fp16 storage 2.5e-3 (three more mantissa bits than bf16), at any depth.  Integer results are bit-exact; an accept decision is only
compared where the oracle's top-2 logit margin at the deciding node exceeds the tolerance.
"""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import device_cache_as_oracle, gpu_model, load_prefix_cache, oracle_model, torch_model

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 2.5e-3}


def tol_for(shape):
    """Tolerance of a whole pass through `shape`: the same flat figure at any depth (2e-2 of the logit scale
    for the 16-bit types).  It holds for the 32-layer models because the projections' activation operands
    are not rounded to 8 bits (fp16 operands or two bf16 terms, see goose.h GOOSE_ACT_*)."""
    return TOL[shape.dtype]


def _gpu_prefill(gm, prefix, chunk):
    """Prefill through the verification path itself: chain trees, every row kept."""
    done = 0
    while done < len(prefix):
        n = min(chunk, len(prefix) - done)
        tree = gi.tree_chain(n)
        out = gm.verify_step_calls(prefix[done:done + n], tree.parent, tree.is_spine, commit=False)
        done += n
        gm.set_P(done)
    return out


def _compare_step(shape, gm, om, cache, tokens, tree, tol, check_hidden=True):
    """Runs one step on both sides from the same state and compares everything.  Returns both results."""
    P = cache[0][0].shape[1]
    assert gm.P == P
    hidden = []
    g = gm.verify_step_calls(tokens, tree.parent, tree.is_spine, want_logits=True, commit=True,
                             layer_hook=(lambda l, x: hidden.append(x.double().cpu().numpy())) if check_hidden else None)
    o = orc.verify_step(om, cache, tokens, tree.parent, tree.is_spine, return_hidden=True)
    B = tree.B
    # integer structure: bit-exact
    assert np.array_equal(g["mask"].cpu().numpy().view(np.uint64), orc.mask_words(o["anc"]))
    assert np.array_equal(g["depth"].cpu().numpy(), o["depth"])
    assert np.array_equal(g["pos"].cpu().numpy(), P + o["depth"])
    # hidden states per layer and logits: within tolerance of the scale
    if check_hidden:
        for l, (gh, oh) in enumerate(zip(hidden, o["hidden"])):
            assert np.abs(gh - oh).max() <= tol * np.abs(oh).max(), f"layer {l}"
    scale = np.abs(o["logits"]).max()
    gl = g["logits"].double().cpu().numpy()
    err = np.abs(gl - o["logits"]).max()
    print(f"{shape.name}: max logit error {err / scale:.2e} of the logit scale {scale:.3f} (tolerance {tol:.0e})", flush=True)
    assert err <= tol * scale, (err, scale)
    # KV rows written for the tree nodes
    for l, (k_new, v_new) in enumerate(o["new_kv"]):
        gk = g["tail_k"][l].double().cpu().numpy()
        gv = g["tail_v"][l].double().cpu().numpy()
        assert np.abs(gk - k_new).max() <= tol * max(1e-9, np.abs(k_new).max())
        assert np.abs(gv - v_new).max() <= tol * max(1e-9, np.abs(v_new).max())
    # the fused argmax is the argmax of the logits the kernel itself produced (lowest index on ties)
    assert np.array_equal(g["argmax"].cpu().numpy(), np.argmax(gl, axis=-1))
    part = np.partition(gl, -2, axis=-1)
    np.testing.assert_allclose(g["margin"].cpu().numpy(), part[:, -1] - part[:, -2], rtol=0, atol=1e-6)
    # predictions agree wherever the oracle's decision is not a near-tie
    safe = o["margin"] > 2 * tol * scale
    assert np.array_equal(g["argmax"].cpu().numpy()[safe], o["x_hat"][safe])
    # the walk on the kernel's own predictions is exactly Alg. UnifiedGreedyWalk ...
    acc, bonus = orc.greedy_walk(tree.parent, tokens, tree.is_spine, g["argmax"].cpu().numpy())
    assert g["accept_len"] == len(acc) and g["bonus"] == bonus
    assert g["path"].tolist() == [0] + acc + [-1] * (B - 1 - len(acc))
    # ... and equals the oracle's walk when every decision on the way was safe
    decisive = all(safe[v] for v in o["path"])
    if decisive:
        assert acc == o["accepted"] and bonus == o["bonus"]
    # compaction: the new cache tail is byte-identical to the rows the layers wrote
    L = len(acc)
    idx = torch.as_tensor([0] + acc, device=gm.device)
    assert gm.P == P + L + 1
    assert torch.equal(gm.k_rows(P, P + L + 1), g["tail_k"][:, :, idx])
    assert torch.equal(gm.v_rows(P, P + L + 1), g["tail_v"][:, :, idx])
    return g, o, decisive


def _run_cycles(shape_name, n_cycles, P0, trees, seed, oracle_prefill, chunk=16, planted=True):
    shape = gi.SHAPES[shape_name]
    tol = tol_for(shape)
    tm = torch_model(shape, seed=seed, gain_jitter=0.1)
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=128, cap=(P0 + 128 * (n_cycles + 1) + 63) // 64 * 64)
    prefix = gi.prefix_tokens(seed, P0, shape.vocab)
    last = _gpu_prefill(gm, prefix, chunk)
    if oracle_prefill:
        cache = orc.prefill(om, prefix)           # fully independent state
        for l, (k, v) in enumerate(cache):        # chain prefill on the GPU == causal prefill of the oracle
            gk = gm.k_rows(0, P0)[l].double().cpu().numpy()
            assert np.abs(gk - k).max() <= tol * np.abs(k).max()
    else:
        cache = device_cache_as_oracle(gm, P0)    # the device's stored bytes are the oracle's input
    # the anchor: prediction after the prefix
    ref_logits, _ = orc.causal_logits(om, prefix)
    root = int(np.argmax(ref_logits[-1]))
    greedy = orc.greedy_decode(om, list(prefix) + [root], 10 * n_cycles) if planted else None
    emitted_g, emitted_o = [root], [root]
    in_sync = True
    accepted_total = 0
    for cyc in range(n_cycles):
        tree = trees[cyc % len(trees)]
        tokens = gi.draft_tokens_uniform(1000 + cyc, tree.parent, shape.vocab, root)
        if planted and in_sync:
            cont = np.array(greedy[len(emitted_o) - 1:len(emitted_o) + 9])
            tokens = gi.plant_drafts(2000 + cyc, tree.parent, tree.is_spine, tokens, cont, shape.vocab,
                                     p_spine=0.8, p_branch=0.8, p_grand=0.8)
        g, o, decisive = _compare_step(shape, gm, om, cache, tokens, tree, tol)
        emitted_g += [int(tokens[v]) for v in g["path"][1:g["accept_len"] + 1]] + [g["bonus"]]
        emitted_o += [int(tokens[v]) for v in o["accepted"]] + [o["bonus"]]
        accepted_total += g["accept_len"]
        if not decisive:
            in_sync = False
            break   # a near-tie was decided differently: later states legitimately differ
        cache = o["cache"] if oracle_prefill else device_cache_as_oracle(gm, gm.P)
        root = o["bonus"]
    if in_sync:
        assert emitted_g == emitted_o
        if planted and oracle_prefill:
            assert emitted_o == ([emitted_o[0]] + greedy)[:len(emitted_o)]   # lossless: plain greedy decoding
        if planted:
            assert accepted_total >= n_cycles // 2  # compaction of multi-node paths really happened
    gm.ctx.close()
    return in_sync


def test_tiny_fp32_cycles_match_the_oracle():
    trees = [gi.tree_tiny_spine(), gi.tree_random(16, 3, spine_len=6), gi.tree_star(9), gi.tree_chain(12),
             gi.tree_single(), gi.tree_random(33, 4, spine_len=8)]
    assert _run_cycles("tiny", 8, 128, trees, seed=0, oracle_prefill=True)


def test_tiny_fp32_empty_prefix_and_big_trees():
    trees = [gi.tree_spine_7b(1), gi.tree_spine_stress(), gi.tree_balanced(), gi.tree_random(65, 2)]
    shape = gi.SHAPES["tiny"]
    tm = torch_model(shape, seed=1, gain_jitter=0.1)
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=128, cap=1024)
    gm.set_P(0)
    cache = orc.empty_cache(om)
    root = 17
    for n, tree in enumerate(trees):
        tokens = gi.draft_tokens_uniform(n, tree.parent, shape.vocab, root)
        g, o, decisive = _compare_step(shape, gm, om, cache, tokens, tree, TOL["f32"])
        assert decisive
        cache, root = o["cache"], o["bonus"]
    gm.ctx.close()


@pytest.mark.parametrize("shape_name", ["tiny_bf16", "small_gqa_qknorm_f16"])
def test_16bit_empty_prefix_and_big_trees(shape_name):
    """MFMA path from an empty cache (no prefix blocks at all, then a ragged first block): every tree shape."""
    trees = [gi.tree_spine_7b(1), gi.tree_single(), gi.tree_spine_stress(), gi.tree_random(65, 2), gi.tree_balanced()]
    shape = gi.SHAPES[shape_name]
    tm = torch_model(shape, seed=1, gain_jitter=0.1)
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=128, cap=1024)
    gm.set_P(0)
    root = 17
    for n, tree in enumerate(trees):
        cache = device_cache_as_oracle(gm, gm.P) if gm.P else orc.empty_cache(om)
        tokens = gi.draft_tokens_uniform(n, tree.parent, shape.vocab, root)
        g, o, decisive = _compare_step(shape, gm, om, cache, tokens, tree, tol_for(shape))
        root = g["bonus"]
    gm.ctx.close()


@pytest.mark.parametrize("shape_name,P0,chunk", [("tiny_bf16", 128, 16), ("small_bf16", 200, 50),
                                                 ("tiny_gqa_bf16", 100, 32), ("small_gqa_qknorm_bf16", 210, 70),
                                                 ("tiny_f16", 128, 16), ("small_gqa_qknorm_f16", 210, 70)])
def test_bf16_cycles_match_the_oracle(shape_name, P0, chunk):
    """MFMA path (bf16 and fp16 storage); the oracle starts every cycle from the device's own stored cache bytes."""
    trees = [gi.tree_tiny_spine(), gi.tree_spine_7b(0), gi.tree_random(33, 4, spine_len=8), gi.tree_spine_13b(),
             gi.tree_spine_stress(), gi.tree_single(), gi.tree_balanced()]
    _run_cycles(shape_name, 7, P0, trees, seed=2, oracle_prefill=False, chunk=chunk)


@pytest.mark.parametrize("shape_name", ["small_bf16", "small_gqa_qknorm_bf16", "small_gqa_qknorm_f16"])
def test_bf16_independent_prefill_stays_within_tolerance(shape_name):
    trees = [gi.tree_spine_7b(3), gi.tree_tiny_spine()]
    _run_cycles(shape_name, 2, 96, trees, seed=5, oracle_prefill=True, chunk=32)


@pytest.mark.parametrize("shape_name", ["small_bf16", "small_gqa_qknorm_f16"])
def test_wide_trees_over_prefix_lengths(shape_name):
    """Trees of 65 to 128 nodes at head size 128 (the kernel that stages the key blocks through an LDS ring)
    over prefix lengths that give every case of the ring: no prefix block at all, one, odd and even counts, a
    ragged last block in either key group's slot, one to three key splits.  The prefix is shortened from
    step to step, so the slots beyond it hold stale rows of the earlier, longer one."""
    shape = gi.SHAPES[shape_name]
    tol = tol_for(shape)
    tm = torch_model(shape, seed=11, gain_jitter=0.1)
    om = oracle_model(shape, tm)
    P_top = 417
    gm = gpu_model(shape, tm, max_B=128, cap=(P_top + 128 + 63) // 64 * 64)
    prefix = gi.prefix_tokens(11, P_top, shape.vocab)
    _gpu_prefill(gm, prefix, 64)
    trees = [gi.tree_random(65, 3, spine_len=9), gi.tree_spine_13b(), gi.tree_random(97, 4, spine_len=12),
             gi.tree_spine_stress(), gi.tree_balanced()]
    for n, P in enumerate([417, 385, 352, 321, 300, 289, 257, 224, 193, 161, 130, 97, 64, 33, 31, 1, 0]):
        gm.set_P(P)
        cache = device_cache_as_oracle(gm, P) if P else orc.empty_cache(om)
        tree = trees[n % len(trees)]
        tokens = gi.draft_tokens_uniform(300 + n, tree.parent, shape.vocab, int(prefix[P - 1]) if P else 17)
        print(f"P={P} B={tree.B}", flush=True)
        _compare_step(shape, gm, om, cache, tokens, tree, tol)
    gm.ctx.close()


def test_16bit_tree_that_fills_the_cache_to_its_last_slot():
    """P + B == cap exactly (the largest tree in the last free slots), and one slot more is refused."""
    from paper_2604_02047_amd.binding import GooseError
    shape = gi.SHAPES["tiny_bf16"]
    tm = torch_model(shape, seed=3, gain_jitter=0.1)
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=128, cap=192)
    _gpu_prefill(gm, gi.prefix_tokens(9, 64, shape.vocab), 64)
    assert gm.P == 64
    tree = gi.tree_spine_stress()
    tokens = gi.draft_tokens_uniform(4, tree.parent, shape.vocab, 5)
    _compare_step(shape, gm, om, device_cache_as_oracle(gm, 64), tokens, tree, tol_for(shape))
    gm.set_P(65)
    with pytest.raises(GooseError):
        gm.verify_step_calls(tokens, tree.parent, tree.is_spine, commit=False)
    gm.ctx.close()
