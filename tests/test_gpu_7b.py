"""Full-size parity: the benchmark's launch configuration (7B shape, B=64 spine tree, KV prefix 1024)
and single layers of the 13B / 33B shapes.

The 7B step is checked twice.  Piecewise, at the one-layer tolerance: every decoder layer from the
device's own input to that layer (input rows and the layer's stored KV prefix are handed to the
oracle; output rows, the update on its own scale and the new KV rows are compared), the LM head on
the final hidden rows, the walk (Alg. UnifiedGreedyWalk) and the compaction bit-exactly; the device-resident entry
point the benchmark replays is then required to reproduce the same step bit for bit.  And as a
whole, all 32 layers on both sides from the same stored prefix, at the same tolerance (2e-2 of the logit
scale), in both activation modes of the library (fp16 operands, two-term bf16 operands).
"""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import LazyLayers, device_cache_as_oracle, gpu_model, oracle_model, to_f64, torch_model
from test_gpu_parity import TOL, _compare_step, _gpu_prefill, tol_for

pytestmark = pytest.mark.gpu

TOL_BF16 = TOL["bf16"]


def _lookahead(gm, root, n):
    """The device model's own next n greedy tokens after `root` (single-node steps), cache length restored."""
    keep = gm.P
    single = gi.tree_single()
    out, tok = [], root
    for _ in range(n):
        tok = gm.verify_step_calls([tok], single.parent, single.is_spine, commit=True)["bonus"]
        out.append(tok)
    gm.set_P(keep)
    return np.asarray(out, dtype=np.int32)


@pytest.mark.timeout(900)
def test_7b_step_in_the_benchmark_configuration():
    from paper_2604_02047_amd import ModelDesc
    from paper_2604_02047_amd.runner import GooseModel
    shape, seed, B, P0 = gi.SHAPES["7b"], 0, 64, 1024
    dev = torch.device("cuda:0")
    cap = 1024 + 256
    print("building the 7B model on the device", flush=True)
    gm = GooseModel(ModelDesc.from_shape(shape), B, cap, lambda l: gi.layer_weights(shape, seed, l, dev),
                    gi.embedding(shape, seed, dev), gi.lm_head(shape, seed, dev), gi.final_norm(shape, seed, dev))
    prefix = gi.prefix_tokens(seed, P0, shape.vocab)
    last = _gpu_prefill(gm, prefix, B)
    root = int(last["argmax"][-1].item())
    tree = gi.tree_spine_7b(seed)
    assert tree.B == B
    cont = _lookahead(gm, root, 12)
    tokens = gi.draft_tokens_pld_like(seed + 1, tree.parent, tree.is_spine, shape.vocab, root, prefix)
    tokens = gi.plant_drafts(seed + 2, tree.parent, tree.is_spine, tokens, cont, shape.vocab,
                             p_spine=0.85, p_branch=0.5, p_grand=0.5)
    P = gm.P
    assert P == P0

    # ---- the step through the individual entry points, hidden rows captured after every layer
    hidden = {}
    g = gm.verify_step_calls(tokens, tree.parent, tree.is_spine, want_logits=True, commit=False,
                             layer_hook=lambda l, x: hidden.__setitem__(l, x.detach().clone()))
    anc, depth = orc.ancestor_mask(tree.parent)
    assert np.array_equal(g["mask"].cpu().numpy().view(np.uint64), orc.mask_words(anc))
    assert np.array_equal(g["pos"].cpu().numpy(), P + depth)
    allow = np.concatenate([np.ones((B, P), bool), anc], axis=1)
    embed = gi.embedding(shape, seed, dev)
    x_embed = embed[torch.as_tensor(np.asarray(tokens, np.int64), device=dev)].float()
    om = orc.OracleModel(shape.n_heads, shape.head_dim, shape.rope_base, shape.rms_eps, [None] * shape.n_layers,
                         None, None, None)

    # ---- every layer on its own, from the device's input to that layer
    for l in range(shape.n_layers):
        print(f"oracle layer {l}", flush=True)
        w = {k: to_f64(v) for k, v in gi.layer_weights(shape, seed, l, dev).items()}
        x_in = (x_embed if l == 0 else hidden[l - 1]).double().cpu().numpy()
        Kc = gm.k_rows(0, P)[l].double().cpu().numpy()
        Vc = gm.v_rows(0, P)[l].double().cpu().numpy()
        x_out, k_new, v_new = orc.decoder_layer(om, w, x_in, Kc, Vc, P + depth, allow)
        got = hidden[l].double().cpu().numpy()
        assert np.abs(got - x_out).max() <= TOL_BF16 * np.abs(x_out).max(), f"layer {l} rows"
        # what the layer added, on its own scale (the residual stream itself can hide a wrong update)
        upd = x_out - x_in
        assert np.abs((got - x_in) - upd).max() <= TOL_BF16 * np.abs(upd).max(), f"layer {l} update"
        gk = g["tail_k"][l].double().cpu().numpy()
        gv = g["tail_v"][l].double().cpu().numpy()
        assert np.abs(gk - k_new).max() <= TOL_BF16 * np.abs(k_new).max(), f"layer {l} K rows"
        assert np.abs(gv - v_new).max() <= TOL_BF16 * np.abs(v_new).max(), f"layer {l} V rows"
        del w

    # ---- LM head on the final hidden rows
    print("oracle LM head", flush=True)
    om.final_norm = to_f64(gi.final_norm(shape, seed, dev))
    om.lm_head = to_f64(gi.lm_head(shape, seed, dev))
    ref = orc.final_logits(om, hidden[shape.n_layers - 1].double().cpu().numpy())
    gl = g["logits"].double().cpu().numpy()
    scale = np.abs(ref).max()
    assert np.abs(gl - ref).max() <= TOL_BF16 * scale
    am = g["argmax"].cpu().numpy()
    assert np.array_equal(am, np.argmax(gl, axis=-1))
    safe = orc.top2_margin(ref) > 2 * TOL_BF16 * scale
    assert safe.sum() >= 8   # random-init logits have small margins; enough decisive rows to mean something
    assert np.array_equal(am[safe], np.argmax(ref, axis=-1)[safe])

    # ---- walk and compaction
    acc, bonus = orc.greedy_walk(tree.parent, tokens, tree.is_spine, am)
    assert g["accept_len"] == len(acc) and g["bonus"] == bonus
    assert g["path"].tolist() == [0] + acc + [-1] * (B - 1 - len(acc))
    assert len(acc) >= 2, "the planted continuation should be accepted for a few nodes"

    # ---- the device-resident entry point (what the benchmark replays) reproduces the step
    t, p, s = gm.stage_tree(tokens, tree.parent, tree.is_spine)
    logits2 = torch.empty((B, shape.vocab), dtype=torch.float32, device=dev)
    margin2 = torch.empty(128, dtype=torch.float32, device=dev)
    gm.set_P(P)
    gm.verify_step_fused(t, p, s, B, cap - B, logits=logits2, margin=margin2)
    torch.cuda.synchronize()
    assert torch.equal(logits2, g["logits"]), "same kernels, same order of arithmetic"
    assert np.array_equal(gm.argmax[:B].cpu().numpy(), am)
    assert int(gm.accept_len.item()) == len(acc) and int(gm.bonus.item()) == bonus
    L = len(acc)
    assert int(gm.d_P.item()) == P + L + 1
    idx = torch.as_tensor([0] + acc, device=dev)
    assert torch.equal(gm.k_rows(P, P + L + 1), g["tail_k"][:, :, idx])
    assert torch.equal(gm.v_rows(P, P + L + 1), g["tail_v"][:, :, idx])
    assert gm.ctx.goose_device_flags() == 0
    gm.ctx.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("act_mode", [0, 1], ids=["fp16_operands", "two_term_operands"])
def test_7b_whole_step_against_the_oracle(act_mode):
    """All 32 layers on both sides from the same stored KV prefix: hidden rows after every layer,
    logits, new KV rows, predictions, walk and compaction (the oracle streams its weights layer by layer)."""
    import dataclasses
    from paper_2604_02047_amd import ModelDesc
    from paper_2604_02047_amd.runner import GooseModel
    shape, seed, B, P0 = gi.SHAPES["7b"], 0, 64, 1024
    dev = torch.device("cuda:0")
    desc = dataclasses.replace(ModelDesc.from_shape(shape), act_mode=act_mode)
    gm = GooseModel(desc, B, 1024 + 256, lambda l: gi.layer_weights(shape, seed, l, dev),
                    gi.embedding(shape, seed, dev), gi.lm_head(shape, seed, dev), gi.final_norm(shape, seed, dev))
    prefix = gi.prefix_tokens(seed, P0, shape.vocab)
    last = _gpu_prefill(gm, prefix, B)
    root = int(last["argmax"][-1].item())
    tree = gi.tree_spine_7b(seed + 5)
    cont = _lookahead(gm, root, 12)
    tokens = gi.draft_tokens_uniform(seed + 6, tree.parent, shape.vocab, root)
    tokens = gi.plant_drafts(seed + 7, tree.parent, tree.is_spine, tokens, cont, shape.vocab,
                             p_spine=0.9, p_branch=0.8, p_grand=0.8)
    layers = LazyLayers(shape.n_layers,
                        lambda l: {k: to_f64(v) for k, v in gi.layer_weights(shape, seed, l, dev).items()})
    om = orc.OracleModel(shape.n_heads, shape.head_dim, shape.rope_base, shape.rms_eps, layers,
                         to_f64(gi.embedding(shape, seed, dev)), to_f64(gi.lm_head(shape, seed, dev)),
                         to_f64(gi.final_norm(shape, seed, dev)))
    print("oracle: whole 7B step", flush=True)
    cache = device_cache_as_oracle(gm, P0)
    g, o, decisive = _compare_step(shape, gm, om, cache, tokens, tree, tol_for(shape))
    print(f"accepted {g['accept_len']} nodes, decisive={decisive}", flush=True)
    assert g["accept_len"] >= 1
    assert gm.ctx.goose_device_flags() == 0    # every weight re-encoded exactly, no operand out of range
    gm.ctx.close()


@pytest.mark.timeout(900)
def test_7b_hundred_cycles_walk_and_compaction_bit_exact():
    """100 consecutive cycles at the benchmark shape with planted drafts: every cycle's walk equals
    Alg. UnifiedGreedyWalk on the kernel's own predictions, and the committed cache rows are, byte for
    byte, the rows the layers wrote for the accepted path."""
    from paper_2604_02047_amd import ModelDesc
    from paper_2604_02047_amd.runner import GooseModel
    shape, seed, B, P0, n_cycles = gi.SHAPES["7b"], 0, 64, 1024, 100
    dev = torch.device("cuda:0")
    cap = (P0 + n_cycles * 20 + 2 * B + 63) // 64 * 64
    gm = GooseModel(ModelDesc.from_shape(shape), B, cap, lambda l: gi.layer_weights(shape, seed, l, dev),
                    gi.embedding(shape, seed, dev), gi.lm_head(shape, seed, dev), gi.final_norm(shape, seed, dev))
    prefix = gi.prefix_tokens(seed, P0, shape.vocab)
    root = int(_gpu_prefill(gm, prefix, B)["argmax"][-1].item())
    accepted, multi = 0, 0
    for t in range(n_cycles):
        tree = gi.tree_spine_7b(t)
        tokens = gi.draft_tokens_uniform(seed * 7919 + t, tree.parent, shape.vocab, root)
        tokens = gi.plant_drafts(seed * 104729 + t, tree.parent, tree.is_spine, tokens, _lookahead(gm, root, 6),
                                 shape.vocab, p_spine=0.6, p_branch=0.5, p_grand=0.3)
        P = gm.P
        g = gm.verify_step_calls(tokens, tree.parent, tree.is_spine, commit=True)
        acc, bonus = orc.greedy_walk(tree.parent, tokens, tree.is_spine, g["argmax"].cpu().numpy())
        L = len(acc)
        assert (g["accept_len"], g["bonus"]) == (L, bonus), f"cycle {t}"
        assert g["path"].tolist() == [0] + acc + [-1] * (B - 1 - L), f"cycle {t}"
        assert gm.P == P + L + 1
        idx = torch.as_tensor([0] + acc, device=dev)
        assert torch.equal(gm.k_rows(P, P + L + 1), g["tail_k"][:, :, idx]), f"cycle {t}"
        assert torch.equal(gm.v_rows(P, P + L + 1), g["tail_v"][:, :, idx]), f"cycle {t}"
        accepted += L
        multi += any(a != j + 1 for j, a in enumerate(acc))   # a path that leaves the spine moves rows
        root = bonus
        if t % 20 == 19:
            print(f"cycle {t + 1}: P={gm.P}, accepted so far {accepted}", flush=True)
    assert accepted >= n_cycles and multi >= 5
    assert gm.ctx.goose_device_flags() == 0
    gm.ctx.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,B,P0,tree_fn", [
    ("13b", 80, 320, gi.tree_spine_13b),
    ("33b", 80, 200, gi.tree_spine_33b),
    ("7b", 128, 450, gi.tree_spine_stress),
    ("llama3_8b", 64, 333, lambda: gi.tree_spine_7b(1)),
    ("qwen3_8b", 80, 250, gi.tree_spine_13b),
    ("7b_f16", 64, 333, lambda: gi.tree_spine_7b(2)),
])
def test_single_layer_of_the_larger_shapes(name, B, P0, tree_fn):
    """One decoder layer with the projection sizes of the larger models (and a small vocabulary),
    every output compared element by element."""
    full = gi.SHAPES[name]
    import dataclasses
    shape = dataclasses.replace(full, name=f"{name}_1layer", n_layers=1, vocab=4096)
    tm = torch_model(shape, seed=3, gain_jitter=0.1, device="cuda:0")
    tm = {k: ([{n: t.cpu() for n, t in lw.items()} for lw in v] if k == "layers" else v.cpu()) for k, v in tm.items()}
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=128, cap=(P0 + 2 * 128 + 63) // 64 * 64)
    prefix = gi.prefix_tokens(11, P0, shape.vocab)
    print(f"{name}: prefill", flush=True)
    _gpu_prefill(gm, prefix, 128)
    cache = orc.prefill(om, prefix)
    tree = tree_fn()
    assert tree.B == B
    tokens = gi.draft_tokens_uniform(12, tree.parent, shape.vocab, int(prefix[-1]))
    print(f"{name}: step", flush=True)
    _compare_step(shape, gm, om, cache, tokens, tree, TOL[shape.dtype])
    gm.ctx.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("workload,vocab", [
    ("13b_B80_P2048", 32000),              # 40 heads; also the LM head at the models' real vocabulary
    ("33b_B80_P4096", 4096),               # 52 heads
    ("7b_stress_B128_P16384", 4096),       # spine tree of 128 nodes over the longest prefix
    ("7b_balanced_B128_P16384", 4096),     # balanced control tree, same sizes
])
def test_one_layer_at_the_launch_shapes_of_the_larger_workloads(workload, vocab):
    """The attention and projection launch shapes the other benchmark workloads really take (full B, full
    prefix length, the benchmark's cache capacity), on a one-layer model of the same widths: every output
    element by element against the oracle, through the individual entry points (launches sized by the
    host's cache length) and through goose_verify_step as the benchmark replays it (sized by cap - B)."""
    import dataclasses
    import bench
    shape_name, B, P0, tree_kind, steps = bench.WORKLOADS[workload]
    shape = dataclasses.replace(gi.SHAPES[shape_name], name=f"{workload}_1layer", n_layers=1, vocab=vocab)
    tol = TOL[shape.dtype]
    cap = bench.cap_for(P0, B, steps + 5)
    dev = torch.device("cuda:0")
    tm = torch_model(shape, seed=4, gain_jitter=0.1, device="cuda:0")
    tm = {k: ([{n: t.cpu() for n, t in lw.items()} for lw in v] if k == "layers" else v.cpu()) for k, v in tm.items()}
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=B, cap=cap)
    prefix = gi.prefix_tokens(21, P0, shape.vocab)
    print(f"{workload}: prefill of {P0} tokens on the device", flush=True)
    last = _gpu_prefill(gm, prefix, B)
    root = int(last["argmax"][-1].item())
    tree = bench.make_tree(tree_kind, 0)
    assert tree.B == B
    cont = _lookahead(gm, root, 8)
    tokens = gi.draft_tokens_uniform(22, tree.parent, shape.vocab, root)
    tokens = gi.plant_drafts(23, tree.parent, tree.is_spine, tokens, cont, shape.vocab,
                             p_spine=0.9, p_branch=0.8, p_grand=0.8)
    cache = device_cache_as_oracle(gm, P0)          # the stored prefix is an input of both sides
    print(f"{workload}: step through the individual entry points", flush=True)
    g, o, decisive = _compare_step(shape, gm, om, cache, tokens, tree, tol)

    print(f"{workload}: the same step through goose_verify_step, launches sized for P <= {cap - B}", flush=True)
    gm.set_P(P0)
    t, p, s = gm.stage_tree(tokens, tree.parent, tree.is_spine)
    logits = torch.empty((B, shape.vocab), dtype=torch.float32, device=dev)
    margin = torch.empty(128, dtype=torch.float32, device=dev)
    gm.verify_step_fused(t, p, s, B, cap - B, logits=logits, margin=margin)
    torch.cuda.synchronize()
    gl = logits.double().cpu().numpy()
    scale = np.abs(o["logits"]).max()
    err = np.abs(gl - o["logits"]).max()
    print(f"{workload}: max logit error {err / scale:.2e} of the logit scale", flush=True)
    assert err <= tol * scale
    am = gm.argmax[:B].cpu().numpy()
    assert np.array_equal(am, np.argmax(gl, axis=-1))
    safe = o["margin"] > 2 * tol * scale
    assert np.array_equal(am[safe], o["x_hat"][safe])
    acc, bonus = orc.greedy_walk(tree.parent, tokens, tree.is_spine, am)
    L = len(acc)
    assert int(gm.accept_len.item()) == L and int(gm.bonus.item()) == bonus
    assert int(gm.d_P.item()) == P0 + L + 1
    # the committed rows are the new K/V rows of the accepted path
    idx = np.asarray([0] + acc)
    k_new, v_new = o["new_kv"][0]
    gk = gm.k_rows(P0, P0 + L + 1)[0].double().cpu().numpy()
    gv = gm.v_rows(P0, P0 + L + 1)[0].double().cpu().numpy()
    assert np.abs(gk - k_new[:, idx]).max() <= tol * np.abs(k_new).max()
    assert np.abs(gv - v_new[:, idx]).max() <= tol * np.abs(v_new).max()
    assert gm.ctx.goose_device_flags() == 0
    gm.ctx.close()
