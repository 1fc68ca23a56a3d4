"""Several requests verified in one pass (the batch sweep of App. D).  The requests share every
projection and one attention launch per tree-size class; a request's rows never mix with
another's, so with the same number of key splits its results equal, bit for bit, what it gives on
its own.  With a different split count (more requests -> fewer splits per head) the attention sums
are ordered differently: then every request is held to the oracle's tolerance instead."""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import device_cache_as_oracle, gpu_model, oracle_model, torch_model
from test_gpu_parity import _gpu_prefill, tol_for

pytestmark = pytest.mark.gpu


def _requests(gm, shape, sizes, P0s, P_maxs):
    reqs = []
    for r, (B, P0, P_max) in enumerate(zip(sizes, P0s, P_maxs)):
        kc, vc = torch.zeros_like(gm.kcache), torch.zeros_like(gm.vcache)
        gm.kcache, gm.vcache = kc, vc
        gm.set_P(0)
        last = _gpu_prefill(gm, gi.prefix_tokens(50 + r, P0, shape.vocab), 64)
        root = int(last["argmax"][-1].item())
        tree = gi.tree_spine_7b(r) if B == 64 else gi.tree_random(B, seed=r, spine_len=min(8, B - 1))
        tokens = gi.draft_tokens_uniform(60 + r, tree.parent, shape.vocab, root)
        t, p, s = gm.stage_tree(tokens, tree.parent, tree.is_spine)
        reqs.append({"tokens": t, "parent": p, "is_spine": s, "B": B, "P_max": P_max, "kcache": kc, "vcache": vc,
                     "P0": P0, "k0": kc.clone(), "v0": vc.clone(), "tree": tree, "host_tokens": tokens})
    return reqs


def _alone(gm, reqs):
    out = []
    for q in reqs:
        gm.kcache, gm.vcache = q["kcache"], q["vcache"]
        gm.set_P(q["P0"])
        ids = torch.full((gm.desc.vocab, 10), -1, dtype=torch.int32, device=gm.device)
        sc = torch.zeros((gm.desc.vocab, 10), dtype=torch.float32, device=gm.device)
        gm.verify_step_fused(q["tokens"], q["parent"], q["is_spine"], q["B"], q["P_max"], succ_ids=ids, succ_scores=sc)
        torch.cuda.synchronize()
        out.append({"ids": ids, "scores": sc, "argmax": gm.argmax[:q["B"]].clone(), "L": int(gm.accept_len.item()),
                    "path": gm.path[:q["B"]].clone(), "bonus": int(gm.bonus.item()), "P": int(gm.d_P.item()),
                    "k": q["kcache"].clone(), "v": q["vcache"].clone()})
        q["kcache"].copy_(q["k0"])
        q["vcache"].copy_(q["v0"])
    return out


def _batched(gm, reqs):
    i32 = dict(dtype=torch.int32, device=gm.device)
    for q in reqs:
        q["P"] = torch.full((1,), q["P0"], **i32)
        q["accept_len"], q["path"], q["bonus"] = torch.zeros(1, **i32), torch.zeros(128, **i32), torch.zeros(1, **i32)
        q["succ_ids"] = torch.full((gm.desc.vocab, 10), -1, **i32)      # every request harvests into its own tables
        q["succ_scores"] = torch.zeros((gm.desc.vocab, 10), dtype=torch.float32, device=gm.device)
    argmax_all = torch.full((gm.ctx.max_rows,), -1, **i32)
    gm.ctx.goose_verify_step_batched(gm.model_ptrs(), reqs, argmax_all)
    torch.cuda.synchronize()
    assert gm.ctx.goose_device_flags() == 0
    row0 = 0
    for q in reqs:
        q["argmax"] = argmax_all[row0:row0 + q["B"]].clone()
        row0 += (q["B"] + 31) // 32 * 32
    return argmax_all


def _rows(gm, kc, vc, lo, hi):
    keep = gm.kcache, gm.vcache
    gm.kcache, gm.vcache = kc, vc
    k, v = gm.k_rows(lo, hi), gm.v_rows(lo, hi)
    gm.kcache, gm.vcache = keep
    return k, v


def _check_against_oracle(gm, om, shape, q):
    """Predictions where the oracle's decision is not a near-tie, the walk on the kernel's own
    predictions, the new cache length and the committed KV rows."""
    tol = tol_for(shape)
    keep = gm.kcache, gm.vcache
    gm.kcache, gm.vcache = q["k0"], q["v0"]
    cache = device_cache_as_oracle(gm, q["P0"])   # the device's stored prefix is the oracle's input
    gm.kcache, gm.vcache = keep
    o = orc.verify_step(om, cache, q["host_tokens"], q["tree"].parent, q["tree"].is_spine)
    got = q["argmax"].cpu().numpy()
    safe = o["margin"] > 2 * tol * np.abs(o["logits"]).max()
    assert safe.any() and np.array_equal(got[safe], o["x_hat"][safe])
    acc, bonus = orc.greedy_walk(q["tree"].parent, q["host_tokens"], q["tree"].is_spine, got)
    L = int(q["accept_len"].item())
    assert L == len(acc) and int(q["bonus"].item()) == bonus and q["path"][:L + 1].tolist() == [0] + acc
    assert int(q["P"].item()) == q["P0"] + L + 1
    k_new, v_new = _rows(gm, q["kcache"], q["vcache"], q["P0"], q["P0"] + L + 1)
    for l, (ko, vo) in enumerate(o["new_kv"]):
        ko, vo = ko[:, [0] + acc], vo[:, [0] + acc]
        assert np.abs(k_new[l].double().cpu().numpy() - ko).max() <= tol * np.abs(ko).max()
        assert np.abs(v_new[l].double().cpu().numpy() - vo).max() <= tol * np.abs(vo).max()
    # the prefix itself is untouched
    k_b, v_b = _rows(gm, q["kcache"], q["vcache"], 0, q["P0"])
    k_0, v_0 = _rows(gm, q["k0"], q["v0"], 0, q["P0"])
    assert torch.equal(k_b, k_0) and torch.equal(v_b, v_0)


def _rows_of(sizes):
    return sum((B + 31) // 32 * 32 for B in sizes)


@pytest.mark.parametrize("shape_name,sizes", [("small_bf16", [64, 30, 20]), ("small_gqa_qknorm_bf16", [33, 64]),
                                              ("tiny_bf16", [16, 9, 1, 32]), ("tiny_gqa_bf16", [128]),
                                              ("small_bf16", [32] * 8), ("tiny_bf16", [16, 9, 1, 32, 64, 100, 3]),
                                              ("small_gqa_qknorm_bf16", [32] * 16),
                                              ("small_gqa_qknorm_f16", [64, 20, 32, 100, 7]),
                                              ("small_bf16", [100, 128, 70, 96])])
def test_batched_step_equals_the_requests_alone(shape_name, sizes):
    """Short prefixes: one key split alone and batched, hence identical arithmetic per request
    (also beyond 128 stacked rows, where the projections run in chunks of 128 rows)."""
    shape = gi.SHAPES[shape_name]
    tm = torch_model(shape, seed=7, gain_jitter=0.1)
    gm = gpu_model(shape, tm, max_B=128, cap=384, max_rows=max(128, _rows_of(sizes)))
    P0s = [40 + (37 * r) % 100 for r in range(len(sizes))]
    reqs = _requests(gm, shape, sizes, P0s, [256 - B for B in sizes])
    alone = _alone(gm, reqs)
    _batched(gm, reqs)
    for q, a in zip(reqs, alone):
        assert torch.equal(q["argmax"], a["argmax"])
        assert int(q["accept_len"].item()) == a["L"] and int(q["bonus"].item()) == a["bonus"]
        assert torch.equal(q["path"][:q["B"]], a["path"]) and int(q["P"].item()) == a["P"]
        assert torch.equal(q["succ_ids"], a["ids"]) and torch.equal(q["succ_scores"], a["scores"])   # harvest
        assert int((q["succ_ids"][:, 0] >= 0).sum().item()) == len(set(q["host_tokens"].tolist()))
        k_b, v_b = _rows(gm, q["kcache"], q["vcache"], 0, a["P"])   # the committed cache is identical
        k_a, v_a = _rows(gm, a["k"], a["v"], 0, a["P"])
        assert torch.equal(k_b, k_a) and torch.equal(v_b, v_a)
    om = oracle_model(shape, tm)
    for q in reqs[1:2] + reqs[5:]:     # requests that do not start at row 0, against the oracle
        _check_against_oracle(gm, om, shape, q)
    gm.ctx.close()


@pytest.mark.parametrize("shape_name,sizes,P0s", [("small_bf16", [32, 32, 32, 32], [700, 513, 640, 96]),
                                                  ("small_gqa_qknorm_bf16", [40, 17, 9], [600, 777, 31]),
                                                  ("tiny_gqa_bf16", [90], [500]),
                                                  ("small_gqa_qknorm_bf16", [64, 17, 40, 128, 5], [600, 777, 31, 300, 512]),
                                                  ("small_gqa_qknorm_bf16", [100, 128, 70, 96], [300, 513, 96, 640])])
def test_batched_step_with_long_prefixes_matches_the_oracle(shape_name, sizes, P0s):
    """Prefixes long enough for several key splits, mixed tree-size classes: every request against the oracle."""
    shape = gi.SHAPES[shape_name]
    tm = torch_model(shape, seed=8, gain_jitter=0.1)
    gm = gpu_model(shape, tm, max_B=128, cap=1024, max_rows=max(128, _rows_of(sizes)))
    reqs = _requests(gm, shape, sizes, P0s, [1024 - B for B in sizes])
    _batched(gm, reqs)
    om = oracle_model(shape, tm)
    for q in reqs:
        _check_against_oracle(gm, om, shape, q)
    gm.ctx.close()


def test_batched_step_rejects_what_does_not_fit():
    from paper_2604_02047_amd.binding import GooseError
    shape = gi.SHAPES["tiny_bf16"]
    gm = gpu_model(shape, torch_model(shape, seed=1), max_B=64, cap=256)
    i32 = dict(dtype=torch.int32, device=gm.device)
    tree = gi.tree_chain(40)
    t, p, s = gm.stage_tree(np.zeros(40, np.int32), tree.parent, tree.is_spine)
    q = {"tokens": t, "parent": p, "is_spine": s, "B": 40, "P_max": 100, "kcache": gm.kcache, "vcache": gm.vcache,
         "P": torch.zeros(1, **i32), "accept_len": torch.zeros(1, **i32), "path": torch.zeros(128, **i32),
         "bonus": torch.zeros(1, **i32)}
    with pytest.raises(GooseError):   # 2 x round_up(40, 32) = 128 rows > 64
        gm.ctx.goose_verify_step_batched(gm.model_ptrs(), [q, dict(q)], torch.zeros(128, **i32))
    gm.ctx.close()
