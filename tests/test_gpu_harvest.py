"""Logit harvest into the unigram successor tables (Sec. 4 stage 2; App. C "adjacency table" tier 1,
"logit harvesting"): the HIP kernel against the oracle on the same logits -- ids bit-exact (also
under ties and repeated tokens), scores to fp32 round-off -- alone and inside the fused step."""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import gpu_model, torch_model

pytestmark = pytest.mark.gpu


def _ctx(vocab):
    from paper_2604_02047_amd import GooseContext, ModelDesc
    shape = gi.ModelShape("h", 1, 256, 4, 64, 688, vocab, dtype="bf16")
    return GooseContext(ModelDesc.from_shape(shape), 128, 128)


@pytest.mark.parametrize("V,B,K,quant", [(1000, 1, 10, 0), (1000, 37, 10, 0.25), (32000, 64, 10, 0),
                                         (32000, 128, 16, 0.5), (4093, 128, 1, 0), (50, 9, 10, 1.0)])
def test_harvest_kernel_matches_the_oracle(V, B, K, quant):
    dev = "cuda:0"
    c = _ctx(V)
    rng = np.random.default_rng(V + B)
    logits = rng.normal(size=(B, V)).astype(np.float32) * 4
    if quant:
        logits = (np.round(logits / quant) * quant).astype(np.float32)      # many exact ties
    tokens = rng.integers(0, V, size=B).astype(np.int32)
    if B > 4:
        tokens[B // 2] = tokens[1]                                          # repeated tokens: the later node wins
        tokens[B - 1] = tokens[0]
    ld = V + 24                                                             # a padded row length
    d_logits = torch.full((B, ld), float("nan"), dtype=torch.float32, device=dev)
    d_logits[:, :V] = torch.from_numpy(logits)
    ids0 = rng.integers(0, V, size=(V, K)).astype(np.int32)
    sc0 = rng.random(size=(V, K)).astype(np.float32)
    d_ids, d_sc = torch.from_numpy(ids0).to(dev), torch.from_numpy(sc0).to(dev)
    c.goose_harvest_topk(d_logits, ld, torch.from_numpy(tokens).to(dev), B, K, d_ids, d_sc)
    torch.cuda.synchronize()
    ref_ids, ref_sc = orc.harvest_topk(logits.astype(np.float64), tokens, K, table_ids=ids0, table_scores=sc0)
    assert np.array_equal(d_ids.cpu().numpy(), ref_ids)
    np.testing.assert_allclose(d_sc.cpu().numpy(), ref_sc, rtol=2e-5, atol=1e-9)
    c.close()


def test_harvest_row_that_defeats_the_prefilter():
    """More than a thousand large logits sitting in nine residue classes of the column index: the
    kernel's short candidate list overflows and it must take its plain route; results unchanged."""
    dev = "cuda:0"
    V, B, K = 32000, 3, 10
    c = _ctx(V)
    rng = np.random.default_rng(9)
    logits = rng.normal(size=(B, V)).astype(np.float32)
    cols = np.arange(V)
    logits[1, cols % 256 < 9] += 50.0
    logits[2, :] = 1.5                                            # all equal: ids 0..K-1 in order
    tokens = np.array([5, 6, 7], np.int32)
    d_ids = torch.full((V, K), -1, dtype=torch.int32, device=dev)
    d_sc = torch.zeros((V, K), dtype=torch.float32, device=dev)
    c.goose_harvest_topk(torch.from_numpy(logits).to(dev), V, torch.from_numpy(tokens).to(dev), B, K, d_ids, d_sc)
    torch.cuda.synchronize()
    ref_ids, ref_sc = orc.harvest_topk(logits.astype(np.float64), tokens, K)
    assert np.array_equal(d_ids.cpu().numpy(), ref_ids)
    np.testing.assert_allclose(d_sc.cpu().numpy(), ref_sc, rtol=2e-5, atol=1e-12)
    assert ref_ids[7].tolist() == list(range(K))
    c.close()


def test_harvest_inside_the_fused_step():
    shape = gi.SHAPES["small_bf16"]
    tm = torch_model(shape, seed=2, gain_jitter=0.1)
    gm = gpu_model(shape, tm, max_B=128, cap=256)
    dev = gm.device
    tree = gi.tree_spine_7b(3)
    B, K = tree.B, 10
    tokens = gi.draft_tokens_uniform(5, tree.parent, shape.vocab, 11)
    tokens[40] = tokens[3]                                                  # a repeated token
    t, p, s = gm.stage_tree(tokens, tree.parent, tree.is_spine)
    results = []
    for want_logits in (True, False):
        gm.set_P(0)
        ids = torch.full((shape.vocab, K), -1, dtype=torch.int32, device=dev)
        sc = torch.zeros((shape.vocab, K), dtype=torch.float32, device=dev)
        logits = torch.empty((B, shape.vocab), dtype=torch.float32, device=dev) if want_logits else None
        gm.verify_step_fused(t, p, s, B, 128, logits=logits, succ_ids=ids, succ_scores=sc)
        torch.cuda.synchronize()
        results.append((ids.cpu().numpy(), sc.cpu().numpy(), None if logits is None else logits.cpu().numpy()))
    ids_a, sc_a, gl = results[0]
    ref_ids, ref_sc = orc.harvest_topk(gl.astype(np.float64), tokens, K)
    assert np.array_equal(ids_a, ref_ids)
    np.testing.assert_allclose(sc_a, ref_sc, rtol=2e-5, atol=1e-9)
    # the tables do not depend on whether the caller also asked for the logits
    assert np.array_equal(results[1][0], ids_a) and np.array_equal(results[1][1], sc_a)
    # every node's first successor is its greedy prediction
    am = gm.argmax[:B].cpu().numpy()
    last = {int(tok): i for i, tok in enumerate(tokens)}
    for tok, i in last.items():
        assert ids_a[tok, 0] == am[i]
    gm.ctx.close()
