"""LM head with the fused per-row top-2 reduction: ragged vocabularies, ties, logits on and off.

The prediction rule is the greedy argmax of the target distribution (Sec. 4.2, Alg. UnifiedGreedyWalk); ties go to
the lowest token id on both sides.
"""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import gpu_model, oracle_model, torch_model

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def _model(vocab, hidden=256, seed=5, dtype="bf16"):
    shape = gi.ModelShape(f"head_v{vocab}", 1, hidden, 4, hidden // 4, 688, vocab, dtype=dtype)
    tm = torch_model(shape, seed=seed, gain_jitter=0.1)
    return shape, tm


def _run(gm, x, B, want_logits):
    d = gm.desc
    logits = torch.full((B, d.vocab), float("nan"), dtype=torch.float32, device=gm.device) if want_logits else None
    am = torch.full((128,), -7, dtype=torch.int32, device=gm.device)
    mg = torch.full((128,), float("nan"), dtype=torch.float32, device=gm.device)
    gm.ctx.goose_lm_head_argmax(gm.packed_head, x, B, am, logits, mg)
    torch.cuda.synchronize()
    return am[:B].cpu().numpy(), mg[:B].cpu().numpy(), None if logits is None else logits.cpu().numpy()


@pytest.mark.parametrize("vocab,dtype", [(1000, "bf16"), (1024, "bf16"), (4093, "bf16"), (33, "bf16"), (4093, "f16")])
@pytest.mark.parametrize("B", [1, 33, 64, 100])
def test_top2_matches_the_logits_and_the_oracle(vocab, dtype, B):
    shape, tm = _model(vocab, dtype=dtype)
    TOL_BF16 = 2e-2 if dtype == "bf16" else 2.5e-3
    om = oracle_model(shape, tm)
    gm = gpu_model(shape, tm, max_B=128, cap=128)
    x = gi.gen_normal(77, 900 + B, (B, shape.hidden), 1.0, torch.float32, "cpu")
    xd = x.to(gm.device)
    am, mg, gl = _run(gm, xd, B, True)
    ref = orc.final_logits(om, x.double().numpy())
    scale = np.abs(ref).max()
    assert np.abs(gl - ref).max() <= TOL_BF16 * scale
    # the reduction is exact with respect to the logits the kernel wrote
    assert np.array_equal(am, np.argmax(gl, axis=-1))
    part = np.partition(gl, -2, axis=-1)
    np.testing.assert_allclose(mg, part[:, -1] - part[:, -2], rtol=0, atol=0)
    # decisions agree with the oracle away from near-ties
    safe = orc.top2_margin(ref) > 2 * TOL_BF16 * scale
    assert np.array_equal(am[safe], np.argmax(ref, axis=-1)[safe])
    # without a logits buffer the same predictions come out
    am2, mg2, _ = _run(gm, xd, B, False)
    assert np.array_equal(am, am2) and np.array_equal(mg, mg2)
    gm.ctx.close()


def test_ties_go_to_the_lowest_token_id():
    shape, tm = _model(1000)
    row = tm["lm_head"][123].clone()
    tm["lm_head"][:] = row                      # every token gets the same logit
    gm = gpu_model(shape, tm, max_B=128, cap=128)
    x = gi.gen_normal(78, 901, (40, shape.hidden), 1.0, torch.float32, "cpu").to(gm.device)
    am, mg, gl = _run(gm, x, 40, True)
    assert (gl == gl[:, :1]).all()
    assert (am == 0).all() and (mg == 0).all()
    # one strictly larger pair of equal rows far apart: the lower one wins, margin stays zero
    tm["lm_head"][400] = 2 * row
    tm["lm_head"][911] = 2 * row
    gm.ctx.close()
    gm = gpu_model(shape, tm, max_B=128, cap=128)
    pos = (gl[:, 123] > 0)                      # sign of the common logit, from the first run
    am, mg, _ = _run(gm, x, 40, False)
    assert np.array_equal(am[pos], np.full(pos.sum(), 400)) and np.array_equal(am[~pos], np.zeros((~pos).sum()))
    assert (mg == 0).all()
    gm.ctx.close()
