"""goose_lm_head_argmax_static: the LM-head reduction for callers that cannot allocate.

Its workspace is a static device array instead of a context's buffers; its results must equal
goose_lm_head_argmax's bit for bit, also on a second, smaller call that finds the array dirty.
"""
import dataclasses

import numpy as np
import pytest
import torch

import goose_inputs as gi
import paper_2604_02047_amd as goose
from paper_2604_02047_amd import binding
from paper_2604_02047_amd.runner import GooseModel
from util import gpu_model, torch_model

pytestmark = pytest.mark.gpu


def _ctx_result(gm, x, B):
    am = torch.full((128,), -7, dtype=torch.int32, device=gm.device)
    mg = torch.full((128,), float("nan"), dtype=torch.float32, device=gm.device)
    gm.ctx.goose_lm_head_argmax(gm.packed_head, x, B, am, None, mg)
    torch.cuda.synchronize()
    return am[:B].cpu().numpy(), mg[:B].cpu().numpy()


def _static_result(gm, x, B):
    am = torch.full((128,), -7, dtype=torch.int32, device=gm.device)
    mg = torch.full((128,), float("nan"), dtype=torch.float32, device=gm.device)
    goose.goose_lm_head_argmax_static(gm.desc, gm.packed_head, x, B, am, mg)
    torch.cuda.synchronize()
    assert (am[B:] == -7).all()
    return am[:B].cpu().numpy(), mg[:B].cpu().numpy()


@pytest.mark.parametrize("dtype,act_mode", [("bf16", 0), ("bf16", 1), ("f16", 0)])
def test_static_workspace_matches_the_context_path(dtype, act_mode):
    shape = gi.ModelShape("head_static", 1, 512, 4, 128, 688, 4093, dtype=dtype)
    tm = torch_model(shape, seed=11, gain_jitter=0.1)
    desc = dataclasses.replace(goose.ModelDesc.from_shape(shape), act_mode=act_mode)
    gm = GooseModel(desc, 128, 128, lambda l: tm["layers"][l], tm["embed"], tm["lm_head"], tm["final_norm"])
    # two calls in a row, the second smaller: it finds the first call's rows and records in the array
    for B, stream_id in ((100, 910), (33, 911)):
        x = gi.gen_normal(79, stream_id, (B, shape.hidden), 1.0, torch.float32, "cpu").to(gm.device)
        x0 = x.clone()
        am_s, mg_s = _static_result(gm, x, B)
        am_c, mg_c = _ctx_result(gm, x, B)
        assert torch.equal(x, x0)
        assert np.array_equal(am_s, am_c)
        assert np.array_equal(mg_s, mg_c)
        assert (am_s >= 0).all() and (am_s < shape.vocab).all()
    gm.ctx.close()


def test_static_workspace_refuses_what_does_not_fit():
    shape = gi.ModelShape("head_static", 1, 256, 4, 64, 688, 1000, dtype="bf16")
    tm = torch_model(shape, seed=12)
    gm = gpu_model(shape, tm, max_B=128, cap=128)
    x = torch.zeros((256, shape.hidden), dtype=torch.float32, device=gm.device)
    am = torch.zeros((256,), dtype=torch.int32, device=gm.device)
    with pytest.raises(goose.GooseError) as e:
        goose.goose_lm_head_argmax_static(gm.desc, gm.packed_head, x, 129, am)
    assert e.value.status == binding.GOOSE_ERR_CAPACITY
    wide = dataclasses.replace(gm.desc, vocab=262145)
    with pytest.raises(goose.GooseError) as e:
        goose.goose_lm_head_argmax_static(wide, gm.packed_head, x, 8, am)
    assert e.value.status == binding.GOOSE_ERR_CAPACITY
    gm.ctx.close()
