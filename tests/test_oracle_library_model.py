"""Pin of the oracle's whole-model forward against an independent library implementation.

The paper runs stock Llama-family checkpoints through the Hugging Face
Transformers stack (Sec. 5.1 "Setup", App. C hardware/software table).  Loading
the same random-init weights into that library's Llama model and comparing
logits pins every convention the oracle had to choose (norm, rotary pairing,
score scale, SwiGLU, weight orientation), for the plain causal run and for the
packed tree pass with an explicit mask and position ids.
"""
import numpy as np
import pytest
import torch

import goose_inputs as gi
from oracle import goose_oracle as orc
from util import oracle_model, torch_model

transformers = pytest.importorskip("transformers")

# The library evaluates the rotary cos/sin tables in fp32 whatever the model dtype, so agreement
# stops near 2e-7 on logits of size ~0.3; any convention mistake shows up at 1e-2 or more.
ATOL = 2e-6


def _hf_model(shape, tm):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(
        vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn,
        num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
        num_key_value_heads=shape.kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
        rope_theta=shape.rope_base, max_position_embeddings=4096, tie_word_embeddings=False,
        attention_bias=False, mlp_bias=False, hidden_act="silu", attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": tm["embed"], "lm_head.weight": tm["lm_head"],
          "model.norm.weight": tm["final_norm"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj",
             "g1": "input_layernorm", "g2": "post_attention_layernorm"}
    for l, lw in enumerate(tm["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{l}.{names[k]}.weight"] = v
    missing, unexpected = m.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not [k for k in missing if "rotary" not in k] and not unexpected
    return m


@pytest.fixture(scope="module")
def models():
    shape = gi.SHAPES["tiny"]
    tm = torch_model(shape, seed=3, gain_jitter=0.2)
    return shape, oracle_model(shape, tm), _hf_model(shape, tm)


def test_causal_logits_match_library(models):
    shape, om, hf = models
    toks = gi.prefix_tokens(5, 40, shape.vocab)
    mine, _ = orc.causal_logits(om, toks)
    with torch.no_grad():
        ref = hf(input_ids=torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    assert np.abs(ref).max() > 0.05
    np.testing.assert_allclose(mine, ref, rtol=0, atol=ATOL)


def test_tree_logits_match_library_with_explicit_mask(models):
    shape, om, hf = models
    P = 24
    prefix = gi.prefix_tokens(6, P, shape.vocab)
    tree = gi.tree_random(13, seed=4, spine_len=4)
    toks = gi.draft_tokens_uniform(7, tree.parent, shape.vocab, root_token=11)
    mine, _ = orc.tree_logits(om, orc.prefill(om, prefix), toks, tree.parent)

    # the library run gets the packed sequence prefix+nodes, a hand-built additive mask and positions
    B = tree.B
    allow = np.zeros((P + B, P + B), dtype=bool)
    allow[:P, :P] = np.tril(np.ones((P, P), dtype=bool))
    pos = list(range(P)) + [0] * B
    for i in range(B):
        allow[P + i, :P] = True
        v, hops = i, 0
        while v != -1:
            allow[P + i, P + v] = True
            v = int(tree.parent[v])
            hops += 1
        pos[P + i] = P + hops - 1
    add = torch.zeros(1, 1, P + B, P + B, dtype=torch.float64)
    add.masked_fill_(~torch.from_numpy(allow)[None, None], float("-inf"))
    ids = torch.from_numpy(np.concatenate([prefix, toks]).astype(np.int64))[None]
    with torch.no_grad():
        ref = hf(input_ids=ids, attention_mask=add, position_ids=torch.tensor(pos)[None]).logits[0, P:].numpy()
    np.testing.assert_allclose(mine, ref, rtol=0, atol=ATOL)


# ---- the grouped-query and QK-norm variants (the other model families of Sec. 5.1) ------------------
def _hf_qwen3(shape, tm):
    from transformers import Qwen3Config, Qwen3ForCausalLM
    cfg = Qwen3Config(
        vocab_size=shape.vocab, hidden_size=shape.hidden, intermediate_size=shape.ffn,
        num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_heads,
        num_key_value_heads=shape.kv_heads, head_dim=shape.head_dim, rms_norm_eps=shape.rms_eps,
        rope_theta=shape.rope_base, max_position_embeddings=4096, tie_word_embeddings=False,
        attention_bias=False, hidden_act="silu", attn_implementation="eager", use_sliding_window=False)
    m = Qwen3ForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": tm["embed"], "lm_head.weight": tm["lm_head"],
          "model.norm.weight": tm["final_norm"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj",
             "g1": "input_layernorm", "g2": "post_attention_layernorm", "gq": "self_attn.q_norm",
             "gk": "self_attn.k_norm"}
    for l, lw in enumerate(tm["layers"]):
        for k, v in lw.items():
            sd[f"model.layers.{l}.{names[k]}.weight"] = v
    missing, unexpected = m.load_state_dict({k: v.double() for k, v in sd.items()}, strict=False)
    assert not [k for k in missing if "rotary" not in k] and not unexpected
    return m


@pytest.mark.parametrize("kind", ["gqa", "gqa_qknorm"])
def test_grouped_query_and_qk_norm_match_library(kind):
    base = gi.SHAPES["tiny"]
    shape = gi.ModelShape("t", 2, base.hidden, 4, 64, base.ffn, base.vocab, dtype="f32", n_kv_heads=2,
                          qk_norm=(kind == "gqa_qknorm"), rms_eps=1e-6 if kind == "gqa_qknorm" else 1e-5)
    tm = torch_model(shape, seed=8, gain_jitter=0.2)
    om = oracle_model(shape, tm)
    hf = _hf_qwen3(shape, tm) if shape.qk_norm else _hf_model(shape, tm)
    toks = gi.prefix_tokens(9, 33, shape.vocab)
    mine, _ = orc.causal_logits(om, toks)
    with torch.no_grad():
        ref = hf(input_ids=torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    assert np.abs(ref).max() > 0.05
    np.testing.assert_allclose(mine, ref, rtol=0, atol=ATOL)
    # and the tree pass stays consistent with per-path causal runs for these variants
    tree = gi.tree_random(9, seed=2, spine_len=3)
    dt = gi.draft_tokens_uniform(3, tree.parent, shape.vocab, root_token=5)
    packed, _ = orc.tree_logits(om, orc.prefill(om, toks), dt, tree.parent)
    brute = orc.path_logits_bruteforce(om, toks, dt, tree.parent)
    np.testing.assert_allclose(packed, brute, rtol=0, atol=1e-10)
