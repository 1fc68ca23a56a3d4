"""Seeded synthetic inputs for the tree-verification path.

This module only *produces inputs*: model shapes, weight bytes, prefix token
ids, draft-tree parent arrays and draft token ids.  It holds none of the
method's arithmetic (no mask, depth, attention, argmax, walk or compaction):
the CPU oracle and the HIP library each derive those on their own from what
is generated here.  Both sides, the tests and the benchmark import it.

Everything is a pure function of integer seeds.  Weight values come from a
counter-based 32-bit integer hash evaluated with exact integer arithmetic in
int64 tensors, so the CPU and a GPU produce identical bytes.
"""
from .shapes import ModelShape, SHAPES, shape_by_name  # noqa: F401
from .weights import (  # noqa: F401
    hash32,
    gen_normal,
    layer_weights,
    embedding,
    lm_head,
    norm_gain,
    final_norm,
    TENSOR_IDS,
)
from .trees import (  # noqa: F401
    Tree,
    tree_chain,
    tree_star,
    tree_single,
    tree_tiny_spine,
    tree_spine_7b,
    tree_spine_13b,
    tree_spine_33b,
    tree_spine_stress,
    tree_balanced,
    tree_random,
    relabel_topological,
)
from .tokens import (  # noqa: F401
    prefix_tokens,
    draft_tokens_uniform,
    draft_tokens_pld_like,
    plant_drafts,
)
