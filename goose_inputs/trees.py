"""Draft-tree shape generators (parent arrays in topological order).

A tree is the input the draft side hands to verification: node 0 is the root
(the anchor token of the cycle, Sec. 4), parent[0] = -1 and parent[i] < i.
`is_spine[i]` = 1 tags a context-match (spine) node, 0 a transition (branch)
node, the two source tags of Alg. UnifiedGreedyWalk.  The shapes follow the spine-tree family
of Alg. BuildSpineTree (deep chain + wider branches near the root); budgets and depths are
the benchmark configurations', not produced by running Alg. BuildSpineTree.
Nothing here computes masks, depths or positions.
"""
from dataclasses import dataclass

import numpy as np


@dataclass
class Tree:
    parent: np.ndarray    # int32 [B]
    is_spine: np.ndarray  # uint8 [B]

    @property
    def B(self) -> int:
        return int(self.parent.shape[0])


def _mk(parent, is_spine) -> Tree:
    p = np.asarray(parent, dtype=np.int32)
    s = np.asarray(is_spine, dtype=np.uint8)
    assert p.shape == s.shape and p[0] == -1
    assert all(0 <= p[i] < i for i in range(1, len(p)))
    return Tree(p, s)


def tree_single() -> Tree:
    """Root only: one ordinary decoding step (the fallback case of Alg. "Decoding Loop")."""
    return _mk([-1], [1])


def tree_chain(B: int) -> Tree:
    """Linear chain: the bypass mode's draft (Sec. 4.3)."""
    return _mk([-1] + list(range(B - 1)), [1] * B)


def tree_star(B: int) -> Tree:
    """All drafts are children of the root (a one-level transition-only tree)."""
    return _mk([-1] + [0] * (B - 1), [1] + [0] * (B - 1))


def tree_tiny_spine() -> Tree:
    """B=16: spine 0..7, node 8+i is one branch child of spine node i."""
    parent = [-1] + list(range(7)) + list(range(8))
    return _mk(parent, [1] * 8 + [0] * 8)


def _spine_with_branches(spine_len: int, widths, B: int, grandchild_rng=None) -> Tree:
    parent = [-1] + list(range(spine_len - 1))
    tag = [1] * spine_len
    for s in range(spine_len):
        for _ in range(widths[s]):
            if len(parent) >= B:
                break
            parent.append(s)
            tag.append(0)
            child = len(parent) - 1
            if grandchild_rng is not None and len(parent) < B and grandchild_rng.integers(0, 2) == 1:
                parent.append(child)
                tag.append(0)
    assert len(parent) == B, (len(parent), B)
    return _mk(parent, tag)


def tree_spine_7b(seed: int) -> Tree:
    """B=64: spine 0..15; walking down the spine each node gets up to 3 branch
    children, each followed by a grandchild with probability 1/2, until the
    budget of 64 nodes is used up."""
    rng = np.random.default_rng([seed, 7])
    return _spine_with_branches(16, [3] * 16, 64, rng)


def tree_spine_13b() -> Tree:
    """B=80: spine 0..19, 3 branch children per spine node."""
    return _spine_with_branches(20, [3] * 20, 80)


def tree_spine_33b() -> Tree:
    """B=80: spine 0..23, branch widths decaying 4 -> 1 down the spine (sum 56)."""
    widths = [4] * 4 + [3] * 4 + [2] * 12 + [1] * 4
    return _spine_with_branches(24, widths, 80)


def tree_spine_stress() -> Tree:
    """B=128: spine 0..31, 3 branch children per spine node."""
    return _spine_with_branches(32, [3] * 32, 128)


def tree_balanced(B: int = 128, fanout=(4, 3, 2, 2, 2)) -> Tree:
    """Breadth-first balanced tree with the given per-level fan-out, cut at B nodes
    (the isotropic control shape of Sec. 5.3)."""
    parent = [-1]
    level = [0]
    for f in fanout:
        nxt = []
        for v in level:
            for _ in range(f):
                if len(parent) >= B:
                    break
                parent.append(v)
                nxt.append(len(parent) - 1)
        level = nxt
    assert len(parent) == B
    # no context-match source in a balanced tree: every draft node is a branch node
    return _mk(parent, [1] + [0] * (B - 1))


def tree_random(B: int, seed: int, spine_len: int = 0) -> Tree:
    """Random recursive tree; the first `spine_len` nodes form a tagged chain."""
    rng = np.random.default_rng([seed, 11])
    parent = [-1]
    tag = [1]
    for i in range(1, B):
        if i < spine_len:
            parent.append(i - 1)
            tag.append(1)
        else:
            parent.append(int(rng.integers(0, i)))
            tag.append(0)
    return _mk(parent, tag)


def relabel_topological(tree: Tree, seed: int):
    """Another topological numbering of the same tree.  Returns (tree', perm) with
    perm[new] = old, so inputs permute as x'[new] = x[perm[new]]."""
    rng = np.random.default_rng([seed, 13])
    B = tree.B
    children = [[] for _ in range(B)]
    for i in range(1, B):
        children[tree.parent[i]].append(i)
    ready = [0]
    perm = []
    while ready:
        k = int(rng.integers(0, len(ready)))
        v = ready.pop(k)
        perm.append(v)
        ready.extend(children[v])
    inv = {old: new for new, old in enumerate(perm)}
    parent = [-1 if tree.parent[old] < 0 else inv[int(tree.parent[old])] for old in perm]
    tag = [int(tree.is_spine[old]) for old in perm]
    return _mk(parent, tag), np.asarray(perm, dtype=np.int64)
