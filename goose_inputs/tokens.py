"""Seeded token-id inputs: the committed prefix and the draft tokens on a tree.

Draft tokens are inputs to verification (the draft side of Sec. 4 is not part
of the verified path).  Siblings always carry distinct tokens, as the paper's
tree construction drops duplicates (Sec. 4.2, Alg. BuildSpineTree remark).
"""
import numpy as np


def prefix_tokens(seed: int, P: int, vocab: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 17])
    return rng.integers(0, vocab, size=P, dtype=np.int64).astype(np.int32)


def _fix_siblings(parent: np.ndarray, tokens: np.ndarray, vocab: int, rng, frozen=()) -> None:
    """Re-draw tokens (never those in `frozen`) until siblings are distinct."""
    B = len(parent)
    frozen = set(int(i) for i in frozen)
    seen = {}
    for i in range(1, B):
        key = int(parent[i])
        used = seen.setdefault(key, set())
        if i in frozen:
            used.add(int(tokens[i]))
    for i in range(1, B):
        if i in frozen:
            continue
        used = seen[int(parent[i])]
        while int(tokens[i]) in used:
            tokens[i] = rng.integers(0, vocab)
        used.add(int(tokens[i]))


def draft_tokens_uniform(seed: int, parent: np.ndarray, vocab: int, root_token: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 19])
    tokens = rng.integers(0, vocab, size=len(parent), dtype=np.int64).astype(np.int32)
    tokens[0] = root_token
    _fix_siblings(parent, tokens, vocab, rng)
    return tokens


def draft_tokens_pld_like(seed: int, parent: np.ndarray, is_spine: np.ndarray, vocab: int,
                          root_token: int, prefix: np.ndarray, copy_prob: float = 0.3) -> np.ndarray:
    """Uniform drafts, except that each spine position, with probability
    `copy_prob`, starts (or continues) copying the tokens that follow an earlier
    4-gram of the prefix, the way a context n-gram match fills the spine."""
    rng = np.random.default_rng([seed, 23])
    tokens = draft_tokens_uniform(seed, parent, vocab, root_token)
    spine = [i for i in range(1, len(parent)) if is_spine[i]]
    src = -1
    frozen = []
    for i in spine:
        if src < 0 or src >= len(prefix):
            if rng.random() < copy_prob and len(prefix) > 8:
                src = int(rng.integers(4, len(prefix) - 1))  # position right after a 4-gram
        if 0 <= src < len(prefix):
            tokens[i] = prefix[src]
            frozen.append(i)
            src += 1
            if rng.random() > 0.7:  # the copied run ends
                src = -1
    _fix_siblings(parent, tokens, vocab, rng, frozen)
    return tokens


def plant_drafts(seed: int, parent: np.ndarray, is_spine: np.ndarray, tokens: np.ndarray,
                 continuation: np.ndarray, vocab: int, p_spine: float = 0.6,
                 p_branch: float = 0.5, p_grand: float = 0.3) -> np.ndarray:
    """Write a known continuation into the drafts so that a walk accepts several nodes.

    `continuation[k-1]` is the token the model would emit k steps after the root
    (supplied by the caller; this function only arranges token ids).  The spine
    carries the continuation for a geometric number of nodes (success prob
    `p_spine`), then a deliberately different token; with probability `p_branch`
    one branch child of the last matching spine node carries the next
    continuation token (spine continuation, Sec. 4.2), and its own first child
    the one after that with probability `p_grand`.
    """
    rng = np.random.default_rng([seed, 29])
    tokens = tokens.copy()
    B = len(parent)
    children = [[] for _ in range(B)]
    for i in range(1, B):
        children[int(parent[i])].append(i)
    frozen = []
    v, k = 0, 0  # current node, number of continuation tokens placed
    while k < len(continuation):
        sp = [c for c in children[v] if is_spine[c]]
        if not sp or rng.random() >= p_spine:
            break
        tokens[sp[0]] = continuation[k]
        frozen.append(sp[0])
        v, k = sp[0], k + 1
    # break the spine below v on purpose
    for c in children[v]:
        if is_spine[c] and k < len(continuation):
            tokens[c] = (int(continuation[k]) + 1) % vocab
            frozen.append(c)
    br = [c for c in children[v] if not is_spine[c]]
    if br and k < len(continuation) and rng.random() < p_branch:
        c = br[int(rng.integers(0, len(br)))]
        tokens[c] = continuation[k]
        frozen.append(c)
        k += 1
        if children[c] and k < len(continuation) and rng.random() < p_grand:
            g = children[c][0]
            tokens[g] = continuation[k]
            frozen.append(g)
    _fix_siblings(parent, tokens, vocab, rng, frozen)
    return tokens
