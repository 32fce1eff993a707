"""Token and byte accounting on a fork tree (test infrastructure).

Follows the two savings metrics of the APAR paper, Sec. 3.4:
  * attended tokens - how many tokens are attended to when a given token is
    predicted.  In a fork tree that is the number of tokens before it on its own
    root path; in the flattened (ordinary auto-regressive) reference it is the
    token's position in the linearised sequence (node, then its children's
    subtrees in order: root / first-child / next-sibling order);
  * cached tokens - KV slots held.  With prefix sharing the live leaves of a tree
    hold every token of the tree once; a layout that copies the prefix on each
    fork (App. C.1) holds every leaf's whole root path.
A tree is given as parallel lists: parents[i] (-1 for a root, else < i) and
seg_lens[i] (tokens node i generated itself).
"""
from __future__ import annotations

from typing import List, Sequence


def _children(parents: Sequence[int]) -> List[List[int]]:
    ch: List[List[int]] = [[] for _ in parents]
    for i, p in enumerate(parents):
        if p >= 0:
            ch[p].append(i)
    return ch


def prefix_lens(parents: Sequence[int], seg_lens: Sequence[int]) -> List[int]:
    """Tokens on the root path strictly above each node."""
    pre = [0] * len(parents)
    for i, p in enumerate(parents):
        pre[i] = 0 if p < 0 else pre[p] + seg_lens[p]
    return pre


def path_lens(parents: Sequence[int], seg_lens: Sequence[int]) -> List[int]:
    pre = prefix_lens(parents, seg_lens)
    return [pre[i] + seg_lens[i] for i in range(len(parents))]


def flatten_offsets(parents: Sequence[int], seg_lens: Sequence[int]) -> List[int]:
    """Position of each node's first token in the linearised sequence of its tree."""
    ch = _children(parents)
    off = [0] * len(parents)

    def walk(i: int, pos: int) -> int:
        off[i] = pos
        pos += seg_lens[i]
        for c in ch[i]:
            pos = walk(c, pos)
        return pos

    for i, p in enumerate(parents):
        if p < 0:
            walk(i, 0)
    return off


def attended_tokens_tree(parents: Sequence[int], seg_lens: Sequence[int]) -> int:
    """Sum over every token of the tokens it attends to (itself included) on its root path."""
    pre = prefix_lens(parents, seg_lens)
    return sum(s * pre[i] + s * (s + 1) // 2 for i, s in enumerate(seg_lens))


def attended_tokens_flatten(parents: Sequence[int], seg_lens: Sequence[int]) -> int:
    off = flatten_offsets(parents, seg_lens)
    return sum(s * off[i] + s * (s + 1) // 2 for i, s in enumerate(seg_lens))


def leaf_ids(parents: Sequence[int]) -> List[int]:
    ch = _children(parents)
    return [i for i in range(len(parents)) if not ch[i]]


def cached_tokens_shared(parents: Sequence[int], seg_lens: Sequence[int]) -> int:
    """Tokens held when every leaf is live and prefixes are shared: each token once."""
    return sum(seg_lens)


def cached_tokens_copied(parents: Sequence[int], seg_lens: Sequence[int]) -> int:
    """Tokens held by the copied-prefix layout: every leaf's whole root path."""
    pl = path_lens(parents, seg_lens)
    return sum(pl[i] for i in leaf_ids(parents))


def kv_bytes(tokens: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    return tokens * 2 * n_kv_heads * head_dim * elem_bytes
