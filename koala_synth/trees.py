"""Static candidate-tree templates.

A template fixes, before any token is known, which (depth, rank-path) slots the
draft head will fill.  It is an *input* of the method: the library and the
oracle both receive `parent[]`, `rank[]` and `topk_per_depth[]` and derive
depths, masks and positions from them on their own.

Construction: level 0 is the root.  The candidates of level d are the children
of rank 0..k_d-1 of every node kept at level d-1; they are ordered by (sum of
ranks on the path from the root, then the rank path lexicographically) and the
first w_d of them are kept.  Nodes are numbered level by level in that order,
so parent[i] < i.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class TreeTemplate:
    parent: np.ndarray          # int32[T], parent[0] = -1
    rank: np.ndarray            # int32[T], rank among the parent's top-k (root: 0)
    topk_per_depth: np.ndarray  # int32[D], k_1..k_D
    depth: int                  # D
    paths: tuple                # rank path of every node (root: ())

    @property
    def n_nodes(self) -> int:
        return int(self.parent.shape[0])


def make_tree(topk, widths) -> TreeTemplate:
    topk = [int(k) for k in topk]
    widths = [int(w) for w in widths]
    assert len(widths) == len(topk) + 1 and widths[0] == 1
    parent, rank, paths = [-1], [0], [()]
    level = [0]
    for d, k in enumerate(topk, start=1):
        cands = []
        for u in level:
            for r in range(k):
                p = paths[u] + (r,)
                cands.append((sum(p), p, u, r))
        cands.sort(key=lambda c: (c[0], c[1]))
        keep = cands[: widths[d]]
        assert len(keep) == widths[d], "level wider than its candidate set"
        nxt = []
        for _, p, u, r in keep:
            nxt.append(len(parent))
            parent.append(u)
            rank.append(r)
            paths.append(p)
        level = nxt
    return TreeTemplate(np.asarray(parent, np.int32), np.asarray(rank, np.int32),
                        np.asarray(topk, np.int32), len(topk), tuple(paths))


def chain_tree(length: int) -> TreeTemplate:
    """Root plus `length` descendants, one child per node (chain drafting)."""
    return make_tree([1] * length, [1] * (length + 1))
