"""Candidate-tree bookkeeping derived from parent pointers (oracle; test infrastructure only).

The paper evaluates with tree attention by default (section 4.1 contrasts it
with chain drafts); the tree itself is an input.  Node 0 is the root, and
parent[i] < i.
"""
from __future__ import annotations

import numpy as np


def tree_depths(parent):
    d = np.zeros(len(parent), dtype=np.int64)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def ancestor_mask(parent):
    """mask[i, j] = True iff j is i itself or an ancestor of i."""
    T = len(parent)
    m = np.zeros((T, T), dtype=bool)
    for i in range(T):
        m[i, i] = True
        if parent[i] >= 0:
            m[i] |= m[parent[i]]
    return m


def children_lists(parent):
    ch = [[] for _ in parent]
    for i in range(1, len(parent)):
        ch[parent[i]].append(i)
    return ch


def expanded_nodes(parent):
    """Nodes that have at least one child in the template, in index order."""
    ch = children_lists(parent)
    return [i for i in range(len(parent)) if ch[i]]
