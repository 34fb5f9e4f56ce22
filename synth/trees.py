"""Candidate-tree shapes (inputs to the step, never computed on the hot path).

A tree is a fixed subset of the full top-k tree of Sec. 2.1: node 0 is the
root, a node at depth D carries the rank (index into draft head D's top-k list)
that selects its token.  Nodes are listed in canonical order: by depth, then by
the lexicographic order of the rank path from the root, so parent[n] < n and
"leftmost" equals "smallest index among nodes of equal depth".

The trees of the paper come from calibration on speech data (Sec. 2.4) that is
not available here; `make_tree` is the stand-in: it keeps the M nodes with the
largest path probability under a synthetic per-edge acceptance model
p(head i, rank r) = alpha0 * decay**(i-1) * g(r),  g(r) = (1-q) q**r / (1-q**cap_i).
"""
from dataclasses import dataclass
import heapq
import math
from typing import Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class TreeSpec:
    parent: np.ndarray   # int32 [M], parent[0] = -1
    rank: np.ndarray     # int32 [M], rank[0] = 0 (unused)
    depth: np.ndarray    # int32 [M]
    paths: Tuple[Tuple[int, ...], ...]   # rank path of every node

    @property
    def n_nodes(self) -> int:
        return int(self.parent.shape[0])

    @property
    def max_depth(self) -> int:
        return int(self.depth.max())


def _from_paths(paths: Sequence[Tuple[int, ...]]) -> TreeSpec:
    paths = sorted(set(paths), key=lambda p: (len(p), p))
    index = {p: i for i, p in enumerate(paths)}
    M = len(paths)
    parent = np.full(M, -1, np.int32)
    rank = np.zeros(M, np.int32)
    depth = np.zeros(M, np.int32)
    for i, p in enumerate(paths):
        if p:
            parent[i] = index[p[:-1]]   # KeyError here means the set is not ancestor-closed
            rank[i] = p[-1]
            depth[i] = len(p)
    return TreeSpec(parent=parent, rank=rank, depth=depth, paths=tuple(paths))


def edge_prob(i: int, r: int, cap: int, alpha0=0.75, decay=0.85, q=0.6) -> float:
    """Synthetic acceptance probability of rank r under draft head i (1-based)."""
    g = (1.0 - q) * q ** r / (1.0 - q ** cap)
    return alpha0 * decay ** (i - 1) * g


def make_tree(n_nodes: int, topk_caps: Sequence[int], alpha0=0.75, decay=0.85, q=0.6) -> TreeSpec:
    """The n_nodes nodes (root included) of largest path probability."""
    heap = [(0.0, 0, ())]          # (-log prob rounded, depth, path)
    chosen = []
    while heap and len(chosen) < n_nodes:
        neg, dep, path = heapq.heappop(heap)
        chosen.append(path)
        if dep < len(topk_caps):
            cap = topk_caps[dep]
            for r in range(cap):
                lp = -neg + math.log(edge_prob(dep + 1, r, cap, alpha0, decay, q))
                heapq.heappush(heap, (round(-lp, 9), dep + 1, path + (r,)))
    return _from_paths(chosen)


def path_probs(tree: TreeSpec, topk_caps: Sequence[int], alpha0=0.75, decay=0.85, q=0.6):
    out = []
    for p in tree.paths:
        pr = 1.0
        for i, r in enumerate(p):
            pr *= edge_prob(i + 1, r, topk_caps[i], alpha0, decay, q)
        out.append(pr)
    return np.array(out)


def chain_tree(n_nodes: int) -> TreeSpec:
    """Root plus one rank-0 child per level (plain multi-token draft, no branching)."""
    return _from_paths([tuple([0] * d) for d in range(n_nodes)])


def full_tree(branching: Sequence[int]) -> TreeSpec:
    """The full top-k tree with branching[i] children under every depth-i node."""
    paths = [()]
    level = [()]
    for k in branching:
        level = [p + (r,) for p in level for r in range(k)]
        paths += level
    return _from_paths(paths)


def tree_from_paths(paths) -> TreeSpec:
    return _from_paths([tuple(p) for p in paths])
