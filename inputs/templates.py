"""Retrieval templates: static, unbalanced trees over successor ranks (input structure only).

The paper fixes, per pruning stage, how many retrieved nodes there are at each of the nine
retrieval depths (App. A.1, table "Retrieval templates"), that a stage's template is a prefix
of one root-centred envelope (Sec. 3.2), and the design principle: higher-ranked successors
get more children and reach deeper, the greedy chain reaches depth 9.  It does not print the
rank paths.  This module builds them with one stated rule: a node's cost is the sum of the
ranks on its path; at every depth a template takes the cheapest children of the previous
depth's nodes (ties: smaller rank path first), and a larger stage keeps every node of the
smaller one.  Nothing here does any lookup: the arrays are inputs of the retrieval step, of
the CPU oracle and of the GPU library alike.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

# retrieved nodes per depth 1..9 (App. A.1, table of retrieval templates)
STAGE_DEPTH_COUNTS: Dict[str, Tuple[int, ...]] = {
    "d5": (4, 3, 3, 2, 2, 2, 2, 1, 1),
    "d1": (6, 7, 5, 4, 4, 3, 3, 2, 2),
    "d0": (8, 10, 8, 6, 5, 4, 4, 4, 3),
    "full": (8, 16, 14, 11, 8, 7, 6, 5, 5),
}
STAGE_ORDER = ("d5", "d1", "d0", "full")          # each one a prefix of the next
# retained draft nodes per stage (Sec. 3.2; App. A "Stage-adaptive budget")
STAGE_DRAFT_NODES = {"d5": 40, "d1": 24, "d0": 8}


def retrieval_envelope():
    """The 80-node envelope in prefix order.

    Returns (tpl_parent int32 [80], tpl_rank int32 [80], tpl_depth int32 [80], sizes) where
    tpl_parent[u] is the index of the parent template node (-1: child of the tree's root),
    tpl_rank[u] the successor rank looked up from the parent's token, and sizes[stage] the
    number of leading nodes that form that stage's template.
    """
    paths: List[Tuple[int, ...]] = []              # envelope so far, prefix order
    have = set()
    sizes = {}
    for stage in STAGE_ORDER:
        counts = STAGE_DEPTH_COUNTS[stage]
        new_nodes: List[Tuple[int, ...]] = []
        for d in range(1, 10):
            level = [p for p in list(have) + new_nodes if len(p) == d]
            need = counts[d - 1] - len(level)
            assert need >= 0, "stage templates are nested per depth"
            parents = [()] if d == 1 else [p for p in list(have) + new_nodes if len(p) == d - 1]
            cand = []
            for p in parents:
                n_child = sum(1 for q in level if q[:-1] == p)
                for r in range(n_child, n_child + need):   # ranks stay contiguous per parent
                    cand.append((sum(p) + r, p + (r,)))
            cand.sort()
            chosen: List[Tuple[int, ...]] = []
            for _, path in cand:
                if len(chosen) == need:
                    break
                # rank r of a parent can only be taken once ranks 0..r-1 are
                r, par = path[-1], path[:-1]
                if r == 0 or (par + (r - 1,)) in have or (par + (r - 1,)) in new_nodes + chosen:
                    chosen.append(path)
            assert len(chosen) == need
            new_nodes += chosen
        new_nodes.sort(key=lambda p: (len(p), sum(p), p))
        paths += new_nodes
        have.update(new_nodes)
        sizes[stage] = len(paths)
    index = {p: i for i, p in enumerate(paths)}
    tpl_parent = np.array([-1 if len(p) == 1 else index[p[:-1]] for p in paths], np.int32)
    tpl_rank = np.array([p[-1] for p in paths], np.int32)
    tpl_depth = np.array([len(p) for p in paths], np.int32)
    return tpl_parent, tpl_rank, tpl_depth, sizes


def rank_paths(tpl_parent, tpl_rank):
    """Rank path [r_1..r_d] of every template node."""
    out = []
    for u in range(len(tpl_parent)):
        p, v = [], u
        while v >= 0:
            p.append(int(tpl_rank[v]))
            v = int(tpl_parent[v])
        out.append(tuple(reversed(p)))
    return out
