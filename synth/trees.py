"""Seeded synthetic draft trees (input generation only: no arithmetic of the method).

The paper verifies 60 candidate tokens per step of the target model, arranged
by its drafter as a tree; the drafter is out of reach here, so random trees of
the same size stand in: every node picks its parent among the earlier nodes (or
the committed prefix) that still have room for a child.
"""
from __future__ import annotations

import numpy as np
import torch

from . import workloads


def random_trees(rng: np.random.Generator, B: int, M: int, max_children: int = 4) -> np.ndarray:
    """parent int32 [B, M] in drafting order: parent[b, i] in [-1, i), -1 = the prefix."""
    parent = np.empty((B, M), dtype=np.int32)
    for b in range(B):
        count = {-1: 0}
        for i in range(M):
            open_nodes = [p for p, c in count.items() if c < max_children]
            p = int(rng.choice(open_nodes))
            parent[b, i] = p
            count[p] += 1
            count[i] = 0
    return parent


def level_order(parent: np.ndarray) -> np.ndarray:
    """The same trees with their nodes renumbered level by level, the children of a node next to
    each other (the order in which a tree drafter that expands a level at a time lists its
    candidates): parent int32 [B, M], still with parent[b, i] < i."""
    B, M = parent.shape
    out = np.empty_like(parent)
    for b in range(B):
        kids = {}
        for i in range(M):
            kids.setdefault(int(parent[b, i]), []).append(i)
        order, new_parent = [], []
        frontier = [(-1, -1)]                   # (old node, its new number)
        while frontier:
            nxt = []
            for old, new in frontier:
                for c in kids.get(old, []):
                    order.append(c)
                    new_parent.append(new)
                    nxt.append((c, len(order) - 1))
            frontier = nxt
        out[b] = np.array(new_parent, dtype=np.int32)
    return out


def tree_step(cfg, parent: np.ndarray, step: int, variant: str = "plain", device="cpu"):
    """One verification step over B trees: a pair of logit rows per context (the prefix and every
    node: M + 1 rows per tree), row_index[i] = the row after node i's parent, and as draft token of
    the j-th child of a context the j-th most likely token of the drafter's row.

    Returns (Step with B*(M+1) rows, row_index int32 [B*M], tokens int32 [B*M], uniforms [B*M, 2])
    with the arrays as numpy on the host and the Step / uniforms on `device`."""
    B, M = parent.shape
    st = workloads.make_step(cfg, step=step, rows=B * (M + 1), variant=variant, device=device)
    row_index = (np.arange(B, dtype=np.int64)[:, None] * (M + 1) + parent + 1).astype(np.int32)
    rank = np.zeros((B, M), dtype=np.int64)
    for b in range(B):
        seen = {}
        for i in range(M):
            rank[b, i] = seen.get(parent[b, i], 0)
            seen[parent[b, i]] = rank[b, i] + 1
    top = torch.topk(st.draft_logits.float(), int(rank.max()) + 1, dim=1).indices.cpu().numpy()
    tokens = top[row_index.reshape(-1), rank.reshape(-1)].astype(np.int32)
    un = st.uniforms[: B * M].contiguous()
    return st, row_index.reshape(-1), tokens, un
