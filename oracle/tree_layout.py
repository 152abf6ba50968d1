"""Oracle-side tree bookkeeping (integer only).  TEST INFRASTRUCTURE ONLY.

The prefix tree is the one of the paper's section 3 (problem formulation): a
node is a token segment shared by a subset of the rollouts and every
root-to-leaf path is one rollout.  Path length ("depth") is counted in tokens,
as in the footnote of the space-complexity paragraph of section 3.1.

Packing convention (the paper leaves the DFS order free, section 4 only notes
that the lexicographic order is one valid DFS order): nodes are laid out in
DFS preorder, roots and children visited in ascending node id, and a node's
tokens are contiguous.  This module derives that order on its own; it shares
no code with the library's builder and is compared against it in the tests.
"""
from __future__ import annotations

import numpy as np


def children_lists(parent):
    parent = np.asarray(parent, dtype=np.int64)
    kids = [[] for _ in range(len(parent))]
    roots = []
    for i, p in enumerate(parent):
        if p < 0:
            roots.append(i)
        else:
            kids[int(p)].append(i)
    return roots, kids


def preorder(parent):
    """Node ids in DFS preorder, roots/children in ascending id."""
    roots, kids = children_lists(parent)
    order = []
    stack = list(reversed(roots))
    while stack:
        u = stack.pop()
        order.append(u)
        stack.extend(reversed(kids[u]))
    if len(order) != len(parent):
        raise ValueError("parent[] is not a forest (cycle or unreachable node)")
    return order


def node_offsets(parent, seg_len):
    """offset[u] = index of node u's first token in the packed order."""
    seg_len = np.asarray(seg_len, dtype=np.int64)
    off = np.zeros(len(seg_len), dtype=np.int64)
    t = 0
    for u in preorder(parent):
        off[u] = t
        t += int(seg_len[u])
    return off, t


def start_depths(parent, seg_len):
    """start_depth[u] = number of tokens above node u on its root path."""
    parent = np.asarray(parent, dtype=np.int64)
    seg_len = np.asarray(seg_len, dtype=np.int64)
    sd = np.zeros(len(parent), dtype=np.int64)
    for u in preorder(parent):
        p = int(parent[u])
        sd[u] = 0 if p < 0 else sd[p] + seg_len[p]
    return sd


def leaves(parent):
    _, kids = children_lists(parent)
    return [u for u in range(len(parent)) if not kids[u]]


def node_path(parent, u):
    """Nodes from the root down to u (inclusive)."""
    path = []
    while u >= 0:
        path.append(int(u))
        u = int(parent[u])
    return path[::-1]


def rollout_token_paths(parent, seg_len):
    """One int64 index vector per leaf (in ascending leaf id): the packed token
    indices of that rollout, root first.  'All rollout sequences are located at
    leaf nodes' (notation block of the pseudocode appendix)."""
    off, _ = node_offsets(parent, seg_len)
    out = []
    for leaf in leaves(parent):
        idx = [np.arange(off[u], off[u] + int(seg_len[u]), dtype=np.int64)
               for u in node_path(parent, leaf)]
        out.append(np.concatenate(idx))
    return out


def ancestor_token_indices(parent, seg_len, off, u):
    """Packed indices of every token strictly above node u, root first."""
    nodes = node_path(parent, u)[:-1]
    if not nodes:
        return np.zeros(0, dtype=np.int64)
    return np.concatenate([np.arange(off[a], off[a] + int(seg_len[a]), dtype=np.int64)
                           for a in nodes])


def tree_stats(parent, seg_len):
    """Counts used for reporting.

    C = total sequence tokens / unique tree tokens and S = 1 - 1/C follow the
    caption of the paper's figure 1.  The paper gives no formula for C_attn
    (appendix B.2 only calls it the effective reuse in attention computation);
    the reading used here is dense causal pairs over unique tree pairs.
    'leaf' counts only root-to-leaf rollouts; 'full' lets every node end a
    rollout (the figure's full-tree count)."""
    parent = np.asarray(parent, dtype=np.int64)
    seg_len = np.asarray(seg_len, dtype=np.int64)
    sd = start_depths(parent, seg_len)
    end = sd + seg_len
    lv = leaves(parent)
    n_tokens = int(seg_len.sum())
    # unique (query, visible key) pairs: a token at 0-based position p sees p+1 keys
    unique_pairs = int(sum(int(seg_len[u]) * int(sd[u]) + int(seg_len[u]) * (int(seg_len[u]) + 1) // 2
                           for u in range(len(parent))))
    roll_leaf = int(sum(int(end[u]) for u in lv))
    roll_full = int(end.sum())
    dense_leaf = int(sum(int(end[u]) * (int(end[u]) + 1) // 2 for u in lv))
    dense_full = int(sum(int(e) * (int(e) + 1) // 2 for e in end))
    return dict(n_nodes=len(parent), n_tokens=n_tokens, n_leaves=len(lv),
                max_path_tokens=int(end.max()), unique_pairs=unique_pairs,
                rollout_tokens=roll_leaf, rollout_tokens_full=roll_full,
                dense_pairs=dense_leaf, dense_pairs_full=dense_full,
                C_leaf=roll_leaf / n_tokens, C_full=roll_full / n_tokens,
                C_attn_leaf=dense_leaf / unique_pairs, C_attn_full=dense_full / unique_pairs)
