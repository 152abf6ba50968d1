"""Oracle E: the paper's backward DFS order and its leaf-order schedule with
chunked pops.  TEST INFRASTRUCTURE ONLY (never imported by the product path).
Integer work; results must match bit for bit.

Backward DFS order (pseudocode appendix, algorithm "Backward DFS Order";
section 3.2): in postorder every leaf gets tail = its depth in tokens; an
internal node orders its children by (is internal, tail) ascending, i.e. leaf
children first and, within a kind, the smaller tail first, and takes the tail
of its first child.  The leaf order of the DFS that uses these child orders,
reversed, is the order pi in which the leaves are processed.  Readings: ties
are broken by node id; the roots of a forest are ordered by the same key.

Leaf-order schedule (algorithm "Dynamic Tree Attention Backward", section
3.2): for each leaf of pi in turn, the part of the active stack that the new
leaf does not share is popped (Pop_ByChunk: evenly spaced boundaries at most B
apart, chunks run from the last to the first, each with a recomputing FWD and
a BWD), the new suffix is forwarded and pushed, and, if the next pop will
leave part of what was just forwarded on the stack, a FWD-NoGrad materialises
that part as a detached cache anchor; after the last leaf everything is
popped.  The schedule is returned as a list of operations on depth ranges of
the current leaf's root path:

  ('FWD',    leaf, lo, hi)   regular forward of positions lo+1..hi (push)
  ('REFWD',  leaf, lo, hi)   forward of one chunk inside Pop_ByChunk
  ('BWD',    leaf, lo, hi)   backward of that chunk (its positions are popped)
  ('NOGRAD', leaf, lo, hi)   FWD-NoGrad anchor

`leaf` names the root-to-leaf path whose depths the range refers to (for pops
that is the previous leaf).  block <= 0 means an infinite block size.

Pinned in tests/test_oracle_pins.py: a hand-worked example, stack discipline
(every position is pushed once, popped once, chunks <= B and evenly spaced),
the paper's operation counts (one regular FWD per leaf, at most one FWD-NoGrad
per leaf), and invariance: running the operations with the segment primitives
of the push/pop oracle reproduces the rollout-expansion gradients.
"""
from __future__ import annotations

import numpy as np

from .tree_layout import children_lists, node_offsets, node_path, start_depths


def _end_depths(parent, seg_len):
    return start_depths(parent, seg_len) + np.asarray(seg_len, dtype=np.int64)


def backward_dfs_order(parent, seg_len):
    """Leaves (node ids) in the order pi."""
    roots, kids = children_lists(parent)
    end = _end_depths(parent, seg_len)
    n = len(parent)
    tail = [0] * n
    key = lambda u: (1 if kids[u] else 0, tail[u], u)
    # postorder = reversed preorder with children pushed in any fixed order
    pre, stack = [], list(roots)
    while stack:
        u = stack.pop()
        pre.append(u)
        stack.extend(kids[u])
    for v in reversed(pre):
        if not kids[v]:
            tail[v] = int(end[v])
        else:
            kids[v].sort(key=key)
            tail[v] = tail[kids[v][0]]
    rho, stack = [], sorted(roots, key=key)[::-1]
    while stack:
        u = stack.pop()
        if not kids[u]:
            rho.append(u)
        stack.extend(reversed(kids[u]))
    return rho[::-1]


def common_prefix_tokens(parent, seg_len, a, b):
    """LCP of the token sequences of the root paths of nodes a and b."""
    end = _end_depths(parent, seg_len)
    l = 0
    for x, y in zip(node_path(parent, a), node_path(parent, b)):
        if x != y:
            break
        l = int(end[x])
    return l


def chunk_boundaries(lo, hi, block):
    n = hi - lo
    if block <= 0 or block >= n:
        return [lo, hi]
    m = -(-n // block)
    return [lo + (n * j) // m for j in range(m + 1)]


def schedule(parent, seg_len, block=0):
    """Operation list of the leaf-order schedule, and pi."""
    pi = backward_dfs_order(parent, seg_len)
    end = _end_depths(parent, seg_len)
    ops = []

    def pop_by_chunk(leaf, hi, lo):
        b = chunk_boundaries(lo, hi, block) if hi > lo else [lo]
        for j in range(len(b) - 2, -1, -1):
            ops.append(("REFWD", leaf, b[j], b[j + 1]))
            ops.append(("BWD", leaf, b[j], b[j + 1]))

    l_backward = 0
    for i, s in enumerate(pi):
        n = int(end[s])
        if i > 0:
            l_lcp = common_prefix_tokens(parent, seg_len, pi[i - 1], s)
            pop_by_chunk(pi[i - 1], l_backward, l_lcp)
        else:
            l_lcp = 0
        ops.append(("FWD", s, l_lcp, n))
        l_backward = n
        l_anchor = common_prefix_tokens(parent, seg_len, s, pi[i + 1]) if i + 1 < len(pi) else 0
        p_pop = n - l_anchor
        if block > 0 and p_pop >= block:
            m = -(-p_pop // block)
            l_anchor = n - (-(-p_pop // m))
        if l_lcp < l_anchor:
            ops.append(("NOGRAD", s, l_lcp, l_anchor))
    if pi:
        pop_by_chunk(pi[-1], l_backward, 0)
    return ops, pi


def path_ranges(parent, seg_len, leaf, lo, hi):
    """Packed token ranges [(t0, t1)], one per node, of depths [lo, hi) on the
    root path of `leaf`, root side first."""
    off, _ = node_offsets(parent, seg_len)
    sd = start_depths(parent, seg_len)
    out = []
    for u in node_path(parent, leaf):
        a, b = max(lo, int(sd[u])), min(hi, int(sd[u]) + int(seg_len[u]))
        if a < b:
            out.append((int(off[u]) + a - int(sd[u]), int(off[u]) + b - int(sd[u])))
    return out
