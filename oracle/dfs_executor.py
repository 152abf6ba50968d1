"""Oracle C: the paper's push / pop execution with an active stack, one segment
at a time.  TEST INFRASTRUCTURE ONLY (never imported by the product path).

The vanilla dynamic-tree-attention backward (paper section 3.1; pseudocode
appendix, algorithm "Vanilla Dynamic Tree Attention Backward" and the
notation block with the FWD / BWD primitives) walks the prefix tree depth
first and keeps an active stack S with the tokens and the key/value cache of
the current root-to-node path:

  push   FWD(depth(u) -> depth(v)): forward the child's token segment on top of
         the stack (its queries see the whole stack and, causally, the segment
         itself), then append the segment's keys/values to the stack;
  visit  recurse into the child's subtree;
  pop    BWD(depth(v) -> depth(u)): backpropagate the segment's attached
         gradients; its queries send gradient into every key/value on the
         stack, where it is accumulated; when a segment is popped, all of its
         descendants have already added theirs, so its key/value gradient is
         final.

This file writes those steps out for the attention layer alone, in fp64, in
the paper's order: the attached gradient of a segment is the per-tree-token dO
(the sum over the rollouts that share the token).  Nothing is tiled or
reordered beyond what the algorithm states.  Chunked pops (the Pop_ByChunk
procedure of the optimised algorithm: boundaries t_0 < ... < t_m, chunks run
from the last to the first, each with its own FWD and BWD) are available per
segment because the product exposes calls on parts of a segment.

Pinned in tests/test_oracle_pins.py: the executor's tensors equal the
rollout-expansion oracle (a different formulation), a chain reduces to
torch's scaled_dot_product_attention, central finite differences of one
segment call, FWD/BWD counts and peak stack length (= longest path), and
invariance to how a segment is cut into chunks.
"""
from __future__ import annotations

import numpy as np

from .tree_layout import children_lists, node_offsets


def fwd_segment(q_seg, k_stack, v_stack, scale):
    """FWD of one segment for one head.

    k_stack, v_stack: [L,d], the active stack INCLUDING the segment itself as
    its last m rows; q_seg: [m,d].  Query j (stack position L-m+j) sees stack
    positions 0 .. L-m+j.  Returns O [m,d], LSE [m], P [m,L]."""
    m, L = q_seg.shape[0], k_stack.shape[0]
    s = scale * (q_seg @ k_stack.T)
    pos = np.arange(L - m, L)[:, None]
    s = np.where(np.arange(L)[None, :] <= pos, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    l = e.sum(axis=1, keepdims=True)
    p = e / l
    return p @ v_stack, (mx + np.log(l))[:, 0], p


def bwd_segment(q_seg, k_stack, v_stack, o_seg, p, do_seg, scale):
    """BWD of one segment for one head: gradient of sum(O_seg * dO_seg).

    Returns dQ_seg [m,d] (final for these tokens) and the segment's
    CONTRIBUTIONS dK, dV [L,d] to every key/value on the stack, which the
    caller accumulates."""
    dv = p.T @ do_seg
    dp = do_seg @ v_stack.T
    delta = (do_seg * o_seg).sum(axis=1, keepdims=True)
    ds = p * (dp - delta)
    return scale * (ds @ k_stack), scale * (ds.T @ q_seg), dv


def chunk_boundaries(lo, hi, block):
    """Evenly spaced t_0 = lo < t_1 < ... < t_m = hi with t_{j+1} - t_j <= block
    (Pop_ByChunk's first step).  block <= 0 or >= hi - lo gives one chunk."""
    n = hi - lo
    if block <= 0 or block >= n:
        return [lo, hi]
    m = -(-n // block)
    return [lo + (n * j) // m for j in range(m + 1)]


def vanilla_dta(parent, seg_len, q, k, v, do, scale, chunk_block=0):
    """Runs the push / pop traversal over the whole forest.

    q, do: [T,Hq,d]; k, v: [T,Hkv,d] in the packed DFS order (preorder,
    children in ascending node id).  Returns a dict with O, LSE, dQ, dK, dV,
    the call trace [('FWD'|'BWD', node, t_begin, t_end)] in execution order and
    the peak number of tokens on the stack.  With chunk_block > 0 every pop
    is cut into chunks of at most that many tokens, run last chunk first, each
    preceded by a recomputing FWD of the chunk (which is traced as 'REFWD')."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    roots, kids = children_lists(parent)
    off, _ = node_offsets(parent, seg_len)

    O = np.full((T, Hq, d), np.nan)
    LSE = np.full((T, Hq), np.nan)
    dQ = np.full((T, Hq, d), np.nan)
    dK = np.full((T, Hkv, d), np.nan)
    dV = np.full((T, Hkv, d), np.nan)
    trace = []
    stack = []                       # packed token index of every stack position
    gk = np.zeros((0, Hkv, d))       # gradient accumulated so far into the stack's keys
    gv = np.zeros((0, Hkv, d))       # ... and values
    peak = 0

    def fwd(lo, hi, node, tag):
        """Segment = stack positions [lo, hi); the stack already holds it."""
        idx = np.asarray(stack[:hi])
        own = idx[lo:hi]
        for h in range(Hq):
            g = h // G
            o, lse, _ = fwd_segment(q[own, h], k[idx, g], v[idx, g], scale)
            O[own, h] = o
            LSE[own, h] = lse
        trace.append((tag, node, int(own[0]), int(own[-1]) + 1))

    def bwd(lo, hi, node):
        idx = np.asarray(stack[:hi])
        own = idx[lo:hi]
        for h in range(Hq):
            g = h // G
            o, _, p = fwd_segment(q[own, h], k[idx, g], v[idx, g], scale)   # the graph FWD built
            dq, dk, dv = bwd_segment(q[own, h], k[idx, g], v[idx, g], o, p, do[own, h], scale)
            dQ[own, h] = dq
            gk[:hi, g] += dk
            gv[:hi, g] += dv
        trace.append(("BWD", node, int(own[0]), int(own[-1]) + 1))

    def dfs(v_node):
        nonlocal gk, gv, peak
        lo = len(stack)
        n = int(seg_len[v_node])
        # push
        stack.extend(range(int(off[v_node]), int(off[v_node]) + n))
        gk = np.concatenate([gk, np.zeros((n, Hkv, d))])
        gv = np.concatenate([gv, np.zeros((n, Hkv, d))])
        peak = max(peak, len(stack))
        fwd(lo, lo + n, v_node, "FWD")
        for c in kids[v_node]:
            dfs(c)
        # pop, last chunk first; a chunk's own keys are final once it has run
        bounds = chunk_boundaries(lo, lo + n, chunk_block)
        for j in range(len(bounds) - 2, -1, -1):
            if len(bounds) > 2:
                fwd(bounds[j], bounds[j + 1], v_node, "REFWD")
            bwd(bounds[j], bounds[j + 1], v_node)
            own = np.asarray(stack[bounds[j]:bounds[j + 1]])
            dK[own] = gk[bounds[j]:bounds[j + 1]]
            dV[own] = gv[bounds[j]:bounds[j + 1]]
            del stack[bounds[j]:]
            gk = gk[:bounds[j]]
            gv = gv[:bounds[j]]

    for r in roots:
        dfs(r)
    return dict(O=O, LSE=LSE, dQ=dQ, dK=dK, dV=dV, trace=trace, peak_stack=peak)
