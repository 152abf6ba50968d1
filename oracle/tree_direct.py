"""Oracle B: the per-token definition evaluated on the tree itself, no rollout
expansion.  TEST INFRASTRUCTURE ONLY (never imported by the product path).

Each unique tree token's query attends to exactly the keys on its root-to-node
path: the whole segments of its ancestor nodes plus the causal part of its own
segment (the 'push' step of paper section 3.1 runs a segment on top of the
parent prefix's cached keys/values).  Gradients flowing into a key are the sum
over every query that sees it, i.e. over all descendants (the 'pop' step).
Ancestors are found by walking parent[]; there is no tiling or reordering.

This second formulation exists so that full-size configurations, where
expanding all rollouts is far too slow, can still be checked on whole tensors
or sampled nodes.  It is tied to Oracle A (they must agree to ~1e-12) in
tests/test_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

from .tree_layout import node_offsets, ancestor_token_indices, preorder


def _node_scores(q_own, k_ctx, n_anc, scale):
    """Scores of one node's queries against [ancestor keys ++ own keys], with
    the causal mask on the own block."""
    m = q_own.shape[0]
    s = scale * (q_own @ k_ctx.T)
    own = s[:, n_anc:]
    own[np.triu(np.ones((m, m), dtype=bool), k=1)] = -np.inf
    return s


def forward(parent, seg_len, q, k, v, scale, q_heads=None, nodes=None):
    """O [T,Hq,d], LSE [T,Hq]; rows of nodes / heads not requested stay NaN."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T, Hq, d = q.shape
    G = Hq // k.shape[1]
    off, _ = node_offsets(parent, seg_len)
    heads = range(Hq) if q_heads is None else q_heads
    O = np.full((T, Hq, d), np.nan)
    LSE = np.full((T, Hq), np.nan)
    for u in (preorder(parent) if nodes is None else nodes):
        anc = ancestor_token_indices(parent, seg_len, off, u)
        own = np.arange(off[u], off[u] + int(seg_len[u]), dtype=np.int64)
        ctx = np.concatenate([anc, own])
        for h in heads:
            g = h // G
            s = _node_scores(q[own, h], k[ctx, g], len(anc), scale)
            mx = s.max(axis=1, keepdims=True)
            e = np.exp(s - mx)
            l = e.sum(axis=1, keepdims=True)
            O[own, h] = (e / l) @ v[ctx, g]
            LSE[own, h] = (mx + np.log(l))[:, 0]
    return O, LSE


def backward(parent, seg_len, q, k, v, do, scale, q_heads=None, nodes=None):
    """dQ [T,Hq,d], dK, dV [T,Hkv,d] for per-tree-token upstream gradient do.

    With nodes given, only those nodes' queries are processed: their dQ rows are
    complete, while dK/dV then hold only those queries' contributions."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    off, _ = node_offsets(parent, seg_len)
    heads = range(Hq) if q_heads is None else q_heads
    dQ = np.zeros((T, Hq, d))
    dK = np.zeros((T, Hkv, d))
    dV = np.zeros((T, Hkv, d))
    for u in (preorder(parent) if nodes is None else nodes):
        anc = ancestor_token_indices(parent, seg_len, off, u)
        own = np.arange(off[u], off[u] + int(seg_len[u]), dtype=np.int64)
        ctx = np.concatenate([anc, own])
        for h in heads:
            g = h // G
            s = _node_scores(q[own, h], k[ctx, g], len(anc), scale)
            mx = s.max(axis=1, keepdims=True)
            e = np.exp(s - mx)
            p = e / e.sum(axis=1, keepdims=True)
            o = p @ v[ctx, g]
            dp = do[own, h] @ v[ctx, g].T
            delta = (do[own, h] * o).sum(axis=1, keepdims=True)
            ds = p * (dp - delta)
            dQ[own, h] = scale * (ds @ k[ctx, g])
            dK[ctx, g] += scale * (ds.T @ q[own, h])
            dV[ctx, g] += p.T @ do[own, h]
    return dQ, dK, dV
