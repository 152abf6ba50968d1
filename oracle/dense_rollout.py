"""Oracle A: expand every rollout and run ordinary dense causal attention.
TEST INFRASTRUCTURE ONLY (never imported by the product path).

Dynamic tree attention is an exact reorganisation: a shared prefix is
forwarded once and reused by the descendant rollouts, and the gradients of all
descendant rollouts are accumulated into it (paper section 3.1, push / leaf /
pop steps), while the objective is the plain sum of per-rollout losses
(equation 1).  The plain definition of the result is therefore: treat every
root-to-leaf rollout as an independent sequence, run causal softmax attention
on it, and sum the per-rollout gradients of every shared token.  That is what
this file writes out, in fp64, one rollout and one head at a time.

Conventions where the paper is silent: scaled dot-product softmax attention,
causal including the diagonal; grouped-query heads map q head h to kv head
h // (Hq // Hkv); LSE is the natural log of the sum of exp(scale * q.k).

Pinned (tests/test_oracle_pins.py) against torch's scaled_dot_product_attention
on a chain, closed forms with K = 0, central finite differences, an explicit
T x T ancestor-mask brute force, and algebraic invariants of softmax.
"""
from __future__ import annotations

import numpy as np

from .tree_layout import rollout_token_paths


def dense_causal_forward(q, k, v, scale):
    """One sequence, one head.  q,k,v: [n,d] fp64.  Returns O [n,d], LSE [n], P [n,n]."""
    n = q.shape[0]
    s = scale * (q @ k.T)
    s = np.where(np.tril(np.ones((n, n), dtype=bool)), s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    p = e / l
    return p @ v, (m + np.log(l))[:, 0], p


def dense_causal_backward(q, k, v, o, p, do, scale):
    """Gradient of sum(O * dO) w.r.t. q, k, v for one sequence and one head."""
    dv = p.T @ do
    dp = do @ v.T
    delta = (do * o).sum(axis=1, keepdims=True)
    ds = p * (dp - delta)
    dq = scale * (ds @ k)
    dk = scale * (ds.T @ q)
    return dq, dk, dv


def forward(parent, seg_len, q, k, v, scale, q_heads=None, rollouts=None, return_spread=False):
    """Tree O [T,Hq,d] and LSE [T,Hq] from per-rollout dense attention.

    Every rollout that contains a token produces a value for it; these must
    agree (a token's output depends only on its prefix).  The first writer's
    value is kept and the largest disagreement is returned when asked.
    Entries of heads / tokens not covered by q_heads / rollouts stay NaN."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T, Hq, d = q.shape
    G = Hq // k.shape[1]
    paths = rollout_token_paths(parent, seg_len)
    if rollouts is not None:
        paths = [paths[i] for i in rollouts]
    heads = range(Hq) if q_heads is None else q_heads
    O = np.full((T, Hq, d), np.nan)
    LSE = np.full((T, Hq), np.nan)
    spread = 0.0
    for idx in paths:
        for h in heads:
            o, lse, _ = dense_causal_forward(q[idx, h], k[idx, h // G], v[idx, h // G], scale)
            seen = ~np.isnan(LSE[idx, h])
            if seen.any():
                spread = max(spread, float(np.abs(O[idx[seen], h] - o[seen]).max()),
                             float(np.abs(LSE[idx[seen], h] - lse[seen]).max()))
            O[idx[~seen], h] = o[~seen]
            LSE[idx[~seen], h] = lse[~seen]
    return (O, LSE, spread) if return_spread else (O, LSE)


def equal_split_weights(parent, seg_len, n_tokens):
    """w[i][j] = 1 / (number of rollouts containing token path_i[j])."""
    paths = rollout_token_paths(parent, seg_len)
    cnt = np.zeros(n_tokens, dtype=np.float64)
    for idx in paths:
        cnt[idx] += 1.0
    return [1.0 / cnt[idx] for idx in paths]


def backward(parent, seg_len, q, k, v, do, scale, weights=None, q_heads=None):
    """Tree dQ [T,Hq,d], dK, dV [T,Hkv,d].

    do is the upstream gradient per TREE token, i.e. already the sum over the
    rollouts sharing the token.  It is split back into per-rollout gradients
    dO_i = w_i * dO with weights that sum to one over the rollouts containing
    each token (equal split unless given); each rollout is backpropagated as an
    independent dense sequence and the gradients are scatter-added per token
    (and, for K and V, over the q heads of each group)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    paths = rollout_token_paths(parent, seg_len)
    if weights is None:
        weights = equal_split_weights(parent, seg_len, T)
    heads = range(Hq) if q_heads is None else q_heads
    dQ = np.zeros((T, Hq, d))
    dK = np.zeros((T, Hkv, d))
    dV = np.zeros((T, Hkv, d))
    for idx, w in zip(paths, weights):
        for h in heads:
            g = h // G
            o, _, p = dense_causal_forward(q[idx, h], k[idx, g], v[idx, g], scale)
            dq, dk, dv = dense_causal_backward(q[idx, h], k[idx, g], v[idx, g], o, p,
                                               do[idx, h] * np.asarray(w)[:, None], scale)
            # idx has no repeated entries, so fancy-index += is a true scatter-add
            dQ[idx, h] += dq
            dK[idx, g] += dk
            dV[idx, g] += dv
    return dQ, dK, dV
