"""Oracle K: gradient of chosen keys/values, summed over every query that sees them.
TEST INFRASTRUCTURE ONLY (never imported by the product path).

The pop step of paper section 3.1 back-propagates a node only after all of its
descendants have added their gradient to the node's keys and values, and the
objective is the plain sum over rollouts (equation 1).  Written out for one
key kappa that lives in node u, for one kv head and the q heads h of its group:

    visible(kappa) = tokens of u at or after kappa  +  all tokens of u's descendants
    for t in visible(kappa):
        s_tk  = scale * q[t,h] . k[k]          for every key k on t's root path
        lse_t = ln sum_k exp(s_tk)
        p_tk  = exp(s_tk - lse_t)
        o_t   = sum_k p_tk v[k]
        D_t   = dO[t,h] . o_t
    dV[kappa] = sum_h sum_t p_{t,kappa} dO[t,h]
    dK[kappa] = scale * sum_h sum_t p_{t,kappa} (dO[t,h] . v[kappa] - D_t) q[t,h]

The code below does exactly this, one node of queries at a time: the nodes whose
root path contains a requested key are found by walking parent[], each such
node's rows are evaluated in full against their own root path (as in the
tree-direct oracle, but written with torch ops so that the same lines can run
on a GPU's fp64 units when a full-size tree makes the host too slow), and the
columns of the requested keys are summed up.  Rows of a node are independent
of each other; `max_rows` only limits how many are held in memory at once.

Nothing here is shared with the HIP library.  Pinned in
tests/test_oracle_pins.py against the dense per-rollout oracle, against central
finite differences of a token-by-token brute-force objective, and against the
column-sum identity of softmax.
"""
from __future__ import annotations

import numpy as np
import torch

from .tree_layout import children_lists, node_offsets, node_path


def _as64(x, device):
    if isinstance(x, torch.Tensor):
        return x.to(device=device, dtype=torch.float64)
    return torch.as_tensor(np.asarray(x), dtype=torch.float64, device=device)


def key_gradients(parent, seg_len, q, k, v, do, scale, keys, device="cpu", max_rows=None):
    """dK, dV rows of the packed key indices `keys` for ONE kv head.

    q, do : [T, G, d]  the G q heads of the group;  k, v : [T, d]  the kv head
    keys  : 1-D ints, packed token indices (any order, no repeats)
    Returns (dK [len(keys), d], dV [len(keys), d]) as fp64 numpy arrays, and the
    number of (query row, key) pairs evaluated, for reporting."""
    parent = np.asarray(parent, dtype=np.int64)
    seg_len = np.asarray(seg_len, dtype=np.int64)
    keys = np.asarray(keys, dtype=np.int64)
    q, k, v, do = (_as64(x, device) for x in (q, k, v, do))
    T, G, d = q.shape
    off, total = node_offsets(parent, seg_len)
    assert total == T and k.shape == (T, d) and len(set(keys.tolist())) == len(keys)

    # node that owns each requested key
    node_of_token = np.empty(T, dtype=np.int64)
    for u in range(len(parent)):
        node_of_token[off[u]:off[u] + seg_len[u]] = u
    owners = set(int(node_of_token[x]) for x in keys)

    # every node whose root path contains an owner: the owners and their descendants
    _, kids = children_lists(parent)
    query_nodes, stack = set(), list(owners)
    while stack:
        u = stack.pop()
        if u in query_nodes:
            continue
        query_nodes.add(u)
        stack.extend(kids[u])

    slot_of_token = np.full(T, -1, dtype=np.int64)      # position of a token in `keys`, -1 = not requested
    slot_of_token[keys] = np.arange(len(keys))
    dK = torch.zeros((len(keys), d), dtype=torch.float64, device=device)
    dV = torch.zeros_like(dK)
    pairs = 0
    for w in sorted(query_nodes):
        path = node_path(parent, w)
        ctx = np.concatenate([np.arange(off[a], off[a] + seg_len[a]) for a in path])
        n_own = int(seg_len[w])
        n_anc = len(ctx) - n_own
        # which context columns are requested keys, and where their sums go
        cols = np.flatnonzero(slot_of_token[ctx] >= 0)
        if len(cols) == 0:
            continue
        slots = torch.as_tensor(slot_of_token[ctx[cols]], device=device)
        cols_t = torch.as_tensor(cols, device=device)
        ctx_t = torch.as_tensor(ctx, device=device)
        k_ctx, v_ctx = k[ctx_t], v[ctx_t]
        step = n_own if not max_rows else int(max_rows)
        for r0 in range(0, n_own, step):
            r1 = min(n_own, r0 + step)
            rows = torch.arange(off[w] + r0, off[w] + r1, device=device)
            # row r of the node (0-based inside it) sees ancestors and own tokens 0..r
            hidden = torch.arange(len(ctx), device=device)[None, :] > (n_anc + torch.arange(r0, r1, device=device))[:, None]
            for h in range(G):
                s = scale * (q[rows, h] @ k_ctx.T)
                s = s.masked_fill(hidden, float("-inf"))
                lse = torch.logsumexp(s, dim=1, keepdim=True)
                p = torch.exp(s - lse)
                o = p @ v_ctx
                delta = (do[rows, h] * o).sum(dim=1, keepdim=True)
                p_sel = p[:, cols_t]                                   # [rows, requested keys in ctx]
                dp_sel = do[rows, h] @ v_ctx[cols_t].T
                ds_sel = p_sel * (dp_sel - delta)
                dV.index_add_(0, slots, p_sel.T @ do[rows, h])
                dK.index_add_(0, slots, scale * (ds_sel.T @ q[rows, h]))
            pairs += (r1 - r0) * len(ctx)
    return dK.cpu().numpy(), dV.cpu().numpy(), pairs
