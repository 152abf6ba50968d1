"""Synthetic rollout prefix trees, given as (parent[], seg_len[]) arrays.

A node is a token segment shared by every rollout that passes through it; a
root-to-leaf path is one rollout (paper section 3, problem formulation).  The
five shapes below stand in for the paper's tau^2-bench / GRPO rollouts, which
are not available: a shared prompt with sampled responses, a multi-turn agent
forest with a shared system prompt, a deep long-context tree, and a large mixed
forest.  Three more (6..8) take the shape of the paper's low-compression
settings (appendix, throughput under low compression rates): short shared
prefixes, C between 1.4 and 1.01.  All draws use numpy's PCG64 via default_rng(seed) so that every run,
on any machine, sees the same trees.
"""
from __future__ import annotations

import numpy as np

# name -> (tree seed, tensor seed)
CONFIGS = {1: (1001, 2001), 2: (1002, 2002), 3: (1003, 2003), 4: (1004, 2004), 5: (1005, 2005),
           6: (1006, 2006), 7: (1007, 2007), 8: (1008, 2008)}

_HEADS = {
    1: dict(n_q_heads=4, n_kv_heads=4, head_dim=64, dtype="f32"),
    2: dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16"),
    3: dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16"),
    4: dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16"),
    5: dict(n_q_heads=64, n_kv_heads=8, head_dim=128, dtype="bf16"),
    6: dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16"),
    7: dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16"),
    8: dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16"),
}


def config_heads(cfg: int) -> dict:
    """Head counts, head_dim and dtype of benchmark configuration `cfg` (1..8)."""
    return dict(_HEADS[cfg])


def _as_arrays(parent, seg_len):
    return np.asarray(parent, dtype=np.int32), np.asarray(seg_len, dtype=np.int32)


def _cfg1():
    parent = [-1] + [0] * 4 + [1 + (i - 5) // 2 for i in range(5, 13)]
    seg = [128] + [32] * 4 + [16] * 8
    return _as_arrays(parent, seg)


def _cfg2(rng, prompt=1024, n_resp=16, lo=256, hi=2048):
    parent = [-1] + [0] * n_resp
    seg = [prompt] + [int(x) for x in rng.integers(lo, hi + 1, size=n_resp)]
    return _as_arrays(parent, seg)


def _cfg3(rng, sys_len=4096, n_dialogues=8, n_turns=6, lo=128, hi=1024, p_branch=0.3):
    parent, seg = [-1], [sys_len]
    for _ in range(n_dialogues):
        # turn 1 is a single node under the system prompt; after each of turns
        # 1..n_turns-1 the next turn has two children with probability p_branch
        frontier = [len(parent)]
        parent.append(0)
        seg.append(int(rng.integers(lo, hi + 1)))
        for _turn in range(1, n_turns):
            nxt = []
            for node in frontier:
                nchild = 2 if rng.random() < p_branch else 1
                for _c in range(nchild):
                    nxt.append(len(parent))
                    parent.append(node)
                    seg.append(int(rng.integers(lo, hi + 1)))
            frontier = nxt
    return _as_arrays(parent, seg)


def _cfg4(root=16384, levels=8, seg=512):
    parent, segs = [-1], [root]
    frontier = [0]
    for _ in range(levels):
        nxt = []
        for node in frontier:
            for _c in range(2):
                nxt.append(len(parent))
                parent.append(node)
                segs.append(seg)
        frontier = nxt
    return _as_arrays(parent, segs)


def _cfg5(rng, n_trees=64, cap=262144, min_len=16):
    parent, seg = [], []
    for _ in range(n_trees):
        root = len(parent)
        parent.append(-1)
        seg.append(int(rng.integers(512, 8192 + 1)))
        depth = int(rng.integers(1, 6))
        frontier = [root]
        for _lvl in range(depth):
            nxt = []
            for node in frontier:
                for _c in range(int(rng.integers(1, 5))):
                    nxt.append(len(parent))
                    parent.append(node)
                    seg.append(int(round(float(np.exp(rng.uniform(np.log(32.0), np.log(2048.0)))))))
            frontier = nxt
    seg = np.asarray(seg, dtype=np.float64)
    # one global scale brings the forest to the token cap while keeping the
    # shape of the length distributions; the floor keeps segments non-trivial
    scale = min(1.0, cap / float(seg.sum()))
    seg = np.maximum(min_len, np.rint(seg * scale)).astype(np.int32)
    return np.asarray(parent, dtype=np.int32), seg, scale


def _prompt_groups(rng, n_prompts, n_resp, prompt_lo, prompt_hi, resp_lo, resp_hi):
    """A forest of `n_prompts` trees: a prompt and `n_resp` sampled responses."""
    parent, seg = [], []
    for _ in range(n_prompts):
        root = len(parent)
        parent.append(-1)
        seg.append(int(rng.integers(prompt_lo, prompt_hi + 1)))
        for x in rng.integers(resp_lo, resp_hi + 1, size=n_resp):
            parent.append(root)
            seg.append(int(x))
    return _as_arrays(parent, seg)


def _cfg6(rng):
    # agent rollouts with the global prompt removed: what is left to share is the
    # first part of each dialogue (average rollout about 1.6K tokens, C about 1.4)
    return _prompt_groups(rng, 64, 2, 700, 1100, 400, 1000)


def _cfg7(rng):
    # grade-school-maths style: a short question, 8 long sampled answers
    # (average rollout about 1.8K tokens, C about 1.09)
    return _prompt_groups(rng, 8, 8, 100, 240, 800, 2500)


def _cfg8(rng):
    # competition-maths style: one short problem, 16 answers of about 16K tokens
    # (C about 1.008)
    return _prompt_groups(rng, 1, 16, 130, 130, 12288, 20480)


def config_tree(cfg: int):
    """Return (parent, seg_len, info) for benchmark configuration `cfg` (1..8)."""
    rng = np.random.default_rng(CONFIGS[cfg][0])
    info = {"cfg": cfg, "tree_seed": CONFIGS[cfg][0], "tensor_seed": CONFIGS[cfg][1]}
    if cfg == 1:
        p, s = _cfg1()
    elif cfg == 2:
        p, s = _cfg2(rng)
    elif cfg == 3:
        p, s = _cfg3(rng)
    elif cfg == 4:
        p, s = _cfg4()
    elif cfg == 5:
        p, s, scale = _cfg5(rng)
        info["length_scale"] = scale
    elif cfg == 6:
        p, s = _cfg6(rng)
    elif cfg == 7:
        p, s = _cfg7(rng)
    elif cfg == 8:
        p, s = _cfg8(rng)
    else:
        raise ValueError(f"unknown config {cfg}")
    return p, s, info


def scaled_config_tree(cfg: int, shrink: int):
    """A sibling of configuration `cfg` with every segment length divided by
    `shrink` (floor 1, ragged remainders kept by rounding up odd cases), small
    enough for the exhaustive CPU oracle but with the same branching."""
    p, s, info = config_tree(cfg)
    s = np.maximum(1, (s.astype(np.int64) + shrink - 1) // shrink).astype(np.int32)
    if cfg == 4:
        # keep the tree deep but not 511 nodes wide: cut to 4 branching levels
        keep = 1 + 2 + 4 + 8 + 16
        p, s = p[:keep], s[:keep]
    if cfg == 5:
        # keep the first trees of the forest only
        roots = np.flatnonzero(p < 0)
        cut = int(roots[6]) if len(roots) > 6 else len(p)
        p, s = p[:cut], s[:cut]
    info["shrink"] = shrink
    return p, s, info


def chain_tree(lengths):
    """A single path: node i+1 is the only child of node i."""
    lengths = list(lengths)
    parent = [-1] + list(range(len(lengths) - 1))
    return _as_arrays(parent, lengths)


def random_tree(rng, n_nodes: int, max_len: int, n_roots: int = 1, shuffle_ids: bool = True):
    """A random forest with `n_nodes` nodes whose ids are NOT in DFS order when
    `shuffle_ids` is set, so that the packing permutation is exercised."""
    n_roots = min(n_roots, n_nodes)
    parent = np.full(n_nodes, -1, dtype=np.int64)
    for i in range(n_roots, n_nodes):
        parent[i] = int(rng.integers(0, i))
    seg = rng.integers(1, max_len + 1, size=n_nodes).astype(np.int64)
    if shuffle_ids:
        perm = rng.permutation(n_nodes)           # new id of old node i
        new_parent = np.full(n_nodes, -1, dtype=np.int64)
        new_seg = np.zeros(n_nodes, dtype=np.int64)
        for old in range(n_nodes):
            new_parent[perm[old]] = -1 if parent[old] < 0 else perm[parent[old]]
            new_seg[perm[old]] = seg[old]
        parent, seg = new_parent, new_seg
    return parent.astype(np.int32), seg.astype(np.int32)
