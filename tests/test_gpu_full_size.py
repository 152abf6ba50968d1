"""GPU parity at the benchmark's full sizes (configurations 2-7, bf16), in the
launch configuration bench.py times.  The fp64 oracle cannot cover whole tensors
here, so it is run on sampled outputs it can compute one by one:

  * O, LSE and dQ rows of sampled nodes (tree-direct oracle, every q head of one
    kv group; a node's rows depend only on its own root path);
  * dK, dV rows of a sampled subtree's nodes: every query that sees those keys
    lies inside the subtree, so the oracle restricted to the subtree's queries is
    complete for them;
  * dK, dV of sampled SHARED-PREFIX keys (first tiles of the largest root, whose
    walks are the ones the schedule splits into partial sums; the boundary between
    a root and its first child; other roots of a forest; an interior node) against
    every descendant query, with the per-key oracle;
  * configuration 2: whole tensors, all five outputs, for one kv group;
and on properties that hold at any size:
  * sum_k dV[k, g] == sum over the group's q heads and all tokens of dO (rows of P
    sum to one), per kv head and feature;
  * sum_t q_t . dQ_t == sum_k k_k . dK_k per kv group (scores are bilinear);
  * token 0 of every root sees only itself: O = V, LSE = scale * q.k.
"""
import math

import numpy as np
import pytest
import torch

import paper_2602_00482_amd as dta
from oracle import key_gradient as K
from oracle import tree_direct as B
from oracle import tree_layout as L
from workloads import config_heads, config_tree

pytestmark = pytest.mark.gpu

TOL = 1e-2


def _run(cfg, heads=None):
    parent, seg, meta = config_tree(cfg)
    h = config_heads(cfg)
    Hq, Hkv, d = h["n_q_heads"], h["n_kv_heads"], h["head_dim"]
    if heads is not None:
        Hq, Hkv = heads
    T = int(seg.sum())
    g = torch.Generator(device="cuda")
    g.manual_seed(meta["tensor_seed"])
    mk = lambda heads: torch.randn((T, heads, d), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q, k, v, do = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
    scale = 1.0 / math.sqrt(d)
    p = dta.AttnParams(Hq, Hkv, d, scale, dta.BF16)
    tree = dta.tree_build(parent, seg)
    o, lse = dta.tree_attn_fwd(tree, p, q, k, v)
    dq, dk, dv = dta.tree_attn_bwd(tree, p, q, k, v, o, lse, do)
    torch.cuda.synchronize()
    tree.destroy()
    return parent, seg, (Hq, Hkv, d, scale), dict(q=q, k=k, v=v, do=do, o=o, lse=lse, dq=dq, dk=dk, dv=dv)


def _rel(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def _subtree_nodes(parent, root):
    kids = {}
    for i, pa in enumerate(parent):
        kids.setdefault(int(pa), []).append(i)
    out, stack = [], [root]
    while stack:
        u = stack.pop()
        out.append(u)
        stack.extend(kids.get(u, []))
    return out


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 6, 7, 8])
def test_full_size_sampled_rows_and_invariants(cfg):
    parent, seg, (Hq, Hkv, d, scale), t = _run(cfg)
    G = Hq // Hkv
    T = int(seg.sum())
    off, _ = L.node_offsets(parent, seg)
    sd = L.start_depths(parent, seg)
    rng = np.random.default_rng(cfg)
    grp = int(rng.integers(0, Hkv))                    # one whole kv group
    heads = list(range(grp * G, (grp + 1) * G))

    # ---------------- properties over whole tensors
    dv_sum = t["dv"].double().sum(dim=0).cpu().numpy()                               # [Hkv, d]
    do_sum = t["do"].double().view(T, Hkv, G, d).sum(dim=(0, 2)).cpu().numpy()
    assert np.abs(dv_sum - do_sum).max() / np.abs(do_sum).max() < TOL
    lhs = (t["q"].double() * t["dq"].double()).sum(dim=(0, 2)).view(Hkv, G).sum(dim=1).cpu().numpy()
    rhs = (t["k"].double() * t["dk"].double()).sum(dim=(0, 2)).cpu().numpy()
    assert np.abs(lhs - rhs).max() / max(np.abs(lhs).max(), np.abs(rhs).max()) < 2 * TOL
    for r in np.flatnonzero(parent < 0)[:8]:
        t0 = int(off[r])
        assert torch.equal(t["o"][t0].view(Hkv, G, d), t["v"][t0].unsqueeze(1).expand(Hkv, G, d))
        s0 = scale * (t["q"][t0].double().view(Hkv, G, d) * t["k"][t0].double().unsqueeze(1)).sum(-1)
        assert (t["lse"][t0].double().view(Hkv, G) - s0).abs().max().item() < 1e-4

    # ---------------- the oracle on slices: only the tokens it touches are copied to the host
    def oracle_on(nodes_for_queries):
        """Run the tree-direct oracle for the queries of these nodes on a compact
        copy of the tokens involved (their root paths)."""
        need = set()
        for u in nodes_for_queries:
            need.update(L.node_path(parent, u))
        keep = sorted(need, key=lambda u: off[u])
        remap = {u: i for i, u in enumerate(keep)}
        sub_parent = np.array([-1 if parent[u] < 0 else remap[int(parent[u])] for u in keep], dtype=np.int32)
        sub_seg = np.array([seg[u] for u in keep], dtype=np.int32)
        tok = np.concatenate([np.arange(off[u], off[u] + seg[u]) for u in keep])
        ti = torch.from_numpy(tok).cuda()
        sub = {n: t[n][ti][:, heads if n in ("q", "do") else [grp]].double().cpu().numpy() for n in ("q", "k", "v", "do")}
        qn = [remap[u] for u in nodes_for_queries]
        O, LSE = B.forward(sub_parent, sub_seg, sub["q"], sub["k"], sub["v"], scale, nodes=qn)
        dQ, dK, dV = B.backward(sub_parent, sub_seg, sub["q"], sub["k"], sub["v"], sub["do"], scale, nodes=qn)
        sub_off, _ = L.node_offsets(sub_parent, sub_seg)
        return keep, remap, sub_off, tok, O, LSE, dQ, dK, dV

    # (1) O, LSE, dQ on sampled nodes (deepest leaf, a random leaf, a random interior node)
    leaves = L.leaves(parent)
    deepest = max(leaves, key=lambda u: sd[u] + seg[u])
    picks = {deepest, int(rng.choice(leaves)), int(rng.integers(0, len(parent)))}
    for u in picks:
        keep, remap, sub_off, tok, O, LSE, dQ, _, _ = oracle_on([u])
        rows_sub = np.arange(sub_off[remap[u]], sub_off[remap[u]] + seg[u])
        rows = torch.from_numpy(tok[rows_sub]).cuda()
        got_o = t["o"][rows][:, heads].double().cpu().numpy()
        got_l = t["lse"][rows][:, heads].double().cpu().numpy()
        got_dq = t["dq"][rows][:, heads].double().cpu().numpy()
        eo, el, eq = _rel(got_o, O[rows_sub]), _rel(got_l, LSE[rows_sub]), _rel(got_dq, dQ[rows_sub])
        print(f"cfg{cfg} node {u} (len {seg[u]}, depth {sd[u]}): o={eo:.2e} lse={el:.2e} dq={eq:.2e}", flush=True)
        assert eo <= TOL and el <= TOL and eq <= TOL

    # (2) dK, dV inside a sampled subtree of affordable size
    sub_tok = {u: sum(int(seg[x]) for x in _subtree_nodes(parent, u)) for u in range(len(parent))} \
        if len(parent) <= 600 else None
    cands = [u for u in range(len(parent)) if parent[u] >= 0]
    if sub_tok is None:
        cands = [int(x) for x in rng.choice(cands, size=200, replace=False)]
        sub_tok = {u: sum(int(seg[x]) for x in _subtree_nodes(parent, u)) for u in cands}
    cands = [u for u in cands if 1 < len(_subtree_nodes(parent, u)) and sub_tok[u] <= 6000] or \
            [u for u in cands if sub_tok[u] <= 6000]
    if not cands:   # every subtree is larger (16 answers of 16K tokens): dK, dV are covered by the per-key test below
        return
    root = max(cands, key=lambda u: sub_tok[u])
    nodes = _subtree_nodes(parent, root)
    keep, remap, sub_off, tok, _, _, _, dK, dV = oracle_on(nodes)
    rows_sub = np.concatenate([np.arange(sub_off[remap[u]], sub_off[remap[u]] + seg[u]) for u in nodes])
    rows = torch.from_numpy(tok[rows_sub]).cuda()
    got_dk = t["dk"][rows][:, [grp]].double().cpu().numpy()
    got_dv = t["dv"][rows][:, [grp]].double().cpu().numpy()
    ek, ev = _rel(got_dk, dK[rows_sub]), _rel(got_dv, dV[rows_sub])
    print(f"cfg{cfg} subtree of node {root}: {len(nodes)} nodes, {len(rows_sub)} keys: dk={ek:.2e} dv={ev:.2e}", flush=True)
    assert ek <= TOL and ev <= TOL


@pytest.mark.parametrize("cfg,block,heads", [(2, 0, None), (3, 2048, None), (5, 0, (6, 3))])
def test_full_size_segment_calls_agree_with_the_one_launch_path(cfg, block, heads):
    """The paper's executor order at full size: the calls of dta_tree_plan issued
    one by one on zeroed accumulators, against the one-launch results checked
    above (both bf16 evaluations of the same sums).  The last case has three kv
    heads: its one-launch forward and dK/dV run as resident blocks drawing items
    from three queues whose home heads do not line up with the 8 XCDs, while the
    segment calls are small launches with one block per item."""
    parent, seg, (Hq, Hkv, d, scale), t = _run(cfg, heads)
    T = int(seg.sum())
    p = dta.AttnParams(Hq, Hkv, d, scale, dta.BF16)
    tree = dta.tree_build(parent, seg)
    plan = dta.tree_plan(tree, block)
    o = torch.zeros_like(t["q"])
    lse = torch.zeros((T, Hq), dtype=torch.float32, device="cuda")
    dq = torch.zeros_like(t["q"])
    dk = torch.zeros((T, Hkv, d), dtype=torch.float32, device="cuda")
    dv = torch.zeros_like(dk)
    ws = torch.empty(max(256, dta.workspace_bytes(tree, p, True)), dtype=torch.uint8, device="cuda")
    for op, node, t0, t1 in plan["calls"]:
        if op == dta.OP_BWD:
            dta.tree_attn_bwd_segment(tree, p, t0, t1, t["q"], t["k"], t["v"], o, lse, t["do"], dq, dk, dv, ws)
        else:
            dta.tree_attn_fwd_segment(tree, p, t0, t1, t["q"], t["k"], t["v"], o, lse)
    torch.cuda.synchronize()
    tree.destroy()
    rel = lambda a, b: float((a.double() - b.double()).abs().max() / b.double().abs().max())
    errs = dict(o=rel(o, t["o"]), lse=rel(lse, t["lse"]), dq=rel(dq, t["dq"]), dk=rel(dk, t["dk"]), dv=rel(dv, t["dv"]))
    print(f"cfg{cfg} block {block}: {len(plan['calls'])} calls " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()),
          flush=True)
    assert errs["lse"] <= 1e-5
    assert all(e <= TOL for e in errs.values())


def test_results_do_not_depend_on_which_block_draws_which_item():
    """Configuration 6 is large enough for the dK/dV launch to run as resident
    blocks that draw their work items from queues, so the assignment of items to
    blocks differs from run to run; the results must not (no atomics on data, the
    partial sums of split tiles are added in a fixed order)."""
    _, _, _, a = _run(6)
    _, _, _, b = _run(6)
    for n in ("o", "lse", "dq", "dk", "dv"):
        assert torch.equal(a[n], b[n]), n


def test_forward_without_workspace_gives_the_same_bits():
    """The forward's workspace is optional: without it the launch hands one item
    to each block, with it (configuration 2 has enough items) resident blocks
    draw the items from queues.  Same arithmetic per item, so the same bits."""
    parent, seg, meta = config_tree(2)
    h = config_heads(2)
    Hq, Hkv, d = h["n_q_heads"], h["n_kv_heads"], h["head_dim"]
    T = int(seg.sum())
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    mk = lambda heads: torch.randn((T, heads, d), generator=g, device="cuda").to(torch.bfloat16)
    q, k, v = mk(Hq), mk(Hkv), mk(Hkv)
    p = dta.AttnParams(Hq, Hkv, d, 1.0 / math.sqrt(d), dta.BF16)
    tree = dta.tree_build(parent, seg)
    assert dta.workspace_bytes(tree, p, False) > 0
    o1, l1 = dta.tree_attn_fwd(tree, p, q, k, v)                       # binding allocates the workspace
    o2, l2 = dta.tree_attn_fwd(tree, p, q, k, v, workspace=torch.empty(0, dtype=torch.uint8, device="cuda"))
    torch.cuda.synchronize()
    tree.destroy()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)


def test_config2_whole_tensors_for_one_kv_group():
    """Every row of O, LSE, dQ, dK, dV of one kv group (its four q heads) at the
    benchmark size, against the tree-direct fp64 oracle on the CPU."""
    parent, seg, (Hq, Hkv, d, scale), t = _run(2)
    G = Hq // Hkv
    grp = 5
    hs = slice(grp * G, (grp + 1) * G)
    host = lambda x: x.double().cpu().numpy()
    q, do = host(t["q"][:, hs]), host(t["do"][:, hs])
    k, v = host(t["k"][:, grp:grp + 1]), host(t["v"][:, grp:grp + 1])
    O, LSE = B.forward(parent, seg, q, k, v, scale)
    dQ, dK, dV = B.backward(parent, seg, q, k, v, do, scale)
    errs = dict(o=_rel(host(t["o"][:, hs]), O), lse=_rel(host(t["lse"][:, hs]), LSE),
                dq=_rel(host(t["dq"][:, hs]), dQ), dk=_rel(host(t["dk"][:, grp:grp + 1]), dK),
                dv=_rel(host(t["dv"][:, grp:grp + 1]), dV))
    print("cfg2 whole tensors, kv group 5: " + " ".join(f"{n}={e:.2e}" for n, e in errs.items()), flush=True)
    assert all(e <= TOL for e in errs.values()), errs


def _shared_prefix_keys(parent, seg, rng):
    """Packed key indices whose gradients collect many descendants: the first 168
    keys of the root with the largest subtree (two key tiles of the dK/dV
    schedule, the longest walks of the launch), 96 keys across the end of that
    root's segment and the start of its first child, 64 keys from the middle of
    the root, the first 40 keys of up to three other roots, 64 keys of a random
    interior node, 64 keys from the middle of the longest leaf and the last 40
    keys of the packed order."""
    off, T = L.node_offsets(parent, seg)
    _, kids = L.children_lists(parent)
    sub = {}
    for u in reversed(L.preorder(parent)):
        sub[u] = int(seg[u]) + sum(sub[c] for c in kids[u])
    roots = [u for u in range(len(parent)) if parent[u] < 0]
    big = max(roots, key=lambda u: sub[u])
    r0, r1 = int(off[big]), int(off[big]) + int(seg[big])
    keys = set(range(r0, min(r1, r0 + 168)))
    keys.update(range(max(r0, r1 - 48), min(T, r1 + 48)))
    mid = (r0 + r1) // 2
    keys.update(range(mid, min(r1, mid + 64)))
    for u in [x for x in roots if x != big][:3]:
        keys.update(range(int(off[u]), int(off[u]) + min(40, int(seg[u]))))
    interior = [u for u in range(len(parent)) if kids[u] and parent[u] >= 0]
    if interior:
        u = int(rng.choice(interior))
        keys.update(range(int(off[u]), int(off[u]) + min(64, int(seg[u]))))
    # keys whose queries are only the rest of their own segment: 64 from the middle of
    # the longest leaf (diagonal tiles and what follows them), and the last 40 keys of
    # the packed order (the ragged tail of the last key tile)
    leaves = [u for u in range(len(parent)) if not kids[u]]
    u = max(leaves, key=lambda x: int(seg[x]))
    mid = int(off[u]) + int(seg[u]) // 2
    keys.update(range(mid, min(int(off[u]) + int(seg[u]), mid + 64)))
    keys.update(range(max(0, T - 40), T))
    return np.array(sorted(keys), dtype=np.int64)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 8])
def test_full_size_shared_prefix_key_gradients(cfg):
    """dK and dV of shared-prefix keys, element by element, against the per-key
    oracle summed over EVERY query that sees them (for a root key: all tokens of
    its tree, for the four or eight q heads of the group).  The oracle's torch
    lines run in fp64 on the GPU here (its matrix products go to the vendor
    BLAS): at configuration 4 they are 10^13 floating-point operations; the same
    lines are tied to the CPU evaluation below and in the CPU pins."""
    parent, seg, (Hq, Hkv, d, scale), t = _run(cfg)
    G = Hq // Hkv
    rng = np.random.default_rng(40 + cfg)
    grp = int(rng.integers(0, Hkv))
    hs = slice(grp * G, (grp + 1) * G)
    keys = _shared_prefix_keys(parent, seg, rng)
    dK, dV, pairs = K.key_gradients(parent, seg, t["q"][:, hs], t["k"][:, grp], t["v"][:, grp], t["do"][:, hs],
                                    scale, keys, device="cuda", max_rows=2048)
    idx = torch.from_numpy(keys).cuda()
    got_dk = t["dk"][idx, grp].double().cpu().numpy()
    got_dv = t["dv"][idx, grp].double().cpu().numpy()
    ek, ev = _rel(got_dk, dK), _rel(got_dv, dV)
    print(f"cfg{cfg} kv group {grp}: {len(keys)} shared-prefix keys, oracle evaluated {pairs:.3e} (query row, "
          f"visible key) pairs per q head: dk={ek:.2e} dv={ev:.2e}", flush=True)
    assert ek <= TOL and ev <= TOL


def test_per_key_oracle_gives_the_same_values_on_the_cpu_and_on_the_gpu():
    """Ties the fp64 evaluation on the GPU used above to the CPU one (same lines,
    other BLAS), on a scaled-down sibling of configuration 3."""
    from workloads import make_inputs_numpy, scaled_config_tree
    parent, seg, _ = scaled_config_tree(3, 16)
    T = int(seg.sum())
    x = make_inputs_numpy(T, 4, 1, 64, seed=77, dtype="bf16")
    keys = _shared_prefix_keys(parent, seg, np.random.default_rng(3))
    a = K.key_gradients(parent, seg, x["q"], x["k"][:, 0], x["v"][:, 0], x["do"], 0.125, keys)
    b = K.key_gradients(parent, seg, x["q"], x["k"][:, 0], x["v"][:, 0], x["do"], 0.125, keys, device="cuda",
                        max_rows=100)
    assert a[2] == b[2]
    for u, w in zip(a[:2], b[:2]):
        assert np.abs(u - w).max() <= 1e-11 * max(1.0, np.abs(u).max())
