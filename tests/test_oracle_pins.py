"""Pins for the CPU oracle: every check here compares the oracle with something
other than itself (a library routine, a closed form, finite differences, a
token-by-token brute force, an algebraic invariant, counts printed by the paper
or derived by hand).  No GPU, no HIP library."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import dense_rollout as A
from oracle import tree_direct as B
from oracle import tree_layout as L
from workloads import chain_tree, config_tree, make_inputs_numpy, random_tree

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _inputs(T, Hq, Hkv, d, seed):
    x = make_inputs_numpy(T, Hq, Hkv, d, seed)
    return (x["q"].astype(np.float64), x["k"].astype(np.float64),
            x["v"].astype(np.float64), x["do"].astype(np.float64))


# ---------------------------------------------------------------- brute force
def _token_tables(parent, seg_len):
    """Pure-python per-token tables built by walking parents token by token:
    tok_node[t], and vis[t] = sorted list of visible key tokens (incl. t)."""
    parent = [int(p) for p in parent]
    seg_len = [int(s) for s in seg_len]
    n = len(parent)
    kids = {i: [] for i in range(n)}
    roots = []
    for i, p in enumerate(parent):
        (roots if p < 0 else kids[p]).append(i)
    first = {}
    t = 0

    def visit(u):
        nonlocal t
        first[u] = t
        t += seg_len[u]
        for c in sorted(kids[u]):
            visit(c)
    for r in sorted(roots):
        visit(r)
    vis = {}
    for u in range(n):
        above = []
        a = parent[u]
        while a >= 0:
            above = list(range(first[a], first[a] + seg_len[a])) + above
            a = parent[a]
        for j in range(seg_len[u]):
            vis[first[u] + j] = above + list(range(first[u], first[u] + j + 1))
    return first, vis, t


def _brute_forward(vis, q, k, v, scale, G):
    T, Hq, d = q.shape
    O = np.zeros((T, Hq, d))
    LSE = np.zeros((T, Hq))
    for t in range(T):
        for h in range(Hq):
            s = [scale * float(np.dot(q[t, h], k[j, h // G])) for j in vis[t]]
            tot = sum(math.exp(x) for x in s)
            LSE[t, h] = math.log(tot)
            for x, j in zip(s, vis[t]):
                O[t, h] += math.exp(x) / tot * v[j, h // G]
    return O, LSE


SMALL_TREES = [
    ([-1], [5]),
    ([-1, 0, 0], [3, 2, 4]),
    ([-1, 0, 1, 1, 0], [2, 3, 1, 2, 3]),
    ([2, 2, -1, 0, -1, 4], [2, 1, 3, 2, 2, 1]),       # ids out of DFS order, two roots
]


@pytest.mark.parametrize("parent,seg", SMALL_TREES)
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 2)])
def test_forward_matches_token_by_token_brute_force(parent, seg, Hq, Hkv):
    first, vis, T = _token_tables(parent, seg)
    q, k, v, _ = _inputs(T, Hq, Hkv, 8, seed=11)
    scale = 0.37
    Ob, Lb = _brute_forward(vis, q, k, v, scale, Hq // Hkv)
    Oa, La = A.forward(parent, seg, q, k, v, scale)
    Od, Ld = B.forward(parent, seg, q, k, v, scale)
    for O, Ls in ((Oa, La), (Od, Ld)):
        assert np.abs(O - Ob).max() < 1e-12
        assert np.abs(Ls - Lb).max() < 1e-12
    # the oracle's own preorder agrees with the brute-force visit order
    off, T2 = L.node_offsets(parent, seg)
    assert T2 == T and all(int(off[u]) == first[u] for u in range(len(parent)))


def test_all_tiny_trees_exhaustively():
    """Every forest with <= 4 nodes and seg_len in {1,2}: A == B == brute force."""
    import itertools
    rng = np.random.default_rng(5)
    count = 0
    for n in range(1, 5):
        for par in itertools.product(*[range(-1, i) for i in range(n)]):
            for seg in itertools.product([1, 2], repeat=n):
                if rng.random() > 0.25 and n == 4:
                    continue
                _, vis, T = _token_tables(par, seg)
                q, k, v, _ = _inputs(T, 2, 1, 4, seed=count)
                Ob, Lb = _brute_forward(vis, q, k, v, 0.5, 2)
                Oa, La = A.forward(par, seg, q, k, v, 0.5)
                Od, Ld = B.forward(par, seg, q, k, v, 0.5)
                assert np.abs(Oa - Ob).max() < 1e-12 and np.abs(Od - Ob).max() < 1e-12
                assert np.abs(La - Lb).max() < 1e-12 and np.abs(Ld - Lb).max() < 1e-12
                count += 1
    assert count > 100


# ------------------------------------------------------------ library routine
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (8, 2)])
def test_chain_is_textbook_causal_attention_torch_sdpa(Hq, Hkv):
    """A single-chain tree reduces to ordinary causal attention; torch's
    scaled_dot_product_attention and its autograd are the outside reference."""
    parent, seg = chain_tree([7, 1, 12, 5])
    T, d = int(seg.sum()), 16
    q, k, v, do = _inputs(T, Hq, Hkv, d, seed=3)
    scale = 1.0 / math.sqrt(d)
    G = Hq // Hkv
    tq = torch.tensor(q.transpose(1, 0, 2), requires_grad=True)     # [H,T,d]
    tk = torch.tensor(k.transpose(1, 0, 2), requires_grad=True)
    tv = torch.tensor(v.transpose(1, 0, 2), requires_grad=True)
    out = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(G, dim=0)[None], tv.repeat_interleave(G, dim=0)[None],
        is_causal=True, scale=scale)[0]
    out.backward(torch.tensor(do.transpose(1, 0, 2)))
    ref = {"o": out.detach().numpy().transpose(1, 0, 2),
           "dq": tq.grad.numpy().transpose(1, 0, 2),
           "dk": tk.grad.numpy().transpose(1, 0, 2),
           "dv": tv.grad.numpy().transpose(1, 0, 2)}
    for mod in (A, B):
        O, LSE = mod.forward(parent, seg, q, k, v, scale)
        dQ, dK, dV = mod.backward(parent, seg, q, k, v, do, scale)
        assert np.abs(O - ref["o"]).max() < 1e-12
        assert np.abs(dQ - ref["dq"]).max() < 1e-11
        assert np.abs(dK - ref["dk"]).max() < 1e-11
        assert np.abs(dV - ref["dv"]).max() < 1e-11
        # LSE against torch.logsumexp of the masked scores
        s = scale * torch.einsum("htd,hsd->hts", tq.detach(), tk.detach().repeat_interleave(G, dim=0))
        s = s.masked_fill(torch.triu(torch.ones(T, T, dtype=torch.bool), 1), -float("inf"))
        assert np.abs(LSE - torch.logsumexp(s, -1).numpy().T).max() < 1e-12


def test_tree_rows_equal_sdpa_on_each_expanded_rollout():
    """O at every position a token occupies equals dense attention on that
    rollout, with torch's routine (not the oracle's) doing the dense part."""
    rng = np.random.default_rng(21)
    parent, seg = random_tree(rng, 7, 5)
    T = int(seg.sum())
    q, k, v, _ = _inputs(T, 2, 1, 8, seed=4)
    O, _ = B.forward(parent, seg, q, k, v, 0.3)
    for idx in L.rollout_token_paths(parent, seg):
        tq = torch.tensor(q[idx].transpose(1, 0, 2))[None]
        tk = torch.tensor(k[idx].transpose(1, 0, 2)).repeat_interleave(2, dim=0)[None]
        tv = torch.tensor(v[idx].transpose(1, 0, 2)).repeat_interleave(2, dim=0)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.3)[0]
        assert np.abs(O[idx] - ref.numpy().transpose(1, 0, 2)).max() < 1e-12


# --------------------------------------------------------------- closed forms
@pytest.mark.parametrize("mod", [A, B])
def test_zero_keys_closed_form(mod):
    """K = 0: every visible key gets the same weight, so LSE = ln(pos+1) and O is
    the mean of V over the ancestor path; pins key-set size and membership."""
    rng = np.random.default_rng(8)
    parent, seg = random_tree(rng, 9, 6, n_roots=2)
    _, vis, T = _token_tables(parent, seg)
    q, _, v, _ = _inputs(T, 2, 2, 8, seed=9)
    O, LSE = mod.forward(parent, seg, q, np.zeros((T, 2, 8)), v, 1.7)
    for t in range(T):
        assert abs(LSE[t, 0] - math.log(len(vis[t]))) < 1e-13
        assert np.abs(O[t] - v[vis[t]].mean(axis=0)).max() < 1e-13


@pytest.mark.parametrize("mod", [A, B])
def test_first_token_and_constant_values(mod):
    parent, seg, _ = config_tree(1)
    seg = np.maximum(1, seg // 8)
    T = int(seg.sum())
    q, k, v, _ = _inputs(T, 4, 2, 8, seed=10)
    O, LSE = mod.forward(parent, seg, q, k, v, 0.25)
    # position 0 sees only itself
    assert np.abs(O[0] - v[0].repeat(2, axis=0)).max() < 1e-14
    assert np.abs(LSE[0] - 0.25 * np.einsum("hd,hd->h", q[0], k[0].repeat(2, axis=0))).max() < 1e-13
    # V == c  =>  O == c
    O2, _ = mod.forward(parent, seg, q, k, np.full_like(v, 3.5), 0.25)
    assert np.abs(O2 - 3.5).max() < 1e-13


# --------------------------------------------------------- finite differences
def _objective(parent, seg, q, k, v, do, scale):
    O, _ = B.forward(parent, seg, q, k, v, scale)
    return float((O * do).sum())


@pytest.mark.parametrize("mod", [A, B])
def test_gradients_against_central_finite_differences(mod):
    rng = np.random.default_rng(33)
    parent, seg = random_tree(rng, 6, 4)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 4, 2, 6, seed=12)
    scale = 0.41
    dQ, dK, dV = mod.backward(parent, seg, q, k, v, do, scale)
    eps = 1e-5
    for name, arr, grad in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
        for _ in range(25):
            i = tuple(int(rng.integers(0, s)) for s in arr.shape)
            old = arr[i]
            arr[i] = old + eps
            fp = _objective(parent, seg, q, k, v, do, scale)
            arr[i] = old - eps
            fm = _objective(parent, seg, q, k, v, do, scale)
            arr[i] = old
            fd = (fp - fm) / (2 * eps)
            assert abs(fd - grad[i]) < 1e-7 * max(1.0, abs(fd)), (name, i, fd, grad[i])


def test_forward_objective_used_for_fd_is_brute_force_checked():
    """The finite-difference objective uses B.forward, itself pinned above; make
    the dependency explicit on the same tree shape."""
    rng = np.random.default_rng(33)
    parent, seg = random_tree(rng, 6, 4)
    _, vis, T = _token_tables(parent, seg)
    q, k, v, _ = _inputs(T, 4, 2, 6, seed=12)
    Ob, _ = _brute_forward(vis, q, k, v, 0.41, 2)
    assert np.abs(B.forward(parent, seg, q, k, v, 0.41)[0] - Ob).max() < 1e-12


# ----------------------------------------------------------------- invariants
def test_A_equals_B_on_config1_and_random_trees():
    parent, seg, _ = config_tree(1)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 4, 4, 16, seed=2001)
    Oa, La, spread = A.forward(parent, seg, q, k, v, 0.25, return_spread=True)
    Ob, Lb = B.forward(parent, seg, q, k, v, 0.25)
    assert spread < 1e-12
    assert np.abs(Oa - Ob).max() < 1e-12 and np.abs(La - Lb).max() < 1e-12
    for a, b in zip(A.backward(parent, seg, q, k, v, do, 0.25), B.backward(parent, seg, q, k, v, do, 0.25)):
        assert np.abs(a - b).max() < 1e-11
    rng = np.random.default_rng(77)
    for trial in range(6):
        parent, seg = random_tree(rng, int(rng.integers(1, 12)), 7, n_roots=int(rng.integers(1, 3)))
        T = int(seg.sum())
        q, k, v, do = _inputs(T, 4, 2, 8, seed=100 + trial)
        for a, b in zip(A.backward(parent, seg, q, k, v, do, 0.3), B.backward(parent, seg, q, k, v, do, 0.3)):
            assert np.abs(a - b).max() < 1e-11


def test_rollout_split_weights_do_not_matter():
    """Summation over rollouts (equation 1): any split of a shared token's dO
    over the rollouts containing it gives the same tree gradients."""
    parent, seg, _ = config_tree(1)
    seg = np.maximum(1, seg // 4)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 4, 2, 8, seed=13)
    base = A.backward(parent, seg, q, k, v, do, 0.35)
    rng = np.random.default_rng(14)
    paths = L.rollout_token_paths(parent, seg)
    raw = [rng.gamma(1.0, size=len(p)) for p in paths]
    tot = np.zeros(T)
    for p, r in zip(paths, raw):
        tot[p] += r
    weights = [r / tot[p] for p, r in zip(paths, raw)]
    for a, b in zip(base, A.backward(parent, seg, q, k, v, do, 0.35, weights=weights)):
        assert np.abs(a - b).max() < 1e-12


@pytest.mark.parametrize("mod", [A, B])
def test_softmax_and_gradient_identities(mod):
    rng = np.random.default_rng(15)
    parent, seg = random_tree(rng, 8, 6)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 4, 2, 8, seed=16)
    dQ, dK, dV = mod.backward(parent, seg, q, k, v, do, 0.3)
    # sum_k dV_k = sum_t dO_t per kv head (rows of P sum to one), q heads of a group added
    assert np.abs(dV.sum(axis=0) - do.reshape(T, 2, 2, 8).sum(axis=(0, 2))).max() < 1e-11
    # scores are bilinear in (q, k): sum_t q_t.dQ_t and sum_k k_k.dK_k both equal
    # sum_{t,k} dS_tk * s_tk, per kv group
    lhs = np.einsum("thd,thd->h", q, dQ).reshape(2, 2).sum(axis=1)
    rhs = np.einsum("tgd,tgd->g", k, dK)
    assert np.abs(lhs - rhs).max() < 1e-10
    # linearity in dO
    do2 = rng.standard_normal(do.shape)
    g1 = mod.backward(parent, seg, q, k, v, do2, 0.3)
    g12 = mod.backward(parent, seg, q, k, v, do + do2, 0.3)
    for a, b, c in zip((dQ, dK, dV), g1, g12):
        assert np.abs(a + b - c).max() < 1e-11


def test_node_split_and_child_order_invariance():
    """Splitting a segment into a unary chain, or renumbering children (another
    valid DFS order, section 4), changes no per-token value."""
    parent = np.array([-1, 0, 0, 1, 1], dtype=np.int32)
    seg = np.array([6, 4, 5, 3, 2], dtype=np.int32)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 2, 1, 8, seed=17)
    ref = B.forward(parent, seg, q, k, v, 0.3) + B.backward(parent, seg, q, k, v, do, 0.3)
    # split node 0 (6 tokens) into 0:(2) -> 5:(4); children of 0 move under 5.
    # preorder (ascending ids) would visit 5 after 1,2, so renumber to keep packing:
    parent2 = np.array([-1, 0, 1, 1, 2, 2], dtype=np.int32)      # 0:2tok,1:4tok,(old1)->2,(old2)->3,(old3)->4,(old4)->5
    seg2 = np.array([2, 4, 4, 5, 3, 2], dtype=np.int32)
    # packed order of old tree: 0,1,3,4,2 ; new tree preorder: 0,1,2,4,5,3 -> same token order
    out = B.forward(parent2, seg2, q, k, v, 0.3) + B.backward(parent2, seg2, q, k, v, do, 0.3)
    for a, b in zip(ref, out):
        assert np.abs(a - b).max() < 1e-12
    # child order: swap ids of the two children of the root; tokens move, values follow
    parent3 = np.array([-1, 0, 0, 2, 2], dtype=np.int32)         # old node 1 is now id 2, old 2 is id 1
    seg3 = np.array([6, 5, 4, 3, 2], dtype=np.int32)
    # old packed order of nodes: 0,1,3,4,2 ; new packed order: 0,(old2),(old1),(old3),(old4)
    off_old, _ = L.node_offsets(parent, seg)
    perm = np.concatenate([np.arange(off_old[u], off_old[u] + seg[u]) for u in (0, 2, 1, 3, 4)])
    out3 = B.forward(parent3, seg3, q[perm], k[perm], v[perm], 0.3) + \
        B.backward(parent3, seg3, q[perm], k[perm], v[perm], do[perm], 0.3)
    for a, b in zip(ref, out3):
        assert np.abs(a[perm] - b).max() < 1e-12


def test_duplicate_leaf_doubles_ancestor_gradient_contribution():
    parent = np.array([-1, 0], dtype=np.int32)
    seg = np.array([5, 3], dtype=np.int32)
    q, k, v, do = _inputs(8, 2, 1, 8, seed=18)
    do[:5] = 0.0                                   # only the leaf carries loss
    _, dK1, dV1 = B.backward(parent, seg, q, k, v, do, 0.3)
    parent2 = np.array([-1, 0, 0], dtype=np.int32)
    seg2 = np.array([5, 3, 3], dtype=np.int32)
    dup = lambda x: np.concatenate([x, x[5:]])
    _, dK2, dV2 = B.backward(parent2, seg2, dup(q), dup(k), dup(v), dup(do), 0.3)
    assert np.abs(dK2[:5] - 2 * dK1[:5]).max() < 1e-12
    assert np.abs(dV2[:5] - 2 * dV1[:5]).max() < 1e-12
    assert np.abs(dK2[5:8] - dK1[5:]).max() < 1e-12 and np.abs(dK2[8:] - dK1[5:]).max() < 1e-12


def test_sibling_independence():
    parent = np.array([-1, 0, 0], dtype=np.int32)
    seg = np.array([4, 3, 5], dtype=np.int32)
    q, k, v, _ = _inputs(12, 2, 2, 8, seed=19)
    O1, L1 = B.forward(parent, seg, q, k, v, 0.3)
    k2, v2 = k.copy(), v.copy()
    k2[4:7] += 1.0
    v2[4:7] -= 2.0
    O2, L2 = B.forward(parent, seg, q, k2, v2, 0.3)
    assert np.array_equal(O1[7:], O2[7:]) and np.array_equal(L1[7:], L2[7:])
    assert np.array_equal(O1[:4], O2[:4])
    assert not np.allclose(O1[4:7], O2[4:7])


# ------------------------------------------------------------------ statistics
def test_config1_counts_golden():
    want = {}
    for line in open(os.path.join(GOLDEN, "config1_counts.txt")):
        if line.strip() and not line.startswith("#"):
            name, val = line.split()
            want[name] = int(val)
    parent, seg, _ = config_tree(1)
    st = L.tree_stats(parent, seg)
    for name, val in want.items():
        assert st[name] == val, name
    # unique pairs counted token by token
    _, vis, T = _token_tables(parent, seg)
    assert sum(len(vis[t]) for t in range(T)) == want["unique_pairs"]


def test_compression_and_sharing_rate_golden():
    """S = 1 - 1/C with the pairs printed in the caption of figure 1."""
    for line in open(os.path.join(GOLDEN, "figure1_compression.txt")):
        if line.strip() and not line.startswith("#"):
            C, S = map(float, line.split())
            assert abs((1.0 - 1.0 / C) * 100.0 - S) < 0.06
    # a forest of n identical-prefix rollouts: C known in closed form
    parent, seg = np.array([-1, 0, 0, 0]), np.array([10, 5, 5, 5])
    st = L.tree_stats(parent, seg)
    assert st["C_leaf"] == pytest.approx(45 / 25)
    assert st["C_full"] == pytest.approx(55 / 25)
    assert st["C_attn_leaf"] <= st["C_leaf"]


def test_tree_token_identity_over_dfs_leaf_order():
    """Unique tree tokens = |pi_1| + sum_i (|pi_i| - LCP(pi_{i-1}, pi_i)) over a
    DFS leaf order (cost bookkeeping of the partitioning algorithm, appendix)."""
    rng = np.random.default_rng(23)
    for _ in range(10):
        parent, seg = random_tree(rng, int(rng.integers(1, 15)), 6, shuffle_ids=False)
        paths = L.rollout_token_paths(parent, seg)       # ascending leaf id; ids are a preorder here? not always
        # sort rollouts lexicographically by their token-index vectors: a valid DFS order
        paths = sorted(paths, key=lambda p: tuple(p.tolist()))
        total = len(paths[0])
        for a, b in zip(paths[:-1], paths[1:]):
            lcp = 0
            while lcp < min(len(a), len(b)) and a[lcp] == b[lcp]:
                lcp += 1
            total += len(b) - lcp
        assert total == int(seg.sum())


# ------------------------------------------- push / pop executor (oracle C)
from oracle import dfs_executor as X


def test_executor_equals_rollout_expansion_and_counts_its_steps():
    """The stack-based push/pop traversal (a third formulation) must give the
    tensors of the rollout-expansion oracle; every node is forwarded once and
    popped once, a child's FWD follows its parent's and its BWD precedes it,
    and the stack never holds more than the longest root-to-leaf path."""
    rng = np.random.default_rng(71)
    for n_nodes, max_len, n_roots in ((1, 5, 1), (9, 6, 1), (14, 5, 3)):
        parent, seg = random_tree(rng, n_nodes, max_len, n_roots=n_roots)
        T = int(seg.sum())
        q, k, v, do = _inputs(T, 4, 2, 8, seed=40 + n_nodes)
        scale = 0.3
        r = X.vanilla_dta(parent, seg, q, k, v, do, scale)
        O, LSE = A.forward(parent, seg, q, k, v, scale)
        dQ, dK, dV = A.backward(parent, seg, q, k, v, do, scale)
        for name, ref in (("O", O), ("LSE", LSE), ("dQ", dQ), ("dK", dK), ("dV", dV)):
            assert np.abs(r[name] - ref).max() < 1e-11, name
        fwd = [t[1] for t in r["trace"] if t[0] == "FWD"]
        bwd = [t[1] for t in r["trace"] if t[0] == "BWD"]
        assert sorted(fwd) == sorted(bwd) == list(range(n_nodes))
        assert fwd == L.preorder(parent)                       # pushes happen in DFS preorder
        pos_f = {u: i for i, t in enumerate(r["trace"]) for u in [t[1]] if t[0] == "FWD"}
        pos_b = {u: i for i, t in enumerate(r["trace"]) for u in [t[1]] if t[0] == "BWD"}
        for u in range(n_nodes):
            assert pos_f[u] < pos_b[u]
            if parent[u] >= 0:
                assert pos_f[int(parent[u])] < pos_f[u] and pos_b[u] < pos_b[int(parent[u])]
        assert r["peak_stack"] == max(len(p) for p in L.rollout_token_paths(parent, seg))


def test_segment_primitives_on_a_chain_are_rows_of_torch_sdpa():
    """FWD of the last segment of a chain = the last rows of ordinary causal
    attention over the whole chain; BWD with dO on those rows only = torch's
    autograd of the same (outside library routine)."""
    L_, m, d = 23, 7, 16
    rng = np.random.default_rng(5)
    q = rng.standard_normal((L_, d)); k = rng.standard_normal((L_, d)); v = rng.standard_normal((L_, d))
    do = rng.standard_normal((m, d))
    scale = 1.0 / math.sqrt(d)
    o, lse, p = X.fwd_segment(q[L_ - m:], k, v, scale)
    tq = torch.tensor(q, requires_grad=True); tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    out = torch.nn.functional.scaled_dot_product_attention(tq[None, None], tk[None, None], tv[None, None],
                                                           is_causal=True, scale=scale)[0, 0]
    assert np.abs(o - out.detach().numpy()[L_ - m:]).max() < 1e-12
    s = scale * tq.detach() @ tk.detach().T
    s = s.masked_fill(torch.triu(torch.ones(L_, L_, dtype=torch.bool), 1), -float("inf"))
    assert np.abs(lse - torch.logsumexp(s, -1).numpy()[L_ - m:]).max() < 1e-12
    full_do = torch.zeros(L_, d, dtype=torch.float64)
    full_do[L_ - m:] = torch.tensor(do)
    out.backward(full_do)
    dq, dk, dv = X.bwd_segment(q[L_ - m:], k, v, o, p, do, scale)
    assert np.abs(dq - tq.grad.numpy()[L_ - m:]).max() < 1e-11
    assert np.abs(tq.grad.numpy()[:L_ - m]).max() == 0.0
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-11
    assert np.abs(dv - tv.grad.numpy()).max() < 1e-11


def test_segment_backward_against_central_finite_differences():
    rng = np.random.default_rng(8)
    L_, m, d, scale = 9, 4, 5, 0.37
    q = rng.standard_normal((m, d)); k = rng.standard_normal((L_, d)); v = rng.standard_normal((L_, d))
    do = rng.standard_normal((m, d))
    f = lambda: float((X.fwd_segment(q, k, v, scale)[0] * do).sum())
    o, _, p = X.fwd_segment(q, k, v, scale)
    dq, dk, dv = X.bwd_segment(q, k, v, o, p, do, scale)
    eps = 1e-5
    for arr, grad in ((q, dq), (k, dk), (v, dv)):
        for i in np.ndindex(arr.shape):
            old = arr[i]
            arr[i] = old + eps; fp = f()
            arr[i] = old - eps; fm = f()
            arr[i] = old
            assert abs((fp - fm) / (2 * eps) - grad[i]) < 1e-8


def test_chunked_pops_change_nothing_and_run_last_chunk_first():
    """Pop_ByChunk: boundaries evenly spaced and at most `block` apart, chunks
    run from the last to the first, each with a recomputing FWD; the tensors do
    not depend on the block size."""
    assert X.chunk_boundaries(10, 30, 0) == [10, 30]
    assert X.chunk_boundaries(10, 30, 20) == [10, 30]
    for lo, hi, block in ((0, 17, 4), (5, 6, 1), (3, 103, 7), (0, 64, 16)):
        b = X.chunk_boundaries(lo, hi, block)
        gaps = np.diff(b)
        assert b[0] == lo and b[-1] == hi and gaps.min() >= 1 and gaps.max() <= block
        assert len(b) - 1 == -(-(hi - lo) // block) and gaps.max() - gaps.min() <= 1
    rng = np.random.default_rng(72)
    parent, seg = random_tree(rng, 8, 11)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 4, 2, 8, seed=77)
    base = X.vanilla_dta(parent, seg, q, k, v, do, 0.25)
    for block in (1, 3, 4):
        r = X.vanilla_dta(parent, seg, q, k, v, do, 0.25, chunk_block=block)
        for name in ("O", "LSE", "dQ", "dK", "dV"):
            assert np.abs(r[name] - base[name]).max() < 1e-12, (block, name)
        per_node = {}
        for tag, node, t0, t1 in r["trace"]:
            if tag == "BWD":
                per_node.setdefault(node, []).append((t0, t1))
        for node, chunks in per_node.items():
            assert all(a[0] == b[1] for a, b in zip(chunks, chunks[1:]))     # right to left, contiguous
            assert max(t1 - t0 for t0, t1 in chunks) <= block


# --------------------------- rollouts -> prefix tree, partitioning (oracle D)
import itertools

from oracle import rollout_tree as R


def _random_rollouts(rng, n, alphabet, max_len, p_extend=0.5):
    """Sequences that share prefixes: each new one copies a random prefix of an
    earlier one (sometimes all of it: containment / duplicates) and appends."""
    seqs = [list(rng.integers(0, alphabet, size=int(rng.integers(1, max_len + 1))))]
    for _ in range(n - 1):
        src = seqs[int(rng.integers(0, len(seqs)))]
        keep = int(rng.integers(0, len(src) + 1))
        extra = int(rng.integers(0 if keep else 1, max_len + 1)) if rng.random() < p_extend or keep == 0 else 0
        s = list(src[:keep]) + list(rng.integers(0, alphabet, size=extra))
        seqs.append(s if s else [int(rng.integers(0, alphabet))])
    return [[int(t) for t in s] for s in seqs]


def _paths(tree):
    """Token sequence of the root-to-node path of every node."""
    off = np.concatenate([[0], np.cumsum(tree["seg_len"])])
    out = []
    for u, p in enumerate(tree["parent"]):
        own = tree["tokens"][off[u]:off[u + 1]]
        out.append((out[p] if p >= 0 else []) + list(own))
    return out


def test_prefix_tree_round_trip_and_structure():
    rng = np.random.default_rng(91)
    for trial in range(60):
        seqs = _random_rollouts(rng, int(rng.integers(1, 12)), int(rng.integers(1, 4)), 7)
        tree = R.build_tree(seqs)
        paths = _paths(tree)
        for s, u in zip(seqs, tree["seq_node"]):
            assert paths[u] == s                                   # every rollout is a root-to-node path
        parent, seg_len = tree["parent"], tree["seg_len"]
        kids = [[] for _ in parent]
        for u, p in enumerate(parent):
            assert p < u                                           # preorder numbering
            if p >= 0:
                kids[p].append(u)
        ends = set(tree["seq_node"])
        off = np.concatenate([[0], np.cumsum(seg_len)])
        for u in range(len(parent)):
            assert seg_len[u] >= 1
            assert len(kids[u]) != 1 or u in ends                  # maximal merging: no pointless unary node
            assert len(kids[u]) > 0 or u in ends                   # every leaf ends a rollout
            firsts = [tree["tokens"][off[c]] for c in kids[u]]
            assert firsts == sorted(set(firsts))                   # children: distinct first tokens, ascending
        roots = [tree["tokens"][off[u]] for u, p in enumerate(parent) if p < 0]
        assert roots == sorted(set(roots))
        # packed order is the library's DFS preorder (children in ascending id): identity layout
        assert L.preorder(parent) == list(range(len(parent)))
        # tree tokens = appendix formula |pi_1| + sum(|pi_i| - LCP(pi_{i-1}, pi_i)) over the lexicographic order
        pi = [seqs[i] for i in tree["order"]]
        assert pi == sorted(pi)
        T = len(pi[0]) + sum(len(pi[i]) - R.lcp(pi[i - 1], pi[i]) for i in range(1, len(pi)))
        assert T == len(tree["tokens"]) == sum(seg_len)


def test_prefix_tree_worked_example():
    """Hand-checked: 'abc', 'abd', 'ab', 'x', 'abd' -> a b | c, d ; x."""
    seqs = [[1, 2, 3], [1, 2, 4], [1, 2], [9], [1, 2, 4]]
    t = R.build_tree(seqs)
    assert t["parent"] == [-1, 0, 0, -1] and t["seg_len"] == [2, 1, 1, 1]
    assert t["tokens"] == [1, 2, 3, 4, 9] and t["seq_node"] == [1, 2, 0, 3, 2]
    assert t["order"] == [2, 0, 1, 4, 3]
    assert R.lcp([1, 2, 3], [1, 2, 4]) == 2 and R.lcp([1], [1, 2]) == 1 and R.lcp([], [1]) == 0


def test_partition_is_optimal_contiguous_and_within_the_duplication_bound():
    rng = np.random.default_rng(92)
    for trial in range(80):
        seqs = _random_rollouts(rng, int(rng.integers(1, 9)), 3, 6)
        N = len(seqs)
        pi = sorted(seqs)
        T = R.group_cost(pi, 0, N - 1)
        for K in range(1, N + 1):
            order, cuts = R.partition(seqs, K)
            assert [seqs[i] for i in order] == pi
            assert len(cuts) == K and cuts[0][0] == 0 and cuts[-1][1] == N - 1
            assert all(a <= b for a, b in cuts) and all(c[1] + 1 == d[0] for c, d in zip(cuts, cuts[1:]))
            costs = [R.group_cost(pi, a, b) for a, b in cuts]
            # brute force: best achievable largest group cost over ALL splits into at most K contiguous groups
            best = min(max(R.group_cost(pi, a, b) for a, b in
                           zip((0,) + tuple(c + 1 for c in cs), cs + (N - 1,)))
                       for k in range(1, K + 1) for cs in itertools.combinations(range(N - 1), k - 1))
            assert max(costs) == best
            # section 4: at most (K-1) * longest sequence tokens beyond the single tree
            assert T <= sum(costs) <= T + (K - 1) * max(len(s) for s in seqs)


# ------------------------- backward DFS order and leaf-order schedule (oracle E)
from oracle import dfs_schedule as S


def _run_schedule(parent, seg, q, k, v, do, scale, ops):
    """Executes the operation list with the one-segment primitives."""
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    off, _ = L.node_offsets(parent, seg)
    path_tok = lambda leaf: np.concatenate([np.arange(off[u], off[u] + int(seg[u])) for u in L.node_path(parent, leaf)])
    O = np.full((T, Hq, d), np.nan); LSE = np.full((T, Hq), np.nan)
    dQ = np.full((T, Hq, d), np.nan); dK = np.zeros((T, Hkv, d)); dV = np.zeros((T, Hkv, d))
    popped = np.zeros(T, dtype=int)
    for tag, leaf, lo, hi in ops:
        idx = path_tok(leaf)
        own, ctx = idx[lo:hi], idx[:hi]
        for h in range(Hq):
            g = h // G
            o, lse, p = X.fwd_segment(q[own, h], k[ctx, g], v[ctx, g], scale)
            if tag != "BWD":
                O[own, h], LSE[own, h] = o, lse
            else:
                assert np.array_equal(O[own, h], o)               # forwarded before it is popped
                dq, dk, dv = X.bwd_segment(q[own, h], k[ctx, g], v[ctx, g], o, p, do[own, h], scale)
                dQ[own, h] = dq
                dK[ctx, g] += dk
                dV[ctx, g] += dv
        if tag == "BWD":
            popped[own] += 1
    assert (popped == 1).all()
    return O, LSE, dQ, dK, dV


def test_backward_dfs_order_and_schedule_worked_example():
    """Root R (4 tokens) with children: leaf a (2), internal M (3) with leaves
    b (5) and c (1), leaf e (6).  Depths: a 6, e 10, b 12, c 8.  At M the
    children order is c (tail 8), b (tail 12), so tail(M) = 8; at R: leaves
    first by tail: a (6), e (10), then M.  DFS leaf order a, e, c, b; pi is its
    reverse b, c, e, a."""
    parent = [-1, 0, 0, 2, 2, 0]
    seg = [4, 2, 3, 5, 1, 6]       # ids: 0 R, 1 a, 2 M, 3 b, 4 c, 5 e
    assert S.backward_dfs_order(parent, seg) == [3, 4, 5, 1]
    ops, pi = S.schedule(parent, seg, block=0)
    assert pi == [3, 4, 5, 1]
    assert ops == [
        ("FWD", 3, 0, 12), ("NOGRAD", 3, 0, 7),                 # next leaf c shares R+M = 7 tokens
        ("REFWD", 3, 7, 12), ("BWD", 3, 7, 12),
        ("FWD", 4, 7, 8),
        ("REFWD", 4, 4, 8), ("BWD", 4, 4, 8),                   # c and M leave together: e shares only R
        ("FWD", 5, 4, 10),
        ("REFWD", 5, 4, 10), ("BWD", 5, 4, 10),
        ("FWD", 1, 4, 6),
        ("REFWD", 1, 0, 6), ("BWD", 1, 0, 6),
    ]
    ops4, _ = S.schedule(parent, seg, block=4)
    # first leaf: 12 tokens to pop down to 7 -> p_pop = 5 >= 4: two chunks, anchor at 12 - 3 = 9
    assert ops4[:6] == [("FWD", 3, 0, 12), ("NOGRAD", 3, 0, 9), ("REFWD", 3, 9, 12), ("BWD", 3, 9, 12),
                        ("REFWD", 3, 7, 9), ("BWD", 3, 7, 9)]
    assert S.path_ranges(parent, seg, 3, 2, 9) == [(2, 4), (6, 9), (9, 11)]   # packed: R 0-4, a 4-6, M 6-9, b 9-14


@pytest.mark.parametrize("block", [0, 1, 5, 64])
def test_schedule_discipline_counts_and_invariance(block):
    rng = np.random.default_rng(300 + block)
    for trial in range(6):
        parent, seg = random_tree(rng, int(rng.integers(1, 14)), 9, n_roots=int(rng.integers(1, 3)))
        ops, pi = S.schedule(parent, seg, block)
        leaves = L.leaves(parent)
        assert sorted(pi) == sorted(leaves)
        # stack discipline in depth coordinates
        depth, cur = 0, None
        for tag, leaf, lo, hi in ops:
            assert lo < hi
            if tag == "FWD":
                assert lo == depth and (cur is None or S.common_prefix_tokens(parent, seg, cur, leaf) >= lo)
                depth, cur = hi, leaf
            elif tag == "BWD":
                assert hi == depth and leaf == cur and (block <= 0 or hi - lo <= block)
                depth = lo
            else:
                assert leaf == cur and hi <= depth
        assert depth == 0
        # the paper's counts: one regular FWD per leaf, at most one FWD-NoGrad per leaf
        assert sum(t[0] == "FWD" for t in ops) == len(leaves)
        assert sum(t[0] == "NOGRAD" for t in ops) <= len(leaves)
        assert [t for t in ops if t[0] == "REFWD"] == [("REFWD",) + t[1:] for t in ops if t[0] == "BWD"]
        # invariance: same tensors as the rollout-expansion oracle
        T = int(np.sum(seg))
        q, k, v, do = _inputs(T, 4, 2, 6, seed=trial)
        got = _run_schedule(parent, seg, q, k, v, do, 0.4, ops)
        ref = A.forward(parent, seg, q, k, v, 0.4) + A.backward(parent, seg, q, k, v, do, 0.4)
        for x, y in zip(got, ref):
            assert np.abs(x - y).max() < 1e-11


def test_leaf_first_order_needs_no_anchor_on_a_star():
    """Siblings that are all leaves under one prompt (a GRPO group): every leaf
    after the first shares exactly the prompt with its neighbours, so with an
    infinite block no FWD-NoGrad is needed after the first leaf's."""
    parent = [-1] + [0] * 6
    seg = [10, 3, 7, 2, 9, 4, 5]
    ops, pi = S.schedule(parent, seg, 0)
    assert [seg[u] for u in pi] == sorted(seg[1:], reverse=True)       # reversed smaller-tail-first order
    assert [t for t in ops if t[0] == "NOGRAD"] == [("NOGRAD", pi[0], 0, 10)]


# ------------------------------------------- gradients of chosen keys (oracle K)
def test_key_gradients_equal_rollout_expansion_rows():
    """The per-key oracle (pop step written out key by key) returns exactly the
    rows of the dense per-rollout oracle's dK/dV, for keys of roots, interior
    nodes and leaves, in any order, with the rows of a node held in memory all
    at once or a few at a time."""
    from oracle import key_gradient as K
    rng = np.random.default_rng(91)
    cases = [config_tree(1)[:2]] + [random_tree(rng, int(rng.integers(2, 12)), 9, n_roots=int(rng.integers(1, 3)))
                                    for _ in range(5)]
    for ci, (parent, seg) in enumerate(cases):
        if ci == 0:
            seg = np.maximum(1, seg // 4)
        T = int(seg.sum())
        q, k, v, do = _inputs(T, 4, 2, 8, seed=300 + ci)
        _, dKa, dVa = A.backward(parent, seg, q, k, v, do, 0.33)
        keys = rng.permutation(T)[: max(1, T // 3)]
        for g in range(2):
            for max_rows in (None, 3):
                dK, dV, pairs = K.key_gradients(parent, seg, q[:, 2 * g:2 * g + 2], k[:, g], v[:, g],
                                                do[:, 2 * g:2 * g + 2], 0.33, keys, max_rows=max_rows)
                assert np.abs(dK - dKa[keys, g]).max() < 1e-11
                assert np.abs(dV - dVa[keys, g]).max() < 1e-11
                assert pairs > 0


def test_key_gradients_against_finite_differences_of_a_brute_force_objective():
    """d/dk and d/dv of sum_t O_t . dO_t, with O from the token-by-token pure
    python forward (no oracle code on the reference side)."""
    from oracle import key_gradient as K
    rng = np.random.default_rng(92)
    parent, seg = random_tree(rng, 6, 4)
    _, vis, T = _token_tables(parent, seg)
    q, k, v, do = _inputs(T, 2, 1, 5, seed=17)
    scale = 0.45
    keys = np.arange(T)
    dK, dV, _ = K.key_gradients(parent, seg, q, k[:, 0], v[:, 0], do, scale, keys)
    f = lambda: float((_brute_forward(vis, q, k, v, scale, 2)[0] * do).sum())
    eps = 1e-5
    for arr, grad in ((k, dK), (v, dV)):
        for _ in range(12):
            t, j = int(rng.integers(0, T)), int(rng.integers(0, 5))
            old = arr[t, 0, j]
            arr[t, 0, j] = old + eps
            fp = f()
            arr[t, 0, j] = old - eps
            fm = f()
            arr[t, 0, j] = old
            fd = (fp - fm) / (2 * eps)
            assert abs(fd - grad[t, j]) < 1e-7 * max(1.0, abs(fd)), (t, j, fd, grad[t, j])


def test_key_gradients_of_all_keys_obey_the_column_sum_identity():
    """Rows of P sum to one, so the dV rows of ALL keys add up to the sum of dO
    over tokens and the q heads of the group; a key set that leaves tokens out
    must fall short of it (the function really restricts itself to its keys)."""
    from oracle import key_gradient as K
    rng = np.random.default_rng(93)
    parent, seg = random_tree(rng, 7, 6, n_roots=2)
    T = int(seg.sum())
    q, k, v, do = _inputs(T, 3, 1, 6, seed=18)
    _, dV, _ = K.key_gradients(parent, seg, q, k[:, 0], v[:, 0], do, 0.3, np.arange(T))
    assert np.abs(dV.sum(axis=0) - do.sum(axis=(0, 1))).max() < 1e-11
    _, dV_part, _ = K.key_gradients(parent, seg, q, k[:, 0], v[:, 0], do, 0.3, np.arange(1, T))
    assert np.abs(dV_part - dV[1:]).max() < 1e-12
