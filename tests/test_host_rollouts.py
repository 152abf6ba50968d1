"""Host library: rollout sequences -> prefix tree and the load-balanced
DFS-contiguous partitioning, bit for bit against the CPU oracle (no GPU)."""
import numpy as np
import pytest

import paper_2602_00482_amd as dta
from oracle import rollout_tree as R
from oracle import tree_layout as L


def _random_rollouts(rng, n, alphabet, max_len, p_extend=0.5):
    seqs = [list(rng.integers(0, alphabet, size=int(rng.integers(1, max_len + 1))))]
    for _ in range(n - 1):
        src = seqs[int(rng.integers(0, len(seqs)))]
        keep = int(rng.integers(0, len(src) + 1))
        extra = int(rng.integers(0 if keep else 1, max_len + 1)) if rng.random() < p_extend or keep == 0 else 0
        s = list(src[:keep]) + list(rng.integers(0, alphabet, size=extra))
        seqs.append(s if s else [int(rng.integers(0, alphabet))])
    return [[int(t) for t in s] for s in seqs]


def _check_against_oracle(seqs):
    ref = R.build_tree(seqs)
    r = dta.Rollouts(seqs)
    v = r.view()
    assert v["parent"].tolist() == ref["parent"]
    assert v["seg_len"].tolist() == ref["seg_len"]
    assert v["tokens"].tolist() == ref["tokens"]
    assert v["seq_node"].tolist() == ref["seq_node"]
    assert v["order"].tolist() == ref["order"]
    pi = [seqs[i] for i in ref["order"]]
    assert v["lcp"].tolist() == [0] + [R.lcp(a, b) for a, b in zip(pi, pi[1:])]
    for K in sorted({1, 2, 3, len(seqs) // 2, len(seqs)} & set(range(1, len(seqs) + 1))):
        _, cuts = R.partition(seqs, K)
        gb, gc = r.partition(K)
        assert gb.tolist() == [a for a, _ in cuts] + [len(seqs)]
        assert gc.tolist() == [R.group_cost(pi, a, b) for a, b in cuts]
    r.destroy()
    return v


def test_small_random_rollouts_match_the_oracle():
    rng = np.random.default_rng(201)
    for trial in range(200):
        _check_against_oracle(_random_rollouts(rng, int(rng.integers(1, 14)), int(rng.integers(1, 4)), 8))


def test_grpo_like_group_and_tree_build():
    """One prompt, 16 sampled responses that diverge at random points (the shape
    of the paper's GRPO workloads): the arrays feed dta_tree_build unchanged and
    the packed order is the identity."""
    rng = np.random.default_rng(202)
    prompt = rng.integers(0, 50000, size=700).tolist()
    seqs = []
    for i in range(16):
        base = seqs[int(rng.integers(0, len(seqs)))] if seqs and rng.random() < 0.6 else prompt
        keep = int(rng.integers(len(prompt), len(base) + 1))
        seqs.append(base[:keep] + rng.integers(0, 50000, size=int(rng.integers(50, 900))).tolist())
    v = _check_against_oracle(seqs)
    tree = dta.tree_build(v["parent"], v["seg_len"])
    info = tree.info()
    assert info["n_tokens"] == len(v["tokens"]) and info["n_leaves"] <= 16
    lay = tree.layout()
    assert lay["dfs_order"].tolist() == list(range(len(v["parent"])))
    off, _ = L.node_offsets(v["parent"], v["seg_len"])
    assert lay["node_offset"].tolist() == off.tolist()
    assert info["rollout_tokens"] <= sum(len(s) for s in seqs)     # contained rollouts are not leaves
    tree.destroy()


def test_duplicates_containment_and_single_sequence():
    _check_against_oracle([[5, 5, 5]])
    _check_against_oracle([[1, 2], [1, 2], [1, 2]])
    _check_against_oracle([[1, 2, 3, 4], [1, 2], [1], [1, 2, 3]])
    _check_against_oracle([[3], [2], [1], [2, 2], [2, 1]])
    _check_against_oracle([[2 ** 31 - 1, 0], [2 ** 31 - 1, -5], [-7]])          # ids are compared as signed int32


def test_argument_errors():
    import ctypes as C
    lib = dta.load_library()
    h = C.c_void_p()
    i32 = lambda a: np.asarray(a, dtype=np.int32).ctypes.data_as(C.POINTER(C.c_int32))
    i64 = lambda a: np.asarray(a, dtype=np.int64).ctypes.data_as(C.POINTER(C.c_int64))
    assert lib.dta_rollouts_build(i32([1, 2]), i64([0, 2]), 0, C.byref(h)) == -1      # no sequence
    assert lib.dta_rollouts_build(i32([1, 2]), i64([0, 1, 1]), 2, C.byref(h)) == -1   # empty sequence
    assert lib.dta_rollouts_build(i32([1, 2]), i64([1, 2]), 1, C.byref(h)) == -1      # offsets start at 0
    assert lib.dta_rollouts_build(None, i64([0, 1]), 1, C.byref(h)) == -1
    assert h.value is None
    r = dta.Rollouts([[1, 2], [1, 3]])
    for k in (0, 3, -1):
        with pytest.raises(dta.DtaError) as err:
            r.partition(k)
        assert err.value.status == -1
    lib.dta_rollouts_destroy(None)
    r.destroy()
