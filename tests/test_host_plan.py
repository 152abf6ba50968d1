"""Host library: backward DFS leaf order and leaf-order schedule with chunked
pops (dta_tree_plan), bit for bit against the CPU oracle (no GPU)."""
import numpy as np
import pytest

import paper_2602_00482_amd as dta
from oracle import dfs_schedule as S
from workloads import chain_tree, config_tree, random_tree

TAG = {"FWD": dta.OP_FWD, "REFWD": dta.OP_REFWD, "BWD": dta.OP_BWD, "NOGRAD": dta.OP_FWD_NOGRAD}


def _check(parent, seg, block):
    ops, pi = S.schedule(parent, seg, block)
    tree = dta.tree_build(parent, seg)
    plan = dta.tree_plan(tree, block)
    info = tree.info()
    tree.destroy()
    assert plan["leaf_order"] == pi
    assert plan["ops"] == [(TAG[t], leaf, lo, hi) for t, leaf, lo, hi in ops]
    calls = []
    for (t, leaf, lo, hi), a, b in zip(ops, plan["call_ptr"], plan["call_ptr"][1:]):
        rng = S.path_ranges(parent, seg, leaf, lo, hi)
        if t == "BWD":
            rng = rng[::-1]
        assert [(c[2], c[3]) for c in plan["calls"][a:b]] == rng
        assert all(c[0] == TAG[t] for c in plan["calls"][a:b])
    assert plan["call_ptr"][-1] == len(plan["calls"])
    assert plan["n_fwd"] == info["n_leaves"] == sum(t[0] == "FWD" for t in ops)
    assert plan["n_fwd_nograd"] == sum(t[0] == "NOGRAD" for t in ops) <= info["n_leaves"]
    assert plan["n_chunks"] == sum(t[0] == "BWD" for t in ops)
    assert plan["max_stack_tokens"] == info["max_path_tokens"]
    return plan


@pytest.mark.parametrize("block", [0, 1, 7, 100])
def test_random_forests_match_the_oracle(block):
    rng = np.random.default_rng(400 + block)
    for trial in range(40):
        parent, seg = random_tree(rng, int(rng.integers(1, 30)), 12, n_roots=int(rng.integers(1, 4)))
        _check(parent, seg, block)


def test_benchmark_trees_and_chains():
    for cfg in (1, 2, 3):
        parent, seg, _ = config_tree(cfg)
        for block in (0, 2048):
            _check(parent, seg, block)
    _check(*chain_tree([5, 1, 9]), 4)
    _check(np.array([-1]), np.array([1]), 0)


def test_worked_example():
    plan = _check([-1, 0, 0, 2, 2, 0], [4, 2, 3, 5, 1, 6], 0)
    assert plan["leaf_order"] == [3, 4, 5, 1]
    assert plan["ops"][:2] == [(dta.OP_FWD, 3, 0, 12), (dta.OP_FWD_NOGRAD, 3, 0, 7)]


def test_argument_errors():
    import ctypes as C
    lib = dta.load_library()
    h = C.c_void_p()
    assert lib.dta_tree_plan(None, 0, C.byref(h)) == -1
    assert lib.dta_plan_view(None, None) == -1
    lib.dta_plan_destroy(None)
