"""CPU-only tests of the C-ABI library: it loads, exports every symbol the
header declares, builds tree metadata that agrees with the oracle's own
bookkeeping, produces a valid tile schedule, and returns the documented error
codes.  No compute call is made (there is no GPU here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2602_00482_amd as dta
from oracle import tree_layout as L
from workloads import chain_tree, config_tree, random_tree, scaled_config_tree

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    from paper_2602_00482_amd import probe
    for hdr, mod in (("dta.h", dta), ("dta_probe.h", probe)):
        header = open(os.path.join(ROOT, "include", hdr)).read()
        declared = set(re.findall(r"\b(dta_[a-z0-9_]+)\s*\(", header))
        assert declared == set(mod.exported_symbols), hdr
        lib = mod.load_library()
        for name in declared:
            assert hasattr(lib, name), name
    # the measurement kernels are not in the attention library
    assert not hasattr(dta.load_library(), "dta_probe_mfma_bf16")
    lib = dta.load_library()
    assert lib.dta_status_string(0) == b"DTA_OK"
    assert lib.dta_status_string(-2) == b"DTA_ERR_BAD_TREE"


def _brute_kend(parent, seg, off):
    """kend[k] by definition: one past the last packed token whose root path
    contains k, found by walking every token's ancestors."""
    T = int(np.sum(seg))
    node_of = np.zeros(T, dtype=np.int64)
    for u in range(len(parent)):
        node_of[off[u]:off[u] + seg[u]] = u
    last = np.arange(T)
    for t in range(T):
        u = node_of[t]
        last[off[u]:t + 1] = np.maximum(last[off[u]:t + 1], t)
        a = parent[u]
        while a >= 0:
            last[off[a]:off[a] + seg[a]] = np.maximum(last[off[a]:off[a] + seg[a]], t)
            a = parent[a]
    return last + 1


@pytest.mark.parametrize("seed", range(8))
def test_layout_matches_oracle_bookkeeping(seed):
    rng = np.random.default_rng(seed)
    parent, seg = random_tree(rng, int(rng.integers(1, 30)), 9, n_roots=int(rng.integers(1, 4)))
    tree = dta.tree_build(parent, seg)
    lay, info = tree.layout(), tree.info()
    off, T = L.node_offsets(parent, seg)
    assert list(lay["dfs_order"]) == L.preorder(parent)
    assert (lay["node_offset"] == off).all()
    assert (lay["node_start_depth"] == L.start_depths(parent, seg)).all()
    st = L.tree_stats(parent, seg)
    for key in ("n_nodes", "n_tokens", "n_leaves", "max_path_tokens", "unique_pairs", "rollout_tokens",
                "rollout_tokens_full", "dense_pairs", "dense_pairs_full"):
        assert info[key] == st[key], key
    # subtree ranges are contiguous: [offset, offset + subtree_tokens) holds exactly the descendants
    for u in range(len(parent)):
        inside = [v for v in range(len(parent)) if u in L.node_path(parent, v)]
        assert lay["subtree_tokens"][u] == sum(int(seg[v]) for v in inside)
        assert all(off[u] <= off[v] < off[u] + lay["subtree_tokens"][u] for v in inside)
    # ancestor interval lists cover exactly the ancestor tokens, root first, merged when adjacent
    for u in range(len(parent)):
        a, b = lay["anc_ptr"][u], lay["anc_ptr"][u + 1]
        toks = np.concatenate([np.arange(o, o + n) for o, n in zip(lay["anc_seg_off"][a:b], lay["anc_seg_len"][a:b])]
                              + [np.zeros(0, dtype=np.int64)])
        assert (toks == L.ancestor_token_indices(parent, seg, off, u)).all()
        ends = lay["anc_seg_off"][a:b] + lay["anc_seg_len"][a:b]
        assert (ends[:-1] != lay["anc_seg_off"][a + 1:b]).all()
    assert (lay["token_kend"] == _brute_kend(parent, seg, off)).all()
    tree.destroy()


def test_interval_mask_equals_rollout_membership():
    """visible(t, k) <=> k <= t < kend[k] reproduces exactly the (query, key)
    pairs of the expanded rollouts."""
    rng = np.random.default_rng(3)
    parent, seg = random_tree(rng, 12, 5, n_roots=2)
    tree = dta.tree_build(parent, seg)
    kend = tree.layout()["token_kend"]
    T = int(seg.sum())
    want = np.zeros((T, T), dtype=bool)
    for idx in L.rollout_token_paths(parent, seg):
        for j, t in enumerate(idx):
            want[t, idx[:j + 1]] = True
    k = np.arange(T)
    got = (k[None, :] <= k[:, None]) & (k[:, None] < kend[None, :])
    assert (got == want).all()
    assert int(got.sum()) == tree.info()["unique_pairs"]
    tree.destroy()


def test_config_counts_and_schedule_cover_every_pair():
    p = dta.AttnParams(32, 8, 128, 0.1, dta.BF16)
    for cfg in (1, 2, 3, 5):
        parent, seg, _ = config_tree(cfg)
        tree = dta.tree_build(parent, seg)
        info, sch = tree.info(), tree.schedule_info(p)
        assert sch["fwd_work_items"] == -(-info["n_tokens"] // sch["fwd_q_tile_tokens"])
        # long key-tile walks may be cut into several launch items
        assert sch["bwd_work_items"] >= -(-info["n_tokens"] // sch["bwd_kv_tile_tokens"])
        # a tile streams at least the pairs it owns
        assert sch["fwd_tile_pairs"] >= info["unique_pairs"]
        assert sch["bwd_tile_pairs"] >= info["unique_pairs"]
        # kend[] (4 bytes per token) plus at least 16 bytes per query tile and 32 per key item
        assert sch["metadata_bytes"] >= 4 * info["n_tokens"] + 16 * sch["fwd_work_items"] + 32 * sch["bwd_work_items"]
        assert sch["metadata_bytes"] < 64 * info["n_tokens"]
        tree.destroy()
    parent, seg, _ = config_tree(4)
    tree = dta.tree_build(parent, seg)
    assert tree.info()["n_tokens"] == 277504 and tree.info()["unique_pairs"] == 5285748224
    tree.destroy()


def test_error_codes():
    lib = dta.load_library()
    i32 = lambda a: np.asarray(a, dtype=np.int32).ctypes.data_as(C.POINTER(C.c_int32))
    h = C.c_void_p()
    build = lambda par, seg, n=None, flags=0: lib.dta_tree_build(i32(par), i32(seg), len(par) if n is None else n,
                                                                   flags, C.byref(h))
    assert build([-1], [1]) == 0
    lib.dta_tree_destroy(h)
    assert build([-1], [1], n=0) == -1                     # n_nodes < 1
    assert build([-1], [1], flags=1) == -1                 # unknown flag
    assert lib.dta_tree_build(None, i32([1]), 1, 0, C.byref(h)) == -1
    assert build([-1, 5], [1, 1]) == -2                    # parent out of range
    assert build([-1, 1], [1, 1]) == -2                    # self parent
    assert build([-1, 2, 1], [1, 1, 1]) == -2              # cycle 1 <-> 2
    assert build([-1, 0], [1, 0]) == -2                    # empty segment
    assert build([-1, 0], [2 ** 31 - 1, 2 ** 31 - 1]) == -2   # token count overflow
    assert h.value is None
    tree = dta.tree_build([-1, 0], [3, 4])
    for bad, want in ((dta.AttnParams(4, 3, 128, 1.0, dta.BF16), -3),      # Hq % Hkv
                      (dta.AttnParams(4, 2, 96, 1.0, dta.F32), -3),        # head_dim
                      (dta.AttnParams(4, 2, 32, 1.0, dta.BF16), -3),       # head_dim 64 or 128 only
                      (dta.AttnParams(4, 2, 128, 1.0, 7), -3),             # dtype
                      (dta.AttnParams(0, 1, 128, 1.0, dta.BF16), -1),
                      (dta.AttnParams(4, 2, 128, 0.0, dta.BF16), -1),      # scale: finite, nonzero
                      (dta.AttnParams(4, 2, 128, float("inf"), dta.BF16), -1),
                      (dta.AttnParams(4, 2, 64, float("nan"), dta.F32), -1)):
        with pytest.raises(dta.DtaError) as err:
            tree.schedule_info(bad)
        assert err.value.status == want
        assert dta.workspace_bytes(tree, bad, True) == 0
    good = dta.AttnParams(4, 2, 128, 1.0, dta.BF16)
    # the forward's (optional) workspace: work-queue counters in bf16 mode only
    assert dta.workspace_bytes(tree, good, False) == 256
    assert dta.workspace_bytes(tree, dta.AttnParams(4, 2, 128, 1.0, dta.F32), False) == 0
    assert dta.workspace_bytes(tree, good, True) >= 7 * 4 * 4
    # null tensors are rejected before anything touches the device
    z = C.c_void_p(0)
    assert lib.dta_tree_attn_fwd(tree.handle, C.byref(good), z, z, z, z, z, z, 0, z) == -1
    assert lib.dta_tree_attn_bwd(tree.handle, C.byref(good), z, z, z, z, z, z, z, z, z, z, 0, z) == -1
    assert lib.dta_tree_attn_bwd_stages(tree.handle, C.byref(good), z, z, z, z, z, z, z, z, z, z, 0, z, 0) == -1
    assert lib.dta_tree_attn_bwd_stages(tree.handle, C.byref(good), z, z, z, z, z, z, z, z, z, z, 0, z, 8) == -1
    # the rate probe checks its arguments before launching anything
    from paper_2602_00482_amd import probe
    lib = probe.load_library()
    one = C.c_void_p(1)
    assert lib.dta_probe_mfma_bf16(1, 1, z, one, z, None, None) == -1
    assert lib.dta_probe_mfma_bf16(1, 1, one, z, z, None, None) == -1
    assert lib.dta_probe_mfma_bf16(0, 1, one, one, z, None, None) == -1
    assert lib.dta_probe_mfma_bf16(1, 0, one, one, z, None, None) == -1
    assert lib.dta_probe_mfma_bf16(2 ** 20 + 1, 1, one, one, z, None, None) == -1
    assert lib.dta_probe_overlap(1, 1, 1, z, z) == -1
    assert lib.dta_probe_overlap(0, 1, 1, one, z) == -1
    assert lib.dta_probe_overlap(1, -1, 1, one, z) == -1
    assert lib.dta_probe_overlap(1, 1, 2 ** 24 + 1, one, z) == -1
    dta.load_library().dta_tree_destroy(None)
    tree.destroy()


def test_unary_chain_packs_like_one_segment():
    parent, seg = chain_tree([3, 1, 4])
    tree = dta.tree_build(parent, seg)
    lay = tree.layout()
    assert list(lay["node_offset"]) == [0, 3, 4]
    assert list(lay["token_kend"]) == [8] * 8
    # ancestors of the last node merge into one interval [0, 4)
    assert lay["anc_seg_off"][lay["anc_ptr"][2]:lay["anc_ptr"][3]].tolist() == [0]
    assert lay["anc_seg_len"][lay["anc_ptr"][2]:lay["anc_ptr"][3]].tolist() == [4]
    tree.destroy()


def test_binding_refuses_tensors_of_another_tree_before_any_launch():
    """The C ABI takes no tensor sizes, so a tree built for more tokens than the
    tensors hold would make the kernels index past them.  The wrappers compare
    the row count with the tree's n_tokens first (no GPU is needed to get the
    refusal: CPU tensors of the wrong length are turned away for their length)."""
    import torch
    tree = dta.tree_build([-1, 0], [3, 4])
    assert tree.n_tokens == 7
    p = dta.AttnParams(2, 1, 128, 1.0, dta.BF16)
    mk = lambda rows, heads, dt=torch.bfloat16: torch.zeros((rows, heads, 128), dtype=dt)
    q, k, v = mk(5, 2), mk(5, 1), mk(5, 1)
    lse = torch.zeros((5, 2))
    with pytest.raises(ValueError, match="n_tokens = 7"):
        dta.tree_attn_fwd(tree, p, q, k, v)
    with pytest.raises(ValueError, match="n_tokens = 7"):
        dta.tree_attn_bwd(tree, p, q, k, v, q, lse, q)
    with pytest.raises(ValueError, match="n_tokens = 7"):
        dta.tree_attn_fwd_segment(tree, p, 0, 3, q, k, v, q, lse)
    with pytest.raises(ValueError, match="n_tokens = 7"):
        dta.tree_attn_bwd_segment(tree, p, 0, 3, q, k, v, q, lse, q, q, mk(5, 1, torch.float32),
                                  mk(5, 1, torch.float32), torch.zeros(256, dtype=torch.uint8))
    tree.destroy()
    with pytest.raises(ValueError, match="destroyed"):
        dta.tree_attn_fwd(tree, p, mk(7, 2), mk(7, 1), mk(7, 1))
