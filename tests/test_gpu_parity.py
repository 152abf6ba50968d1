"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs.

Tolerances are the ones the task states: max|err| / max|ref| <= 1e-5 in fp32
mode and <= 1e-2 in bf16 mode, per tensor (O, LSE, dQ, dK, dV)."""
import math

import numpy as np
import pytest

from oracle import dense_rollout as A
from oracle import tree_direct as B
from oracle import tree_layout as L
from workloads import (chain_tree, config_heads, config_tree, make_inputs_numpy, random_tree,
                       scaled_config_tree)
from parity_util import rel_err, run_hip

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def _compare(parent, seg, Hq, Hkv, d, dtype, seed, oracle=B, scale=None):
    T = int(np.sum(seg))
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    inp = make_inputs_numpy(T, Hq, Hkv, d, seed, dtype=dtype)
    got = run_hip(parent, seg, inp, Hq, Hkv, d, scale, dtype)
    O, LSE = oracle.forward(parent, seg, inp["q"], inp["k"], inp["v"], scale)
    dQ, dK, dV = oracle.backward(parent, seg, inp["q"], inp["k"], inp["v"], inp["do"], scale)
    errs = {"o": rel_err(got["o"], O), "lse": rel_err(got["lse"], LSE), "dq": rel_err(got["dq"], dQ),
            "dk": rel_err(got["dk"], dK), "dv": rel_err(got["dv"], dV)}
    print(f"T={T} Hq={Hq} Hkv={Hkv} d={d} {dtype}: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()),
          flush=True)
    for name, e in errs.items():
        assert e <= TOL[dtype], (name, e)
    if T >= 1024:
        _report_by_depth(parent, seg, got, dict(o=O, dq=dQ, dk=dK, dv=dV))
    return errs


def _report_by_depth(parent, seg, got, ref):
    """Printed, not asserted: the same max|err| / max|ref| ratio inside each
    quarter of the position range.  The per-tensor ratio is dominated by shallow
    tokens (position 0 has O = v, the largest |O|), which could hide errors at
    deep positions; this shows them."""
    off, order = L.node_offsets(parent, seg)
    sd = L.start_depths(parent, seg)
    pos = np.empty(int(np.sum(seg)), dtype=np.int64)
    for u in range(len(parent)):
        pos[off[u]:off[u] + seg[u]] = sd[u] + np.arange(seg[u])
    edges = np.quantile(pos, [0, 0.25, 0.5, 0.75, 1.0]).astype(np.int64)
    for b in range(4):
        sel = (pos >= edges[b]) & ((pos < edges[b + 1]) if b < 3 else (pos <= edges[b + 1]))
        if not sel.any():
            continue
        print(f"  positions {edges[b]}..{edges[b + 1]}: " +
              " ".join(f"{n}={rel_err(np.asarray(got[n])[sel], r[sel]):.2e}" for n, r in ref.items()), flush=True)


def test_config1_fp32_exhaustive_dense_rollout_oracle():
    parent, seg, info = config_tree(1)
    h = config_heads(1)
    _compare(parent, seg, h["n_q_heads"], h["n_kv_heads"], h["head_dim"], "f32", info["tensor_seed"], oracle=A)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 1), (6, 2)])
def test_fp32_random_forests(d, Hq, Hkv):
    rng = np.random.default_rng(1234 + d + Hq)
    for trial in range(3):
        parent, seg = random_tree(rng, int(rng.integers(1, 40)), 70, n_roots=int(rng.integers(1, 4)))
        _compare(parent, seg, Hq, Hkv, d, "f32", seed=trial)


def test_fp32_degenerate_trees():
    _compare(np.array([-1]), np.array([1]), 2, 1, 64, "f32", seed=1)          # one token
    _compare(*chain_tree([1] * 9), 2, 2, 64, "f32", seed=2)                    # unary chain of 1-token nodes
    _compare(*chain_tree([100, 37, 64]), 2, 2, 128, "f32", seed=3)             # chain = causal attention
    _compare(np.array([-1] * 5), np.array([3, 70, 1, 64, 65]), 2, 1, 64, "f32", seed=4)   # forest of single nodes


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("Hq,Hkv", [(4, 1), (8, 2), (2, 1), (1, 1), (3, 1), (16, 2), (32, 8), (16, 1), (5, 1)])
def test_bf16_random_forests(Hq, Hkv, d):
    rng = np.random.default_rng(99 + Hq)
    for trial in range(3):
        parent, seg = random_tree(rng, int(rng.integers(1, 40)), 90, n_roots=int(rng.integers(1, 4)))
        _compare(parent, seg, Hq, Hkv, d, "bf16", seed=trial)


@pytest.mark.parametrize("d", [128, 64])
def test_bf16_degenerate_trees(d):
    _compare(np.array([-1]), np.array([1]), 4, 1, d, "bf16", seed=1)
    _compare(*chain_tree([1] * 9), 4, 1, d, "bf16", seed=2)
    _compare(*chain_tree([300, 37, 64, 128]), 4, 2, d, "bf16", seed=3)
    _compare(np.array([-1] * 5), np.array([3, 70, 1, 64, 65]), 4, 1, d, "bf16", seed=4)


@pytest.mark.parametrize("cfg,shrink,d", [(2, 8, 128), (3, 16, 128), (4, 32, 128), (5, 4, 128),
                                          (2, 8, 64), (3, 16, 64), (4, 32, 64), (5, 4, 64)])
def test_bf16_scaled_down_benchmark_configs(cfg, shrink, d):
    """Siblings of the benchmark trees (same branching, shorter segments) checked
    on whole tensors, with the benchmark's head_dim 128 and with head_dim 64; two
    kv groups keep the oracle to seconds."""
    parent, seg, info = scaled_config_tree(cfg, shrink)
    G = config_heads(cfg)["n_q_heads"] // config_heads(cfg)["n_kv_heads"]
    _compare(parent, seg, 2 * G, 2, d, "bf16", seed=info["tensor_seed"])


@pytest.mark.parametrize("d", [128, 64])
def test_bf16_long_walks_on_256_key_tiles(d):
    """A tree whose key tiles walk far enough for the schedule to choose tiles of
    256 keys (the eight-wave form of the dK/dV kernel, pieces of split walks in
    fp32 partial sums; the full-size tests run the same form under queues): a ragged
    5963-token prompt with five long responses, whole tensors of every head
    against the oracle.  Segment lengths are not multiples of the tile size, so
    tiles straddle node boundaries and end in ragged tails."""
    import paper_2602_00482_amd as dta
    rng = np.random.default_rng(256 + d)
    seg = np.array([5963] + [int(x) for x in rng.integers(2200, 2800, size=5)])
    parent = np.array([-1] + [0] * 5)
    tree = dta.tree_build(parent, seg)
    sch = tree.schedule_info(dta.AttnParams(8, 2, d, 1.0 / math.sqrt(d), dta.BF16))
    tree.destroy()
    assert sch["bwd_kv_tile_tokens"] == 256, sch
    _compare(parent, seg, 8, 2, d, "bf16", seed=256 + d)


def test_bf16_head_dim_64_long_shared_prefix_with_split_key_tiles():
    """head_dim 64 on a tree whose prompt tiles are split into fp32 partial sums and
    whose launches are large enough to draw work from queues: a 1500-token prompt
    with 24 responses, whole tensors of one kv group against the oracle."""
    rng = np.random.default_rng(64)
    seg = np.array([1500] + [int(x) for x in rng.integers(200, 900, size=24)])
    parent = np.array([-1] + [0] * 24)
    _compare(parent, seg, 8, 2, 64, "bf16", seed=64)
