"""GPU tests of the C-ABI behaviour around the kernels: staged backward equals
the one-call backward, results are bit-reproducible, the split dK/dV path is
exercised and agrees with the oracle, a negative softmax scale works, and
run-time argument errors are reported."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

import paper_2602_00482_amd as dta
from paper_2602_00482_amd import probe
from oracle import tree_direct as B
from workloads import make_inputs_numpy, random_tree
from parity_util import rel_err, run_hip

pytestmark = pytest.mark.gpu


def _setup(parent, seg, Hq, Hkv, d, dtype, seed, scale=None):
    T = int(np.sum(seg))
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    x = make_inputs_numpy(T, Hq, Hkv, d, seed, dtype=dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    t = {n: torch.from_numpy(a).cuda().to(tdt).contiguous() for n, a in x.items()}
    tree = dta.tree_build(parent, seg)
    p = dta.AttnParams(Hq, Hkv, d, float(scale), dta.F32 if dtype == "f32" else dta.BF16)
    return x, t, tree, p, scale


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64)])
def test_staged_backward_equals_one_call_and_is_reproducible(dtype, d):
    rng = np.random.default_rng(5)
    parent, seg = random_tree(rng, 25, 300, n_roots=2)
    x, t, tree, p, _ = _setup(parent, seg, 8, 2, d, dtype, seed=1)
    o, lse = dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"])
    o2, lse2 = dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"])
    assert torch.equal(o, o2) and torch.equal(lse, lse2)
    ref = dta.tree_attn_bwd(tree, p, t["q"], t["k"], t["v"], o, lse, t["do"])
    again = dta.tree_attn_bwd(tree, p, t["q"], t["k"], t["v"], o, lse, t["do"])
    for a, b in zip(ref, again):
        assert torch.equal(a, b)                 # no atomics anywhere: bit-reproducible
    ws = torch.empty(dta.workspace_bytes(tree, p, True), dtype=torch.uint8, device="cuda")
    dq, dk, dv = (torch.full_like(a, float("nan")) for a in ref)
    args = (tree, p, t["q"], t["k"], t["v"], o, lse, t["do"], dq, dk, dv, ws)
    dta.tree_attn_bwd(*args, stages=dta.BWD_DELTA)
    dta.tree_attn_bwd(*args, stages=dta.BWD_DKDV)
    assert torch.isnan(dq).all()                 # stages that were not asked for leave their outputs alone
    dta.tree_attn_bwd(*args, stages=dta.BWD_DQ)
    torch.cuda.synchronize()
    for a, b in zip(ref, (dq, dk, dv)):
        assert torch.equal(a, b)
    # asked for together, the dQ launch computes the row statistics itself and leaves
    # them in the workspace for a later dK/dV call: same bits again
    ws.fill_(0xff)
    dq, dk, dv = (torch.full_like(a, float("nan")) for a in ref)
    args = (tree, p, t["q"], t["k"], t["v"], o, lse, t["do"], dq, dk, dv, ws)
    dta.tree_attn_bwd(*args, stages=dta.BWD_DELTA | dta.BWD_DQ)
    assert torch.isnan(dk).all()
    dta.tree_attn_bwd(*args, stages=dta.BWD_DKDV)
    torch.cuda.synchronize()
    for a, b in zip(ref, (dq, dk, dv)):
        assert torch.equal(a, b)
    tree.destroy()


def test_split_key_tiles_are_exercised_and_correct():
    """One long root whose key tiles have much longer walks than the leaves':
    the schedule must cut them, and the reduced result must match the oracle."""
    parent = np.array([-1] + [0] * 6, dtype=np.int32)
    seg = np.array([700, 90, 33, 260, 64, 129, 17], dtype=np.int32)
    tree = dta.tree_build(parent, seg)
    p = dta.AttnParams(8, 2, 128, 0.088, dta.BF16)
    sch = tree.schedule_info(p)
    assert sch["bwd_work_items"] > -(-int(seg.sum()) // sch["bwd_kv_tile_tokens"])
    assert dta.workspace_bytes(tree, p, True) > int(seg.sum()) * 8 * 4 + 256
    tree.destroy()
    T = int(seg.sum())
    x = make_inputs_numpy(T, 8, 2, 128, 3, dtype="bf16")
    got = run_hip(parent, seg, x, 8, 2, 128, 0.088, "bf16")
    dQ, dK, dV = B.backward(parent, seg, x["q"], x["k"], x["v"], x["do"], 0.088)
    assert rel_err(got["dq"], dQ) <= 1e-2 and rel_err(got["dk"], dK) <= 1e-2 and rel_err(got["dv"], dV) <= 1e-2


@pytest.mark.parametrize("dtype,d,tol", [("bf16", 128, 1e-2), ("bf16", 64, 1e-2), ("f32", 128, 1e-5)])
def test_negative_and_large_scale(dtype, d, tol):
    rng = np.random.default_rng(9)
    parent, seg = random_tree(rng, 12, 150)
    T = int(seg.sum())
    for scale in (-0.05, 0.3):
        x = make_inputs_numpy(T, 4, 2, d, 4, dtype=dtype)
        got = run_hip(parent, seg, x, 4, 2, d, scale, dtype)
        O, LSE = B.forward(parent, seg, x["q"], x["k"], x["v"], scale)
        dQ, dK, dV = B.backward(parent, seg, x["q"], x["k"], x["v"], x["do"], scale)
        for name, ref in (("o", O), ("lse", LSE), ("dq", dQ), ("dk", dK), ("dv", dV)):
            assert rel_err(got[name], ref) <= tol, (scale, name)


def test_runtime_argument_errors():
    parent, seg = np.array([-1, 0], dtype=np.int32), np.array([40, 30], dtype=np.int32)
    x, t, tree, p, _ = _setup(parent, seg, 4, 2, 128, "bf16", seed=2)
    o, lse = dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"])
    lib = dta.load_library()
    ptr = lambda a: C.c_void_p(a.data_ptr())
    z = C.c_void_p(0)
    need = dta.workspace_bytes(tree, p, True)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dq, dk, dv = torch.empty_like(t["q"]), torch.empty_like(t["k"]), torch.empty_like(t["v"])
    base = [tree.handle, C.byref(p), ptr(t["q"]), ptr(t["k"]), ptr(t["v"]), ptr(o), ptr(lse), ptr(t["do"]),
            ptr(dq), ptr(dk), ptr(dv)]
    assert lib.dta_tree_attn_bwd(*base, ptr(ws), need - 1, z) == -6          # workspace too small
    assert lib.dta_tree_attn_bwd(*base, z, need, z) == -6                    # workspace null
    assert lib.dta_tree_attn_bwd(*base, C.c_void_p(ws.data_ptr() + 16), need, z) == -6   # not 256-aligned
    mis = C.c_void_p(t["q"].data_ptr() + 2)
    assert lib.dta_tree_attn_fwd(tree.handle, C.byref(p), mis, ptr(t["k"]), ptr(t["v"]), ptr(o), ptr(lse),
                                 z, 0, z) == -1                              # misaligned tensor
    assert lib.dta_tree_attn_bwd(*base, ptr(ws), need, z) == 0
    torch.cuda.synchronize()
    tree.destroy()


def test_destroy_right_after_launch_and_metadata_reuse():
    """A tree may be destroyed while its kernels are still queued; trees built
    back to back (whose metadata allocations get recycled) must not disturb
    each other's results."""
    outs = []
    for rep in range(2):
        res = []
        for seed in (11, 12, 13, 14):
            rng = np.random.default_rng(seed)
            parent, seg = random_tree(rng, 9 + seed % 3, 700 + 50 * (seed % 4))
            x, t, tree, p, _ = _setup(parent, seg, 8, 2, 128, "bf16", seed=seed)
            o, lse = dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"])
            grads = dta.tree_attn_bwd(tree, p, t["q"], t["k"], t["v"], o, lse, t["do"])
            tree.destroy()            # kernels may still be running
            res.append((o, lse) + tuple(grads))
        torch.cuda.synchronize()
        outs.append([[a.float().cpu() for a in r] for r in res])
    for a, b in zip(outs[0], outs[1]):
        for u, v in zip(a, b):
            assert torch.equal(u, v)


def test_mfma_rate_probe_is_linear_in_its_iteration_count():
    """The probe's operands are constant over the loop and exactly representable
    (multiples of 1/64 below 2 in size), so every accumulator after n iterations is
    n times its value after one, exactly, as long as the sums stay below 2^24/4096;
    the operation count follows the documented formula; both counters advance."""
    n_blocks = 3
    outs = {}
    for iters in (1, 2, 8):
        out = torch.full((n_blocks * 256,), float("nan"), dtype=torch.float32, device="cuda")
        ticks = torch.zeros(2 * n_blocks, dtype=torch.int64, device="cuda")
        flop, khz = probe.probe_mfma_bf16(n_blocks, iters, out, ticks)
        torch.cuda.synchronize()
        assert flop == n_blocks * 4 * iters * 16 * 2 * 32 * 32 * 16
        assert khz > 0
        assert bool((ticks > 0).all())
        assert bool(torch.isfinite(out).all())
        outs[iters] = out.cpu()
    assert float(outs[1].abs().max()) > 0
    assert torch.equal(outs[2], 2 * outs[1])
    assert torch.equal(outs[8], 8 * outs[1])


def test_overlap_probe_runs_and_writes_every_element():
    out = torch.full((2 * 512,), float("nan"), dtype=torch.float32, device="cuda")
    for m, v in ((3, 0), (0, 3), (3, 3)):
        out.fill_(float("nan"))
        probe.probe_overlap(2, m, v, out)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all())


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [("bf16", 128, 8, 2), ("bf16", 64, 8, 2), ("f32", 64, 4, 2)])
def test_outputs_with_sentinel_guards_on_both_sides_stay_inside_their_rows(dtype, d, Hq, Hkv):
    """Every output (and the workspaces) is a window inside a larger allocation
    filled with a byte pattern; after forward and backward the bytes before and
    after each window must be untouched.  The tree has a ragged tail in every
    tile size (T = 1 mod 32) and split key tiles."""
    rng = np.random.default_rng(23)
    parent, seg = random_tree(rng, 12, 260, n_roots=2)
    seg[0] += (1 - int(seg.sum())) % 32          # T = 1 (mod 32)
    x, t, tree, p, _ = _setup(parent, seg, Hq, Hkv, d, dtype, seed=6)
    T = int(seg.sum())
    GUARD = 1 << 16                               # bytes on each side
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16

    def guarded(shape, dt):
        n = int(np.prod(shape)) * torch.empty(0, dtype=dt).element_size()
        raw = torch.full((GUARD + n + GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        return raw, raw[GUARD:GUARD + n].view(dt).view(*shape)

    bufs = {name: guarded(shape, dt) for name, shape, dt in (
        ("o", (T, Hq, d), tdt), ("lse", (T, Hq), torch.float32), ("dq", (T, Hq, d), tdt),
        ("dk", (T, Hkv, d), tdt), ("dv", (T, Hkv, d), tdt),
        ("ws_fwd", (max(256, dta.workspace_bytes(tree, p, False)),), torch.uint8),
        ("ws_bwd", (max(256, dta.workspace_bytes(tree, p, True)),), torch.uint8))}
    w = {n: b[1] for n, b in bufs.items()}
    dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"], w["o"], w["lse"], w["ws_fwd"])
    dta.tree_attn_bwd(tree, p, t["q"], t["k"], t["v"], w["o"], w["lse"], t["do"], w["dq"], w["dk"], w["dv"],
                      w["ws_bwd"])
    torch.cuda.synchronize()
    tree.destroy()
    for name, (raw, win) in bufs.items():
        assert bool((raw[:GUARD] == 0xA5).all()), f"{name}: bytes before the buffer were written"
        assert bool((raw[-GUARD:] == 0xA5).all()), f"{name}: bytes after the buffer were written"
    # and the windows hold the same results as ordinary allocations
    ref = run_hip(parent, seg, x, Hq, Hkv, d, 1.0 / math.sqrt(d), dtype)
    for name in ("o", "lse", "dq", "dk", "dv"):
        assert np.array_equal(w[name].double().cpu().numpy(), ref[name]), name


def test_more_segment_ranges_than_the_schedule_cache_holds():
    """A tree keeps at most max(1024, 4 x nodes + 64) segment schedules (1024 for this
    one-node tree); beyond that the least recently used one is dropped and its
    device block is reused.  1300 one-row forward
    calls, then the first rows again (their schedules are gone and are rebuilt
    into recycled blocks): all rows must equal the one-launch forward."""
    T = 1300
    x, t, tree, p, _ = _setup([-1], [T], 2, 1, 128, "bf16", seed=8)
    o_ref, lse_ref = dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"])
    o = torch.zeros_like(o_ref)
    lse = torch.zeros_like(lse_ref)
    for r in list(range(T)) + list(range(0, 300)):
        dta.tree_attn_fwd_segment(tree, p, r, r + 1, t["q"], t["k"], t["v"], o, lse)
    torch.cuda.synchronize()
    tree.destroy()
    assert float((lse - lse_ref).abs().max()) <= 1e-5
    assert float((o.double() - o_ref.double()).abs().max() / o_ref.double().abs().max()) <= 1e-2
