"""GPU parity of the segment calls (the attention inside the paper's FWD / BWD
primitives, issued per token segment by its push / pop traversal) against the
fp64 push/pop executor oracle.

The calls are issued in exactly the order the oracle's traversal takes them
(its trace), through the C ABI.  K and V rows are handed to the device only
while their segment is on the active stack and are overwritten with NaN when it
is popped, so a call that read anything outside the current root path would
poison its results.

Tolerances as for the whole-tree calls: max|err| / max|ref| <= 1e-5 (fp32),
<= 1e-2 (bf16), per tensor."""
import math

import numpy as np
import pytest
import torch

import paper_2602_00482_amd as dta
from oracle import dfs_executor as X
from workloads import chain_tree, config_heads, config_tree, make_inputs_numpy, random_tree
from parity_util import rel_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def _run_executor(parent, seg, inp, Hq, Hkv, d, scale, dtype, trace):
    """Replays `trace` [(tag, node, t0, t1)] with segment calls."""
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    dev = torch.device("cuda:0")
    full = {n: torch.from_numpy(a).to(dev).to(tdt).contiguous() for n, a in inp.items()}
    T = full["q"].shape[0]
    nan = float("nan")
    k = torch.full_like(full["k"], nan)
    v = torch.full_like(full["v"], nan)
    o = torch.full_like(full["q"], nan)
    lse = torch.full((T, Hq), nan, dtype=torch.float32, device=dev)
    dq = torch.full_like(full["q"], nan)
    dk_acc = torch.zeros((T, Hkv, d), dtype=torch.float32, device=dev)
    dv_acc = torch.zeros_like(dk_acc)
    tree = dta.tree_build(parent, seg)
    p = dta.AttnParams(Hq, Hkv, d, float(scale), dta.F32 if dtype == "f32" else dta.BF16)
    ws = torch.empty(max(256, dta.workspace_bytes(tree, p, True)), dtype=torch.uint8, device=dev)
    dk_out = torch.full_like(dk_acc, nan)
    dv_out = torch.full_like(dv_acc, nan)
    for tag, node, t0, t1 in trace:
        if tag == "FWD":        # push: the segment's keys/values join the stack
            k[t0:t1] = full["k"][t0:t1]
            v[t0:t1] = full["v"][t0:t1]
        if tag in ("FWD", "REFWD"):
            dta.tree_attn_fwd_segment(tree, p, t0, t1, full["q"], k, v, o, lse)
        else:                   # pop: backward, then the rows leave the stack for good
            dta.tree_attn_bwd_segment(tree, p, t0, t1, full["q"], k, v, o, lse, full["do"], dq,
                                      dk_acc, dv_acc, ws)
            dk_out[t0:t1] = dk_acc[t0:t1]
            dv_out[t0:t1] = dv_acc[t0:t1]
            k[t0:t1] = nan
            v[t0:t1] = nan
    torch.cuda.synchronize()
    res = {n: x.double().cpu().numpy() for n, x in
           dict(o=o, lse=lse, dq=dq, dk=dk_out, dv=dv_out).items()}
    tree.destroy()
    return res


def _compare(parent, seg, Hq, Hkv, d, dtype, seed, chunk_block=0):
    T = int(np.sum(seg))
    scale = 1.0 / math.sqrt(d)
    inp = make_inputs_numpy(T, Hq, Hkv, d, seed, dtype=dtype)
    ref = X.vanilla_dta(parent, seg, inp["q"], inp["k"], inp["v"], inp["do"], scale, chunk_block=chunk_block)
    got = _run_executor(parent, seg, inp, Hq, Hkv, d, scale, dtype, ref["trace"])
    errs = {n: rel_err(got[n], ref[r]) for n, r in
            (("o", "O"), ("lse", "LSE"), ("dq", "dQ"), ("dk", "dK"), ("dv", "dV"))}
    print(f"T={T} nodes={len(parent)} Hq={Hq} Hkv={Hkv} d={d} {dtype} block={chunk_block} "
          f"calls={len(ref['trace'])}: " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    for name, e in errs.items():
        assert e <= TOL[dtype], (name, e)
    return got


def test_config1_fp32_push_pop():
    parent, seg, info = config_tree(1)
    h = config_heads(1)
    _compare(parent, seg, h["n_q_heads"], h["n_kv_heads"], h["head_dim"], "f32", info["tensor_seed"])
    _compare(parent, seg, h["n_q_heads"], h["n_kv_heads"], h["head_dim"], "f32", info["tensor_seed"],
             chunk_block=24)


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 2, 2), (128, 4, 1), (64, 6, 2)])
def test_fp32_random_forests_push_pop(d, Hq, Hkv):
    rng = np.random.default_rng(4321 + d + Hq)
    for trial in range(2):
        parent, seg = random_tree(rng, int(rng.integers(1, 25)), 90, n_roots=int(rng.integers(1, 3)))
        _compare(parent, seg, Hq, Hkv, d, "f32", seed=trial, chunk_block=(0, 37)[trial])


@pytest.mark.parametrize("Hq,Hkv,d", [(4, 1, 128), (8, 2, 128), (16, 2, 128), (3, 1, 128), (8, 2, 64), (3, 1, 64)])
def test_bf16_random_forests_push_pop(Hq, Hkv, d):
    rng = np.random.default_rng(987 + Hq)
    for trial in range(2):
        parent, seg = random_tree(rng, int(rng.integers(2, 16)), 400, n_roots=int(rng.integers(1, 3)))
        _compare(parent, seg, Hq, Hkv, d, "bf16", seed=trial, chunk_block=(0, 150)[trial])


def test_bf16_chain_with_chunked_pops_is_chunked_causal_attention():
    """One long chain popped in chunks: the paper's chunked backpropagation of a
    long suffix (several tiles, ragged chunk sizes)."""
    parent, seg = chain_tree([700, 333, 1100])
    _compare(parent, seg, 8, 2, 128, "bf16", seed=5, chunk_block=257)
    _compare(parent, seg, 4, 4, 64, "f32", seed=6, chunk_block=129)


def test_segment_calls_agree_with_the_whole_tree_call():
    """Same tree, same inputs: the accumulated push/pop result and the one-launch
    result are two evaluations of the same sums (compared to each other within
    twice the bf16 tolerance, dQ / O / LSE rows bit for bit in fp32 mode where
    both run the same arithmetic per row)."""
    rng = np.random.default_rng(31)
    parent, seg = random_tree(rng, 12, 300)
    T, Hq, Hkv, d = int(np.sum(seg)), 8, 2, 128
    scale = 1.0 / math.sqrt(d)
    inp = make_inputs_numpy(T, Hq, Hkv, d, 3, dtype="bf16")
    trace = X.vanilla_dta(parent, seg, *(np.zeros_like(inp[n]) for n in ("q", "k", "v", "do")), scale)["trace"]
    got = _run_executor(parent, seg, inp, Hq, Hkv, d, scale, "bf16", trace)
    from parity_util import run_hip
    one = run_hip(parent, seg, inp, Hq, Hkv, d, scale, "bf16")
    assert rel_err(got["o"], one["o"]) <= 2e-2 and rel_err(got["lse"], one["lse"]) <= 1e-5
    for n in ("dq", "dk", "dv"):
        assert rel_err(got[n], one[n]) <= 2e-2, n


def test_segment_argument_errors():
    parent, seg = chain_tree([40, 24])
    T = 64
    tree = dta.tree_build(parent, seg)
    p = dta.AttnParams(2, 1, 64, 0.125, dta.F32)
    z = lambda *s: torch.zeros(*s, dtype=torch.float32, device="cuda")
    q, k, v, o, lse = z(T, 2, 64), z(T, 1, 64), z(T, 1, 64), z(T, 2, 64), z(T, 2)
    for t0, t1 in ((30, 50), (-1, 10), (10, 10), (20, 10), (50, 65)):     # two nodes, out of range, empty
        with pytest.raises(dta.DtaError) as err:
            dta.tree_attn_fwd_segment(tree, p, t0, t1, q, k, v, o, lse)
        assert err.value.status == -1
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(dta.DtaError) as err:
        dta.tree_attn_bwd_segment(tree, p, 0, 40, q, k, v, o, lse, q, z(T, 2, 64), z(T, 1, 64), z(T, 1, 64), ws)
    assert err.value.status == -6                                            # workspace too small
    dta.tree_attn_fwd_segment(tree, p, 40, 64, q, k, v, o, lse)              # a valid call still works
    torch.cuda.synchronize()
    tree.destroy()


def test_back_to_back_trees_without_synchronisation():
    """Several trees run one after another on the stream, each destroyed right
    after its last call and none synchronised in between (the next tree's
    metadata is uploaded while the previous tree's kernels are still queued):
    every tree's results must equal those of the same tree run alone."""
    rng = np.random.default_rng(77)
    Hq, Hkv, d = 8, 2, 128
    scale = 1.0 / math.sqrt(d)
    p = dta.AttnParams(Hq, Hkv, d, float(scale), dta.BF16)
    jobs = []
    for i in range(4):
        parent, seg = random_tree(rng, 10 + i, 260)
        T = int(np.sum(seg))
        inp = make_inputs_numpy(T, Hq, Hkv, d, 50 + i, dtype="bf16")
        t = {n: torch.from_numpy(a).cuda().to(torch.bfloat16).contiguous() for n, a in inp.items()}
        trace = X.vanilla_dta(parent, seg, *(np.zeros((T, h, 2)) for h in (Hq, Hkv, Hkv, Hq)), scale)["trace"]
        jobs.append((parent, seg, T, t, trace))

    def run(job, sync):
        parent, seg, T, t, trace = job
        tree = dta.tree_build(parent, seg)
        o = torch.zeros_like(t["q"])
        lse = torch.zeros((T, Hq), dtype=torch.float32, device="cuda")
        dq = torch.zeros_like(t["q"])
        dk = torch.zeros((T, Hkv, d), dtype=torch.float32, device="cuda")
        dv = torch.zeros_like(dk)
        ws = torch.empty(max(256, dta.workspace_bytes(tree, p, True)), dtype=torch.uint8, device="cuda")
        for tag, node, t0, t1 in trace:
            if tag == "FWD":
                dta.tree_attn_fwd_segment(tree, p, t0, t1, t["q"], t["k"], t["v"], o, lse)
            else:
                dta.tree_attn_bwd_segment(tree, p, t0, t1, t["q"], t["k"], t["v"], o, lse, t["do"], dq, dk, dv, ws)
        if sync:
            torch.cuda.synchronize()
        tree.destroy()
        return o, lse, dq, dk, dv

    alone = [run(j, True) for j in jobs]
    for rep in range(3):
        together = [run(j, False) for j in jobs]
        torch.cuda.synchronize()
        for a, b in zip(alone, together):
            for x, y in zip(a, b):
                assert torch.equal(x, y)


@pytest.mark.parametrize("dtype,d,block", [("f32", 64, 0), ("f32", 64, 50), ("bf16", 128, 0), ("bf16", 128, 200)])
def test_leaf_order_plan_reproduces_the_whole_tree_results(dtype, d, block):
    """The calls of dta_tree_plan (the paper's leaf-order schedule with chunked
    pops), issued in order on zeroed accumulators, against the rollout-expansion
    oracle."""
    from oracle import dense_rollout as A
    rng = np.random.default_rng(55 + block)
    parent, seg = random_tree(rng, 14, 300 if dtype == "bf16" else 90, n_roots=2)
    T, Hq, Hkv = int(np.sum(seg)), 8, 2
    scale = 1.0 / math.sqrt(d)
    inp = make_inputs_numpy(T, Hq, Hkv, d, 9, dtype=dtype)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    t = {n: torch.from_numpy(a).cuda().to(tdt).contiguous() for n, a in inp.items()}
    tree = dta.tree_build(parent, seg)
    p = dta.AttnParams(Hq, Hkv, d, float(scale), dta.F32 if dtype == "f32" else dta.BF16)
    plan = dta.tree_plan(tree, block)
    nan = float("nan")
    o = torch.full_like(t["q"], nan)
    lse = torch.full((T, Hq), nan, dtype=torch.float32, device="cuda")
    dq = torch.full_like(t["q"], nan)
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
    O, LSE = A.forward(parent, seg, inp["q"], inp["k"], inp["v"], scale)
    dQ, dK, dV = A.backward(parent, seg, inp["q"], inp["k"], inp["v"], inp["do"], scale)
    got = dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)
    for name, ref in (("o", O), ("lse", LSE), ("dq", dQ), ("dk", dK), ("dv", dV)):
        e = rel_err(got[name].double().cpu().numpy(), ref)
        assert e <= TOL[dtype], (name, e)


def test_plan_captured_in_a_graph_replays_to_the_eager_result():
    """An executor that issues hundreds of small segment calls is bound by launch
    overhead; once the tree's segment schedules are resident (after one eager
    pass) the calls only enqueue kernels, so the whole sequence can be captured
    in a HIP graph.  Every replay, with eager work and synchronisation between
    the replays, must reproduce the eager pass bit for bit."""
    rng = np.random.default_rng(77)
    parent, seg = random_tree(rng, 12, 260, n_roots=2)
    T, Hq, Hkv, d = int(np.sum(seg)), 8, 2, 128
    inp = make_inputs_numpy(T, Hq, Hkv, d, 5, dtype="bf16")
    t = {n: torch.from_numpy(a).cuda().to(torch.bfloat16).contiguous() for n, a in inp.items()}
    tree = dta.tree_build(parent, seg)
    p = dta.AttnParams(Hq, Hkv, d, 1.0 / math.sqrt(d), dta.BF16)
    calls = dta.tree_plan(tree, 128)["calls"]
    o = torch.empty_like(t["q"])
    lse = torch.empty((T, Hq), dtype=torch.float32, device="cuda")
    dq = torch.empty_like(t["q"])
    dk = torch.empty((T, Hkv, d), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    ws = torch.empty(max(256, dta.workspace_bytes(tree, p, True)), dtype=torch.uint8, device="cuda")
    outs = (o, lse, dq, dk, dv)

    def run():
        dk.zero_()
        dv.zero_()
        for op, node, t0, t1 in calls:
            if op == dta.OP_BWD:
                dta.tree_attn_bwd_segment(tree, p, t0, t1, t["q"], t["k"], t["v"], o, lse, t["do"], dq, dk, dv, ws)
            else:
                dta.tree_attn_fwd_segment(tree, p, t0, t1, t["q"], t["k"], t["v"], o, lse)

    run()                                   # eager: builds and uploads every segment schedule
    torch.cuda.synchronize()
    want = [x.clone() for x in outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        for x in outs:
            x.fill_(float("nan"))           # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for x, w in zip(outs, want):
            assert torch.equal(x, w), rep
    del graph
    tree.destroy()
