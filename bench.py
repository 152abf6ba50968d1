#!/usr/bin/env python3
"""Benchmark of the tree-attention hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic rollout tree:
dta_tree_build (host metadata + tile schedule + upload) -> dta_tree_attn_fwd ->
dta_tree_attn_bwd, with Q, K, V, dO already resident in HBM.  The reported value
is useful TFLOP/s counting only unique (query, visible key) pairs:
pairs * Hq * 14 * head_dim flop per step (4d forward, 10d backward).

Prints ONE JSON line.  Also measured, inside the same line: per-kernel times
(HIP events on the launch stream) and the roofline of the slowest kernel; the
same library on the dense-expanded forest (every rollout a single chain), for
rollout tokens/s tree vs dense; the fp64 CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

WORKLOAD_NAMES = {
    1: "cfg1_tiny_fp32_tree",
    2: "cfg2_grpo_single_prompt_tree",
    3: "cfg3_multi_turn_agent_forest",
    4: "cfg4_deep_long_context_tree",
    5: "cfg5_large_mixed_forest",
    # low-compression settings (paper appendix, throughput under low compression rates)
    6: "cfg6_low_compression_short_shared_prefix",
    7: "cfg7_low_compression_short_prompt_8_answers",
    8: "cfg8_low_compression_16k_answers",
}
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
# Matrix products each launch ISSUES per unique pair and q head, in units of head_dim.  The
# forward's 4d are also its algorithmic work; the two backward launches issue 6d + 8d = 14d
# for an algorithmic 10d, because the scores and dP are recomputed in both.
KERNEL_FLOP_D = {"fwd": 4, "dq": 6, "dkdv": 8}
ALGORITHMIC_FLOP_D = {"fwd": 4, "bwd": 10}


def committed_traffic_bytes(workload):
    """HBM-side bytes per launch (read + written past the L2) of each kernel on this
    workload, from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary
    profiles/<workload>_hbm_traffic.md (line `traffic_bytes_per_launch: fwd=.. dq=.. dkdv=..`).
    Counters cannot be read from inside a timed run, so this is not measured live; None
    when there is no summary for the workload."""
    import re
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*fwd=(\S+)\s+dq=(\S+)\s+dkdv=(\S+)", text)
    return None if m is None else {"fwd": float(m.group(1)), "dq": float(m.group(2)), "dkdv": float(m.group(3))}


def _device_inputs(T, Hq, Hkv, d, seed, dtype):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    mk = lambda h: torch.randn((T, h, d), generator=g, device="cuda", dtype=torch.float32).to(tdt)
    return dict(q=mk(Hq), k=mk(Hkv), v=mk(Hkv), do=mk(Hq))


class Runner:
    """Holds device buffers for one tree shape and runs steps on them."""

    def __init__(self, parent, seg, heads, seed):
        import torch
        import paper_2602_00482_amd as dta
        self.dta, self.torch = dta, torch
        self.parent, self.seg = parent, seg
        self.T = int(np.sum(seg))
        self.Hq, self.Hkv, self.d = heads["n_q_heads"], heads["n_kv_heads"], heads["head_dim"]
        self.dtype = heads["dtype"]
        self.params = dta.AttnParams(self.Hq, self.Hkv, self.d, 1.0 / math.sqrt(self.d),
                                     dta.F32 if self.dtype == "f32" else dta.BF16)
        x = _device_inputs(self.T, self.Hq, self.Hkv, self.d, seed, self.dtype)
        self.q, self.k, self.v, self.do = x["q"], x["k"], x["v"], x["do"]
        self.o = torch.empty_like(self.q)
        self.lse = torch.empty((self.T, self.Hq), dtype=torch.float32, device="cuda")
        self.dq = torch.empty_like(self.q)
        self.dk = torch.empty_like(self.k)
        self.dv = torch.empty_like(self.v)
        tree = dta.tree_build(parent, seg)
        self.ws = torch.empty(max(256, dta.workspace_bytes(tree, self.params, True)), dtype=torch.uint8,
                              device="cuda")
        tree.destroy()

    def step(self):
        dta = self.dta
        tree = dta.tree_build(self.parent, self.seg)
        tree.prepare(self.params)
        dta.tree_attn_fwd(tree, self.params, self.q, self.k, self.v, self.o, self.lse, self.ws)
        dta.tree_attn_bwd(tree, self.params, self.q, self.k, self.v, self.o, self.lse, self.do,
                          self.dq, self.dk, self.dv, self.ws)
        return tree

    def push_pop_order(self):
        """Calls of the paper's vanilla push / pop traversal (section 3.1): one
        forward per node when it is pushed, one backward when it is popped.
        [('F'|'B', t_begin, t_end)] in packed token coordinates."""
        tree = self.dta.tree_build(self.parent, self.seg)
        lay = tree.layout()
        tree.destroy()
        off = lay["node_offset"]
        kids = [[] for _ in self.parent]
        roots = []
        for u, p in enumerate(self.parent):
            (roots if p < 0 else kids[int(p)]).append(u)
        calls, stack = [], [(r, False) for r in reversed(roots)]
        while stack:
            u, done = stack.pop()
            rng = (int(off[u]), int(off[u]) + int(self.seg[u]))
            if done:
                calls.append(("B",) + rng)
                continue
            calls.append(("F",) + rng)
            stack.append((u, True))
            stack.extend((c, False) for c in reversed(kids[u]))
        return calls

    def step_segments(self, calls, tree=None):
        """The same work as step(), issued segment by segment in push / pop order."""
        dta = self.dta
        tree = dta.tree_build(self.parent, self.seg) if tree is None else tree
        self.dk_acc.zero_()
        self.dv_acc.zero_()
        for tag, t0, t1 in calls:
            if tag == "F":
                dta.tree_attn_fwd_segment(tree, self.params, t0, t1, self.q, self.k, self.v, self.o, self.lse)
            else:
                dta.tree_attn_bwd_segment(tree, self.params, t0, t1, self.q, self.k, self.v, self.o,
                                          self.lse, self.do, self.dq, self.dk_acc, self.dv_acc, self.ws)
        return tree

    def leaf_order_calls(self, block):
        """Calls of the paper's optimised leaf-order schedule with pops chunked at
        `block` tokens (dta_tree_plan); recomputing and anchor forwards included."""
        tree = self.dta.tree_build(self.parent, self.seg)
        plan = self.dta.tree_plan(tree, block)
        tree.destroy()
        return [("B" if op == self.dta.OP_BWD else "F", t0, t1) for op, _, t0, t1 in plan["calls"]]

    def time_segment_steps(self, steps, warmup, calls=None):
        torch = self.torch
        self.dk_acc = torch.empty(self.k.shape, dtype=torch.float32, device="cuda")
        self.dv_acc = torch.empty_like(self.dk_acc)
        calls = self.push_pop_order() if calls is None else calls
        for _ in range(warmup):
            self.step_segments(calls).destroy()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step_segments(calls).destroy()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / steps
        del self.dk_acc, self.dv_acc
        return sec, len(calls)

    def time_segment_graph(self, steps, calls=None):
        """The same call sequence on ONE tree, captured in a HIP graph after an eager
        pass (which builds and uploads the segment schedules) and replayed: what an
        executor pays when the layers of a model reuse the step's tree.  Returns
        seconds per replay, or None if capture is not available."""
        torch = self.torch
        self.dk_acc = torch.empty(self.k.shape, dtype=torch.float32, device="cuda")
        self.dv_acc = torch.empty_like(self.dk_acc)
        calls = self.push_pop_order() if calls is None else calls
        tree = self.dta.tree_build(self.parent, self.seg)
        sec = None
        try:
            self.step_segments(calls, tree)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                self.step_segments(calls, tree)
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            torch.cuda.synchronize()
            sec = (time.perf_counter() - t0) / steps
            del graph
        except RuntimeError as e:
            print(f"bench.py: graph capture of the segment calls failed: {e}", file=sys.stderr)
        tree.destroy()
        del self.dk_acc, self.dv_acc
        return sec

    def time_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step().destroy()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        # destroy() does not block (the device copies are released behind the
        # kernels), so the host part of a step (tree build, schedule, metadata
        # upload) runs while the previous step's kernels execute, as it would in
        # a training loop
        for _ in range(steps):
            self.step().destroy()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def time_tree_build(self, reps=15):
        """Host side of a step on an idle GPU: dta_tree_build, then the tile schedule
        and the metadata upload (dta_tree_attn_prepare).  Median and min, in ms."""
        dta, torch = self.dta, self.torch
        torch.cuda.synchronize()
        b, p = [], []
        for _ in range(reps):
            t0 = time.perf_counter()
            tree = dta.tree_build(self.parent, self.seg)
            t1 = time.perf_counter()
            tree.prepare(self.params)
            t2 = time.perf_counter()
            tree.destroy()
            b.append((t1 - t0) * 1e3)
            p.append((t2 - t1) * 1e3)
        return {"tree_build_ms": {"median": float(np.median(b)), "min": float(np.min(b))},
                "schedule_and_upload_ms": {"median": float(np.median(p)), "min": float(np.min(p))}}

    def time_kernels(self, iters, with_power=False):
        """Average duration of each launch, HIP events on the launch stream."""
        dta, torch = self.dta, self.torch
        tree = dta.tree_build(self.parent, self.seg)
        tree.prepare(self.params)
        a = (tree, self.params, self.q, self.k, self.v, self.o, self.lse, self.do,
             self.dq, self.dk, self.dv, self.ws)
        launches = {
            "fwd": lambda: dta.tree_attn_fwd(tree, self.params, self.q, self.k, self.v, self.o, self.lse, self.ws),
            # as the step issues it: the dQ launch also computes the row statistics D = dO.O
            "dq": lambda: dta.tree_attn_bwd(*a, stages=dta.BWD_DELTA | dta.BWD_DQ),
            "dkdv": lambda: dta.tree_attn_bwd(*a, stages=dta.BWD_DKDV),
        }
        out, out_min, power = {}, {}, {}
        sampler = PowerSampler(period=0.15) if with_power else None
        if sampler:
            sampler.__enter__()
        for name, fn in launches.items():
            fn()
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
            t0 = time.time()
            ev[0].record()
            for i in range(iters):
                fn()
                ev[i + 1].record()
            torch.cuda.synchronize()
            t1 = time.time()
            out[name] = ev[0].elapsed_time(ev[iters]) / iters
            out_min[name] = min(ev[i].elapsed_time(ev[i + 1]) for i in range(iters))
            if sampler:
                power[name] = (t0 + 0.25 * (t1 - t0), t1)
        if sampler:
            sampler.__exit__()
            power = {k: sampler.summary(*v) for k, v in power.items()}
        self.kernel_ms_min = out_min
        self.kernel_power = power if with_power else None
        info = tree.info()
        sched = tree.schedule_info(self.params)
        tree.destroy()
        return out, info, sched


class PowerSampler:
    """Polls `rocm-smi -a` in a thread while the GPU works: socket power, the package
    power limit, the accumulated time the power limiter was active, and the shader
    clock of each XCD.  What it returns says whether the kernels ran at the power limit
    (they do: the published peak assumes 2.4 GHz, the chip settles at 1.6-1.9 GHz)."""

    KEYS = ("current_socket_power", "ppt_residency_acc", "current_gfxclk")

    def __init__(self, period=0.25):
        import threading
        self.samples, self.period, self.stop = [], period, False
        self.thread = threading.Thread(target=self._run, daemon=True)

    def _poll(self):
        import subprocess
        try:
            out = subprocess.run(["/opt/rocm/bin/rocm-smi", "-a"], capture_output=True, text=True, timeout=5).stdout
        except Exception:
            return None
        d = {}
        for line in out.splitlines():
            for key in self.KEYS + ("Max Graphics Package Power",):
                if key in line and "XCP" not in line:
                    d[key] = line.split(":")[-1].strip()
        return d or None

    def _run(self):
        while not self.stop:
            d = self._poll()
            if d:
                self.samples.append((time.time(), d))
            time.sleep(self.period)

    def __enter__(self):
        self.thread.start()
        return self

    def __exit__(self, *a):
        self.stop = True
        self.thread.join(timeout=10)

    def summary(self, t0, t1):
        sel = [d for t, d in self.samples if t0 <= t <= t1]
        if not sel:
            return None
        try:
            power = [float(d["current_socket_power"]) for d in sel if "current_socket_power" in d]
            clocks = [[float(x) for x in d["current_gfxclk"].strip("[]").split(",")] for d in sel if "current_gfxclk" in d]
            ppt = [int(d["ppt_residency_acc"]) for d in sel if "ppt_residency_acc" in d]
            cap = next((float(d["Max Graphics Package Power"]) for d in sel if "Max Graphics Package Power" in d), None)
            mean_clk = [sum(c[i] for c in clocks) / len(clocks) for i in range(len(clocks[0]))] if clocks else None
            return {"samples": len(sel), "socket_power_w_mean": sum(power) / len(power) if power else None,
                    "socket_power_w_max": max(power) if power else None, "package_power_limit_w": cap,
                    "power_limiter_active_count_delta": (ppt[-1] - ppt[0]) if len(ppt) > 1 else None,
                    "shader_clock_mhz_per_xcd": None if mean_clk is None else [round(c) for c in mean_clk],
                    "shader_clock_mhz_min_over_mean": None if mean_clk is None else min(mean_clk) / (sum(mean_clk) / len(mean_clk))}
        except Exception as e:
            return {"error": str(e)}


def _dense_batches(rollout_lens, token_budget):
    batches, cur, tot = [], [], 0
    for n in rollout_lens:
        if cur and tot + n > token_budget:
            batches.append(cur)
            cur, tot = [], 0
        cur.append(int(n))
        tot += int(n)
    if cur:
        batches.append(cur)
    return batches


def run_dense(rollout_lens, heads, steps, warmup, token_budget=393216):
    """The same library on the dense-expanded forest: every rollout is its own
    single-node tree (ordinary variable-length causal attention)."""
    import torch
    total = 0.0
    shapes_done = {}
    for batch in _dense_batches(rollout_lens, token_budget):
        key = tuple(batch)
        if key not in shapes_done:
            r = Runner(np.full(len(batch), -1, dtype=np.int32), np.asarray(batch, dtype=np.int32), heads, seed=7)
            shapes_done[key] = r.time_steps(steps, warmup)
            del r
            torch.cuda.empty_cache()
        total += shapes_done[key]
    return total


def mfma_sustained_rate():
    """Rate the bf16 matrix pipes sustain with nothing else in the way (the
    library's probe kernel: same instruction and block shape as the attention
    kernels, register operands), and the shader clock during that run."""
    import torch
    from paper_2602_00482_amd import probe
    n_blocks, iters = 512, 20000          # two blocks on each of 256 CUs, about 10 ms
    out = torch.empty(n_blocks * 256, dtype=torch.float32, device="cuda")
    ticks = torch.zeros(2 * n_blocks, dtype=torch.int64, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    best = None
    for rep in range(4):                  # first one warms up; the power state settles over the others
        ev[0].record()
        flop, wall_khz = probe.probe_mfma_bf16(n_blocks, iters, out, ticks)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1])
        if rep > 0 and (best is None or ms > best[0]):
            best = (ms, flop)             # the slowest = the sustained, throttled state
    t = ticks.view(n_blocks, 2).double().cpu()
    ratio = float((t[:, 0] / t[:, 1].clamp(min=1)).median())
    return {"tflops": best[1] / (best[0] * 1e-3) / 1e12, "ms": best[0],
            "shader_clock_ghz": ratio * wall_khz * 1e3 / 1e9, "wall_clock_khz": wall_khz,
            "blocks": n_blocks, "iters": iters}


def mfma_valu_overlap():
    """How much vector-ALU work the hardware hides behind another wave's matrix
    products on the same SIMD (the library's overlap probe, register work only).
    The attention kernels' time is products plus exponentials and their
    bookkeeping, so this bounds what any schedule of them can reach."""
    import torch
    from paper_2602_00482_amd import probe
    n_blocks, iters = 256, 20000          # one block of 8 waves per CU
    out = torch.empty(n_blocks * 512, dtype=torch.float32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def run(m, v):
        best = None
        for _ in range(3):
            ev[0].record()
            probe.probe_overlap(n_blocks, m, v, out)
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1])
            best = ms if best is None else min(best, ms)
        return best

    tm = run(iters, 0)
    tv = run(0, iters)
    v_iters = max(1, int(iters * tm / tv))          # same duration for both halves
    tv = run(0, v_iters)
    tb = run(iters, v_iters)
    return {"mfma_only_ms": tm, "exp_only_ms": tv, "both_ms": tb,
            "hidden_frac_of_shorter": (tm + tv - tb) / min(tm, tv), "both_over_sum": tb / (tm + tv)}


def cpu_oracle_baseline(parent, seg, heads, seed, useful_flop, budget_pairs=8.5e8):
    """Oracle A (dense per-rollout, fp64 numpy, as it stands) on a bounded sample of the
    workload, timed on this machine's host cores: whole rollouts (longest first), the q heads
    of one kv group, as many (rollout, q head) pairs as fit a budget of dense score
    entries (about 10-30 s of CPU work).  Every rollout of the sample is handed to the
    oracle as the single-chain tree of its root path, which is what the oracle expands
    the tree into anyway.  The whole job is every rollout x every q head; the measured
    time is extrapolated linearly by dense causal pairs and labelled as such."""
    from oracle import dense_rollout as A
    from oracle import tree_layout as L
    from workloads import make_inputs_numpy
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    Hq, Hkv, d = heads["n_q_heads"], heads["n_kv_heads"], heads["head_dim"]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(d)
    sd = L.start_depths(parent, seg)
    leaves = sorted(L.leaves(parent), key=lambda u: -(int(sd[u]) + int(seg[u])))
    dense_pairs_job = sum((int(sd[u]) + int(seg[u])) * (int(sd[u]) + int(seg[u]) + 1) // 2 for u in leaves) * Hq
    sample, pairs = [], 0
    for u in leaves:                                   # (leaf, number of q heads of the group)
        n = int(sd[u]) + int(seg[u])
        per_head = n * (n + 1) // 2
        nh = int(min(G, max(0, (budget_pairs - pairs) // per_head)))
        if nh == 0 and not sample:
            nh = 1                                     # at least one (rollout, head), whatever its size
        if nh == 0:
            break
        sample.append((u, nh))
        pairs += nh * per_head
    dt = 0.0
    for i, (u, nh) in enumerate(sample):
        path = L.node_path(parent, u)
        chain_parent = np.arange(-1, len(path) - 1, dtype=np.int32)
        chain_seg = np.asarray([seg[a] for a in path], dtype=np.int32)
        x = make_inputs_numpy(int(chain_seg.sum()), nh, 1, d, seed + i, dtype=heads["dtype"])
        t0 = time.perf_counter()
        A.forward(chain_parent, chain_seg, x["q"], x["k"], x["v"], scale)
        A.backward(chain_parent, chain_seg, x["q"], x["k"], x["v"], x["do"], scale)
        dt += time.perf_counter() - t0
    full = dt * dense_pairs_job / pairs
    return {"value": useful_flop / full / 1e12, "unit": "TFLOP/s", "cores": int(threads),
            "kind": "oracle",
            "sample": f"dense per-rollout fp64 oracle, fwd+bwd, {len(sample)} of {len(leaves)} rollouts (longest first) "
                      f"x {'/'.join(str(nh) for _, nh in sample)} of {Hq} q heads = {pairs:.3e} dense causal pairs: "
                      f"{dt:.1f} s measured; the whole job is {dense_pairs_job:.3e} dense pairs, extrapolated "
                      f"linearly to {full:.0f} s; value = the job's unique-pair flop / that time",
            "seconds_measured": dt, "seconds_extrapolated": full}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4,
                    help="benchmark configuration 2..8 of the main line (default: 4, the largest single-GPU one)")
    ap.add_argument("--others", type=str, default="2,3,5,6,7,8", help="configs reported as extra objects ('' = none)")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-segments", action="store_true",
                    help="skip the segment-mode measurements (used for kernel-trace profiles, whose "
                         "per-kernel averages should cover the one-launch path only)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="no timing: two steps of --config, then a plain 1 GiB device copy; the program "
                         "to run under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` (the copy "
                         "calibrates the counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_00482_amd as dta
    from workloads import config_heads, config_tree
    from paper_2602_00482_amd.build import ensure_built
    ensure_built()              # builds only if no library is there
    dta.load_library()          # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    if args.traffic_probe:
        parent, seg, meta = config_tree(args.config)
        r = Runner(parent, seg, config_heads(args.config), meta["tensor_seed"])
        for _ in range(2):
            r.step().destroy()
            torch.cuda.synchronize()
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": WORKLOAD_NAMES[args.config], "steps": 2, "copy_bytes": 1 << 30}))
        return

    def leaf_lengths(parent, seg):
        tree = dta.tree_build(parent, seg)
        lay = tree.layout()
        tree.destroy()
        is_leaf = np.ones(len(parent), dtype=bool)
        is_leaf[parent[parent >= 0]] = False
        return (lay["node_start_depth"] + seg)[is_leaf]

    def measure(cfg, steps, warmup, with_dense, with_cpu, with_segments=True, with_power=False, head_dim=None):
        parent, seg, meta = config_tree(cfg)
        heads = config_heads(cfg)
        if head_dim is not None:
            heads["head_dim"] = head_dim
        r = Runner(parent, seg, heads, meta["tensor_seed"])
        power = None
        if with_power:
            with PowerSampler() as ps:
                t0 = time.time()
                sec = r.time_steps(steps, warmup)
                t1 = time.time()
            power = ps.summary(t0 + 0.3 * (t1 - t0), t1)      # the warm-up steps are at the front
        else:
            sec = r.time_steps(steps, warmup)
        kern, info, sched = r.time_kernels(max(3, min(10, steps)), with_power=with_power)
        if with_segments:
            seg_sec, seg_calls = r.time_segment_steps(max(1, min(5, steps)), 1)
            lo_sec, lo_calls = r.time_segment_steps(max(1, min(5, steps)), 1, r.leaf_order_calls(2048))
            graph_sec = r.time_segment_graph(max(1, min(5, steps)))
        Hq, d = heads["n_q_heads"], heads["head_dim"]
        pairs = info["unique_pairs"]
        useful = pairs * Hq * 14 * d
        res = {
            "workload": WORKLOAD_NAMES[cfg], "n_tokens": info["n_tokens"], "n_nodes": info["n_nodes"],
            "n_leaves": info["n_leaves"], "max_path_tokens": info["max_path_tokens"],
            "unique_pairs": pairs, "heads": f"{Hq}q/{heads['n_kv_heads']}kv", "head_dim": d,
            "tree_seed": meta["tree_seed"], "tensor_seed": meta["tensor_seed"],
            "ms_per_step": sec * 1e3, "useful_tflops": useful / sec / 1e12,
            "mfma_frac_of_peak": useful / sec / 1e12 / PEAK_TFLOPS[heads["dtype"]],
            "kernel_ms": {k: round(v, 4) for k, v in kern.items()},
            "kernel_ms_min": {k: round(v, 4) for k, v in r.kernel_ms_min.items()},
            "host": dict(r.time_tree_build(), metadata_bytes=sched["metadata_bytes"]),
            # per launch, on the products that launch issues (fwd 4d, dq 6d, dkdv 8d) ...
            "kernel_tflops_issued": {k: pairs * Hq * KERNEL_FLOP_D[k] * d / (kern[k] * 1e-3) / 1e12
                                     for k in KERNEL_FLOP_D},
            # ... and on algorithmic work: forward 4d, the two backward launches together 10d
            "kernel_tflops_algorithmic": {
                "fwd": pairs * Hq * 4 * d / (kern["fwd"] * 1e-3) / 1e12,
                "bwd": pairs * Hq * 10 * d / ((kern["dq"] + kern["dkdv"]) * 1e-3) / 1e12},
            "schedule": sched,
            "C_leaf": info["rollout_tokens"] / info["n_tokens"],
            "C_full": info["rollout_tokens_full"] / info["n_tokens"],
            "C_attn_leaf": info["dense_pairs"] / pairs,
            "rollout_tokens_per_s_tree": info["rollout_tokens"] / sec,
        }
        if power is not None:
            res["power_and_clocks_during_timed_steps"] = power
            res["power_and_clocks_per_kernel"] = r.kernel_power
        if with_segments:
            # the same fwd+bwd issued one segment at a time in the paper's push / pop
            # order (2 calls per node, dK/dV accumulated in fp32 across calls)
            res["segment_mode"] = {"ms_per_step": seg_sec * 1e3, "calls": seg_calls,
                                   "useful_tflops": useful / seg_sec / 1e12,
                                   "slowdown_vs_one_launch": seg_sec / sec,
                                   # the same calls on one tree, captured in a HIP graph and replayed
                                   "graph_replay_ms": None if graph_sec is None else graph_sec * 1e3,
                                   # the optimised leaf-order schedule, pops chunked at 2048 tokens
                                   "leaf_order_block2048": {"ms_per_step": lo_sec * 1e3, "calls": lo_calls,
                                                            "slowdown_vs_one_launch": lo_sec / sec}}
        del r
        torch.cuda.empty_cache()
        if with_dense:
            dsec = run_dense(leaf_lengths(parent, seg), heads, steps=max(1, min(3, steps)), warmup=1)
            res["ms_per_step_dense_expanded"] = dsec * 1e3
            res["rollout_tokens_per_s_dense"] = info["rollout_tokens"] / dsec
            res["tree_over_dense"] = dsec / sec
        cpu = None
        if with_cpu:
            cpu = cpu_oracle_baseline(parent, seg, heads, meta["tensor_seed"], useful)
        return res, kern, info, heads, cpu

    main_res, kern, info, heads, cpu = measure(args.config, args.steps, args.warmup,
                                               not args.no_dense, not args.no_cpu, not args.no_segments,
                                               with_power=True)
    Hq, d = heads["n_q_heads"], heads["head_dim"]
    peak = PEAK_TFLOPS[heads["dtype"]]
    pairs_h = info["unique_pairs"] * Hq
    # The dominant launches are the backward's two (dQ, then dK/dV with the reduction of split
    # tiles), which together do the algorithmic 10d per pair and q head; the roofline is
    # priced on that, with each launch's duration (HIP events on the launch stream) and the
    # rate on the products it issues beside it.
    bwd_ms = kern["dq"] + kern["dkdv"]
    achieved = pairs_h * ALGORITHMIC_FLOP_D["bwd"] * d / (bwd_ms * 1e-3) / 1e12
    traffic = committed_traffic_bytes(main_res["workload"])
    sustained = mfma_sustained_rate()
    overlap = mfma_valu_overlap()
    per_kernel = {k: {"avg_launch_ms": kern[k], "issued_flop_per_pair_per_head": KERNEL_FLOP_D[k] * d,
                      "issued_tflops": pairs_h * KERNEL_FLOP_D[k] * d / (kern[k] * 1e-3) / 1e12,
                      "issued_frac_of_peak": pairs_h * KERNEL_FLOP_D[k] * d / (kern[k] * 1e-3) / 1e12 / peak,
                      "traffic": None if traffic is None else traffic[k]} for k in KERNEL_FLOP_D}
    per_kernel["fwd"]["algorithmic_tflops"] = per_kernel["fwd"]["issued_tflops"]
    line = {
        "metric": "tree_attn_fwd_bwd_unique_pair_tflops", "value": main_res["useful_tflops"],
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": heads["dtype"], "data": "synthetic",
        "config": {k: main_res[k] for k in ("workload", "n_tokens", "n_nodes", "n_leaves", "max_path_tokens",
                                            "unique_pairs", "heads", "head_dim", "tree_seed", "tensor_seed")},
        "roofline": {"bound": "mfma", "kernel": "bwd (dq launch + dkdv launch)", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": None if traffic is None else traffic["dq"] + traffic["dkdv"],
                     "flop_per_pair_per_head": ALGORITHMIC_FLOP_D["bwd"] * d, "avg_launch_ms": bwd_ms,
                     "per_kernel": per_kernel,
                     "whole_step_frac": main_res["mfma_frac_of_peak"],
                     # what this GPU's matrix pipes sustain on products alone (measured just now),
                     # beside the published peak that `frac` is priced against
                     "mfma_only_probe": sustained, "frac_of_probe": achieved / sustained["tflops"],
                     # one wave's products against another wave's exponentials on the same SIMD
                     "mfma_valu_overlap_probe": overlap},
        "cpu_baseline": cpu,
        "detail": main_res,
    }
    others = {}
    for c in [int(x) for x in args.others.split(",") if x.strip()]:
        if c == args.config:
            continue
        res, *_ = measure(c, max(2, min(5, args.steps)), 1, not args.no_dense, False, not args.no_segments)
        others[WORKLOAD_NAMES[c]] = res
    if others and 3 in [int(x) for x in args.others.split(",") if x.strip()]:
        # the same kernels instantiated for head_dim 64 (not a BASELINE configuration): the
        # multi-turn forest's tree with 64-wide heads, kernel times only
        res, *_ = measure(3, 3, 1, False, False, False, head_dim=64)
        others[WORKLOAD_NAMES[3] + "_head_dim_64"] = res
    if others:
        line["other_configs"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
