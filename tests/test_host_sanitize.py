"""The pure-host sources of the library (tree metadata and tile schedules, the
leaf-order plan, the rollout prefix tree and its partitioning) built with
-fsanitize=address,undefined and driven over random and malformed inputs.  The
sanitizers abort on any out-of-bounds access, use after free, leak, signed
overflow or misaligned access; what the driver prints is compared, line by
line, with the answers of the regular library through the C ABI."""
import os
import shutil
import subprocess
import tempfile

import numpy as np
import pytest

import paper_2602_00482_amd as dta
from workloads import config_tree, random_tree

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_00482_amd", "csrc")

CFGS = [(8, 2, 128, dta.BF16), (64, 8, 128, dta.BF16), (4, 4, 64, dta.F32), (3, 1, 128, dta.BF16),
        (4, 3, 128, dta.BF16), (4, 2, 96, dta.F32)]          # the last two are refused
BLOCKS = [0, 7, 64]


@pytest.fixture(scope="module")
def driver():
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    out = os.path.join(tempfile.mkdtemp(prefix="dta_sanitize_"), "driver")
    cmd = [gxx, "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp")] + \
          [os.path.join(CSRC, f) for f in ("dta_tree.cpp", "dta_plan.cpp", "dta_rollouts.cpp")] + ["-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    yield out
    shutil.rmtree(os.path.dirname(out), ignore_errors=True)


def _line(name, values):
    return " ".join([name] + [str(int(v)) for v in values])


def _expected_tree(parent, seg):
    try:
        tree = dta.tree_build(parent, seg)
    except dta.DtaError as e:
        return [f"build {e.status}"]
    out = ["build 0"]
    info, lay = tree.info(), tree.layout()
    out.append(_line("info", info.values()))
    for name in ("dfs_order", "node_offset", "subtree_tokens", "anc_ptr", "anc_seg_off", "anc_seg_len", "token_kend"):
        out.append(_line(name, lay[name]))
    for Hq, Hkv, d, dt in CFGS:
        try:
            si = tree.schedule_info(dta.AttnParams(Hq, Hkv, d, 0.125, dt))
            out.append(_line("schedule 0", si.values()))
        except dta.DtaError as e:
            out.append(f"schedule {e.status}")
    for b in BLOCKS:
        plan = dta.tree_plan(tree, b)
        out.append("plan 0")
        out.append(_line("leaf_order", plan["leaf_order"]))
        out.append(_line("ops", [x for op in plan["ops"] for x in op]))
        out.append(_line("calls", [x for c in plan["calls"] for x in c]))
        out.append(_line("call_ptr", plan["call_ptr"]))
    tree.destroy()
    return out


def _expected_seqs(seqs, ks):
    r = dta.Rollouts(seqs)
    v = r.view()
    out = ["rollouts 0"] + [_line(n, v[n]) for n in ("parent", "seg_len", "tokens", "seq_node", "order", "lcp")]
    for k in ks:
        try:
            gb, gc = r.partition(k)
            out += ["partition 0", _line("group_begin", gb), _line("group_cost", gc)]
        except dta.DtaError as e:
            out.append(f"partition {e.status}")
    r.destroy()
    return out


def test_host_sources_under_address_and_undefined_behaviour_sanitizers(driver):
    rng = np.random.default_rng(2024)
    text, expected = [], []
    trees = [random_tree(rng, int(rng.integers(1, 40)), int(rng.integers(1, 200)), n_roots=int(rng.integers(1, 4)))
             for _ in range(25)]
    trees += [config_tree(c)[:2] for c in (1, 2, 3)]
    trees += [([-1], [1]), ([-1, 0, 1, 2], [1, 1, 1, 1]), ([-1, -1, -1], [129, 1, 64])]
    # malformed: parent out of range, self parent, cycle, empty segment, token count overflow
    trees += [([-1, 5], [1, 1]), ([-1, 1], [1, 1]), ([-1, 2, 1], [1, 1, 1]), ([-1, 0], [1, 0]),
              ([-1, 0], [2 ** 31 - 1, 2 ** 31 - 1])]
    for parent, seg in trees:
        parent, seg = [int(x) for x in parent], [int(x) for x in seg]
        text.append(" ".join(map(str, ["tree", len(parent)] + parent + seg + [len(CFGS)] +
                                 [x for c in CFGS for x in c] + [len(BLOCKS)] + BLOCKS)))
        expected += _expected_tree(parent, seg)
    for _ in range(20):
        n = int(rng.integers(1, 30))
        seqs = []
        for _ in range(n):
            base = list(seqs[int(rng.integers(0, len(seqs)))]) if seqs and rng.random() < 0.7 else []
            cut = int(rng.integers(0, len(base) + 1))
            seqs.append(base[:cut] + [int(x) for x in rng.integers(0, 4, size=int(rng.integers(1 if cut == 0 else 0, 12)))])
            if not seqs[-1]:
                seqs[-1] = [0]
        ks = [0, 1, max(1, n // 2), n, n + 1]
        text.append(" ".join(map(str, ["seqs", n] + [x for s in seqs for x in [len(s)] + s] + [len(ks)] + ks)))
        expected += _expected_seqs(seqs, ks)
    res = subprocess.run([driver], input="\n".join(text) + "\n", capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-4000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
    got = [l.rstrip() for l in res.stdout.splitlines() if not l.startswith("segment_items")]
    assert len(got) == len(expected)
    for i, (a, b) in enumerate(zip(got, expected)):
        assert a == b, (i, a[:200], b[:200])
