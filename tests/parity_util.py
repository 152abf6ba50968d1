"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI
binding and compare with the CPU oracle on the same seeded inputs."""
import numpy as np


def rel_err(x, ref):
    """max|x - ref| / max|ref| over the entries where ref is defined (not NaN).
    A reference that is identically zero up to fp64 rounding (the gradients of
    a one-token tree, where dS = p (dP - D) vanishes) is compared absolutely."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    ok = ~np.isnan(ref)
    if not ok.any():
        return 0.0
    if np.isnan(x[ok]).any():
        return float("inf")
    scale = np.abs(ref[ok]).max()
    if scale < 1e-12:
        scale = 1.0
    return float(np.abs(x[ok] - ref[ok]).max() / scale)


def run_hip(parent, seg_len, inp, n_q_heads, n_kv_heads, head_dim, scale, dtype, backward=True):
    """inp: dict of fp32 numpy arrays q,k,v,do in packed order (already rounded
    to the working dtype).  Returns numpy fp64 arrays from the HIP path."""
    import torch
    import paper_2602_00482_amd as dta

    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    dev = torch.device("cuda:0")
    t = {n: torch.from_numpy(a).to(dev).to(tdt).contiguous() for n, a in inp.items()}
    tree = dta.tree_build(parent, seg_len)
    p = dta.AttnParams(n_q_heads, n_kv_heads, head_dim, float(scale), dta.F32 if dtype == "f32" else dta.BF16)
    o, lse = dta.tree_attn_fwd(tree, p, t["q"], t["k"], t["v"])
    out = {"o": o, "lse": lse}
    if backward:
        dq, dk, dv = dta.tree_attn_bwd(tree, p, t["q"], t["k"], t["v"], o, lse, t["do"])
        out.update(dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    res = {n: x.double().cpu().numpy() for n, x in out.items()}
    tree.destroy()
    return res
