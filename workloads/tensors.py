"""Seeded Q, K, V, dO tensors: i.i.d. N(0,1), one row per unique tree token in
the packed DFS order.  No attention arithmetic lives here."""
from __future__ import annotations

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even) and return them
    as fp32.  This is input preparation: both the GPU path and the oracle start
    from the already rounded values, so quantising the inputs is not counted as
    kernel error."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def make_inputs_numpy(n_tokens: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                      seed: int, dtype: str = "f32", with_do: bool = True):
    """Return dict(q,k,v,do) of fp32 numpy arrays, shapes [T,Hq,d] / [T,Hkv,d].
    With dtype == 'bf16' the values are already rounded to bfloat16."""
    rng = np.random.default_rng(seed)
    out = {}
    shapes = {"q": (n_tokens, n_q_heads, head_dim), "k": (n_tokens, n_kv_heads, head_dim),
              "v": (n_tokens, n_kv_heads, head_dim)}
    if with_do:
        shapes["do"] = (n_tokens, n_q_heads, head_dim)
    for name, shp in shapes.items():
        a = rng.standard_normal(size=shp, dtype=np.float32)
        out[name] = round_to_bf16(a) if dtype == "bf16" else a
    return out
