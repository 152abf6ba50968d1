"""MI355X-native dynamic tree attention (AReaL-DTA hot path).

Thin ctypes binding over libdta.so; every step of the path runs in the HIP
library.  Importing this package never falls back to another implementation:
if the library has not been built the binding raises.
"""
from .binding import (DtaError, Tree, AttnParams, tree_build, tree_attn_fwd, tree_attn_bwd,
                      tree_attn_fwd_segment, tree_attn_bwd_segment, tree_attn_bwd_noalloc, Rollouts, tree_plan,
                      OP_FWD, OP_REFWD, OP_BWD, OP_FWD_NOGRAD,
                      workspace_bytes, load_library, F32, BF16, exported_symbols,
                      BWD_DELTA, BWD_DQ, BWD_DKDV, BWD_ALL)

__all__ = ["DtaError", "Tree", "AttnParams", "tree_build", "tree_attn_fwd", "tree_attn_bwd",
           "tree_attn_fwd_segment", "tree_attn_bwd_segment", "tree_attn_bwd_noalloc", "Rollouts", "tree_plan",
           "OP_FWD", "OP_REFWD", "OP_BWD", "OP_FWD_NOGRAD", "workspace_bytes", "load_library", "F32", "BF16", "exported_symbols",
           "BWD_DELTA", "BWD_DQ", "BWD_DKDV", "BWD_ALL"]
