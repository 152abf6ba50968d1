"""ctypes binding for include/dta.h: argument marshalling only.

Function names mirror the C ABI (dta_tree_build -> tree_build, ...).  Tensors
are torch tensors used purely as device memory; the current torch stream is
passed to the library as the HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdta.so")
_lib = None

F32, BF16 = 0, 1

exported_symbols = [
    "dta_tree_build", "dta_tree_info", "dta_tree_layout", "dta_tree_schedule_info",
    "dta_tree_destroy", "dta_tree_attn_workspace_bytes", "dta_tree_attn_prepare",
    "dta_tree_attn_fwd", "dta_tree_attn_bwd", "dta_tree_attn_bwd_stages", "dta_tree_attn_bwd_noalloc",
    "dta_tree_attn_fwd_segment", "dta_tree_attn_bwd_segment", "dta_rollouts_build",
    "dta_rollouts_view", "dta_rollouts_destroy", "dta_rollouts_partition", "dta_tree_plan",
    "dta_plan_view", "dta_plan_destroy", "dta_status_string",
]


class DtaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = load_library().dta_status_string(status).decode()
        super().__init__(f"{where} failed: {name} ({status})")


class _TreeInfo(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "n_nodes", "n_tokens", "n_leaves", "n_roots", "max_path_tokens", "max_depth_nodes",
        "rollout_tokens", "rollout_tokens_full", "unique_pairs", "dense_pairs", "dense_pairs_full")]


class _TreeLayout(C.Structure):
    _fields_ = [("dfs_order", C.POINTER(C.c_int32)), ("node_offset", C.POINTER(C.c_int64)),
                ("node_start_depth", C.POINTER(C.c_int64)), ("subtree_tokens", C.POINTER(C.c_int64)),
                ("anc_ptr", C.POINTER(C.c_int64)), ("anc_seg_off", C.POINTER(C.c_int64)),
                ("anc_seg_len", C.POINTER(C.c_int64)), ("token_kend", C.POINTER(C.c_int32))]


class _ScheduleInfo(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "fwd_q_tile_tokens", "fwd_work_items", "fwd_tile_pairs",
        "bwd_kv_tile_tokens", "bwd_work_items", "bwd_tile_pairs", "metadata_bytes")]


class AttnParams(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("softmax_scale", C.c_float), ("dtype", C.c_int32)]


class _PlanOp(C.Structure):
    _fields_ = [("op", C.c_int32), ("leaf", C.c_int32), ("lo", C.c_int64), ("hi", C.c_int64)]


class _PlanCall(C.Structure):
    _fields_ = [("op", C.c_int32), ("node", C.c_int32), ("t_begin", C.c_int64), ("t_end", C.c_int64)]


class _PlanView(C.Structure):
    _fields_ = [("n_leaves", C.c_int32), ("leaf_order", C.POINTER(C.c_int32)), ("n_ops", C.c_int64),
                ("ops", C.POINTER(_PlanOp)), ("call_ptr", C.POINTER(C.c_int64)), ("n_calls", C.c_int64),
                ("calls", C.POINTER(_PlanCall)), ("n_fwd", C.c_int64), ("n_fwd_nograd", C.c_int64),
                ("n_chunks", C.c_int64), ("max_stack_tokens", C.c_int64)]


class _RolloutsView(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("n_nodes", C.c_int32), ("n_tokens", C.c_int64),
                ("parent", C.POINTER(C.c_int32)), ("seg_len", C.POINTER(C.c_int32)),
                ("tokens", C.POINTER(C.c_int32)), ("seq_node", C.POINTER(C.c_int32)),
                ("order", C.POINTER(C.c_int32)), ("lcp", C.POINTER(C.c_int64))]


def load_library():
    """Load libdta.so (built in-tree by build.py).  No fallback: raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} not found: run `python -m paper_2602_00482_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.dta_tree_build.argtypes = [i32p, i32p, C.c_int32, C.c_uint32, C.POINTER(vp)]
    lib.dta_tree_build.restype = C.c_int
    lib.dta_tree_info.argtypes = [vp, C.POINTER(_TreeInfo)]
    lib.dta_tree_info.restype = C.c_int
    lib.dta_tree_layout.argtypes = [vp, C.POINTER(_TreeLayout)]
    lib.dta_tree_layout.restype = C.c_int
    lib.dta_tree_schedule_info.argtypes = [vp, C.POINTER(AttnParams), C.POINTER(_ScheduleInfo)]
    lib.dta_tree_schedule_info.restype = C.c_int
    lib.dta_tree_destroy.argtypes = [vp]
    lib.dta_tree_destroy.restype = None
    lib.dta_tree_attn_workspace_bytes.argtypes = [vp, C.POINTER(AttnParams), C.c_int]
    lib.dta_tree_attn_workspace_bytes.restype = C.c_size_t
    lib.dta_tree_attn_prepare.argtypes = [vp, C.POINTER(AttnParams)]
    lib.dta_tree_attn_prepare.restype = C.c_int
    lib.dta_tree_attn_fwd.argtypes = [vp, C.POINTER(AttnParams), vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.dta_tree_attn_fwd.restype = C.c_int
    lib.dta_tree_attn_bwd.argtypes = [vp, C.POINTER(AttnParams)] + [vp] * 9 + [vp, C.c_size_t, vp]
    lib.dta_tree_attn_bwd.restype = C.c_int
    lib.dta_tree_attn_bwd_stages.argtypes = [vp, C.POINTER(AttnParams)] + [vp] * 9 + [vp, C.c_size_t, vp, C.c_uint32]
    lib.dta_tree_attn_bwd_stages.restype = C.c_int
    lib.dta_tree_attn_bwd_noalloc.argtypes = [vp, C.POINTER(AttnParams)] + [vp] * 9 + [vp]
    lib.dta_tree_attn_bwd_noalloc.restype = C.c_int
    lib.dta_tree_attn_fwd_segment.argtypes = ([vp, C.POINTER(AttnParams), C.c_int64, C.c_int64] + [vp] * 5 +
                                              [vp, C.c_size_t, vp])
    lib.dta_tree_attn_fwd_segment.restype = C.c_int
    lib.dta_tree_attn_bwd_segment.argtypes = ([vp, C.POINTER(AttnParams), C.c_int64, C.c_int64] + [vp] * 9 +
                                              [vp, C.c_size_t, vp])
    lib.dta_tree_attn_bwd_segment.restype = C.c_int
    lib.dta_rollouts_build.argtypes = [i32p, C.POINTER(C.c_int64), C.c_int32, C.POINTER(vp)]
    lib.dta_rollouts_build.restype = C.c_int
    lib.dta_rollouts_view.argtypes = [vp, C.POINTER(_RolloutsView)]
    lib.dta_rollouts_view.restype = C.c_int
    lib.dta_rollouts_destroy.argtypes = [vp]
    lib.dta_rollouts_destroy.restype = None
    lib.dta_rollouts_partition.argtypes = [vp, C.c_int32, i32p, C.POINTER(C.c_int64)]
    lib.dta_rollouts_partition.restype = C.c_int
    lib.dta_tree_plan.argtypes = [vp, C.c_int64, C.POINTER(vp)]
    lib.dta_tree_plan.restype = C.c_int
    lib.dta_plan_view.argtypes = [vp, C.POINTER(_PlanView)]
    lib.dta_plan_view.restype = C.c_int
    lib.dta_plan_destroy.argtypes = [vp]
    lib.dta_plan_destroy.restype = None
    lib.dta_status_string.argtypes = [C.c_int]
    lib.dta_status_string.restype = C.c_char_p
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        raise DtaError(status, where)


class Tree:
    """Owns a dta_tree_t*; exposes dta_tree_info / dta_tree_layout as numpy copies."""

    def __init__(self, handle, n_nodes):
        self._h = handle
        self.n_nodes = n_nodes
        # the C ABI takes no tensor sizes: the wrappers compare every tensor with this
        self.n_tokens = self.info()["n_tokens"]

    @property
    def handle(self):
        return self._h

    def info(self) -> dict:
        out = _TreeInfo()
        _check(load_library().dta_tree_info(self._h, C.byref(out)), "dta_tree_info")
        return {n: int(getattr(out, n)) for n, _ in _TreeInfo._fields_}

    def layout(self) -> dict:
        out = _TreeLayout()
        _check(load_library().dta_tree_layout(self._h, C.byref(out)), "dta_tree_layout")
        n = self.n_nodes
        T = self.info()["n_tokens"]
        anc_ptr = np.ctypeslib.as_array(out.anc_ptr, shape=(n + 1,)).copy()
        m = int(anc_ptr[-1])
        arr = lambda p, k: np.ctypeslib.as_array(p, shape=(k,)).copy() if k else np.zeros(0, dtype=np.int64)
        return dict(dfs_order=arr(out.dfs_order, n), node_offset=arr(out.node_offset, n),
                    node_start_depth=arr(out.node_start_depth, n),
                    subtree_tokens=arr(out.subtree_tokens, n), anc_ptr=anc_ptr,
                    anc_seg_off=arr(out.anc_seg_off, m), anc_seg_len=arr(out.anc_seg_len, m),
                    token_kend=arr(out.token_kend, T))

    def schedule_info(self, params: AttnParams) -> dict:
        out = _ScheduleInfo()
        _check(load_library().dta_tree_schedule_info(self._h, C.byref(params), C.byref(out)),
               "dta_tree_schedule_info")
        return {n: int(getattr(out, n)) for n, _ in _ScheduleInfo._fields_}

    def prepare(self, params: AttnParams):
        _check(load_library().dta_tree_attn_prepare(self._h, C.byref(params)), "dta_tree_attn_prepare")

    def destroy(self):
        if self._h:
            load_library().dta_tree_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tree_build(parent, seg_len, flags: int = 0) -> Tree:
    """dta_tree_build: parent[] / seg_len[] (host int32) -> Tree."""
    lib = load_library()
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    seg_len = np.ascontiguousarray(seg_len, dtype=np.int32)
    if parent.shape != seg_len.shape or parent.ndim != 1:
        raise ValueError("parent and seg_len must be 1-D arrays of equal length")
    h = C.c_void_p()
    st = lib.dta_tree_build(parent.ctypes.data_as(C.POINTER(C.c_int32)),
                            seg_len.ctypes.data_as(C.POINTER(C.c_int32)),
                            int(parent.shape[0]), int(flags), C.byref(h))
    _check(st, "dta_tree_build")
    return Tree(h, int(parent.shape[0]))


def workspace_bytes(tree: Tree, params: AttnParams, is_bwd: bool) -> int:
    return int(load_library().dta_tree_attn_workspace_bytes(tree.handle, C.byref(params), int(is_bwd)))


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check_tree_tokens(tree, q):
    """The kernels index rows 0 .. n_tokens-1 of every tensor, so tensors of another
    tree (or a stale handle) must be refused here, before any launch."""
    if tree.handle is None or not tree.handle:
        raise ValueError("the tree has been destroyed")
    if q.shape[0] != tree.n_tokens:
        raise ValueError(f"tensors have {q.shape[0]} token rows, the tree has n_tokens = {tree.n_tokens}")


def _check_workspace(workspace):
    if workspace is not None and workspace.numel() and not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous CUDA tensor")


def _check_tensor(t, name, shape, dtype):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if tuple(t.shape) != tuple(shape) or t.dtype != dtype:
        raise ValueError(f"{name}: expected {tuple(shape)} {dtype}, got {tuple(t.shape)} {t.dtype}")


def tree_attn_fwd(tree: Tree, params: AttnParams, q, k, v, o=None, lse=None, workspace=None):
    """dta_tree_attn_fwd on torch's current stream.  Returns (o, lse)."""
    import torch
    dt = torch.float32 if params.dtype == F32 else torch.bfloat16
    _check_tree_tokens(tree, q)
    T = q.shape[0]
    _check_tensor(q, "q", (T, params.n_q_heads, params.head_dim), dt)
    _check_tensor(k, "k", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(v, "v", (T, params.n_kv_heads, params.head_dim), dt)
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((T, params.n_q_heads), dtype=torch.float32, device=q.device)
    _check_tensor(o, "o", q.shape, dt)
    _check_tensor(lse, "lse", (T, params.n_q_heads), torch.float32)
    if workspace is None:
        need = workspace_bytes(tree, params, False)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    _check_workspace(workspace)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = load_library().dta_tree_attn_fwd(tree.handle, C.byref(params), _ptr(q), _ptr(k), _ptr(v),
                                          _ptr(o), _ptr(lse), _ptr(workspace), ws_bytes, _stream())
    _check(st, "dta_tree_attn_fwd")
    return o, lse


BWD_DELTA, BWD_DQ, BWD_DKDV, BWD_ALL = 1, 2, 4, 7


def tree_attn_bwd(tree: Tree, params: AttnParams, q, k, v, o, lse, d_o, dq=None, dk=None, dv=None,
                  workspace=None, stages: int = BWD_ALL):
    """dta_tree_attn_bwd (or dta_tree_attn_bwd_stages when `stages` selects a
    subset) on torch's current stream.  Returns (dq, dk, dv)."""
    import torch
    dt = torch.float32 if params.dtype == F32 else torch.bfloat16
    _check_tree_tokens(tree, q)
    T = q.shape[0]
    _check_tensor(q, "q", (T, params.n_q_heads, params.head_dim), dt)
    _check_tensor(k, "k", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(v, "v", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(o, "o", q.shape, dt)
    _check_tensor(d_o, "d_o", q.shape, dt)
    _check_tensor(lse, "lse", (T, params.n_q_heads), torch.float32)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    _check_tensor(dq, "dq", q.shape, dt)
    _check_tensor(dk, "dk", k.shape, dt)
    _check_tensor(dv, "dv", v.shape, dt)
    if workspace is None:
        need = workspace_bytes(tree, params, True)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check_workspace(workspace)
    ws_bytes = workspace.numel() * workspace.element_size()
    lib = load_library()
    args = (tree.handle, C.byref(params), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
            _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), ws_bytes, _stream())
    if stages == BWD_ALL:
        _check(lib.dta_tree_attn_bwd(*args), "dta_tree_attn_bwd")
    else:
        _check(lib.dta_tree_attn_bwd_stages(*args, int(stages)), "dta_tree_attn_bwd_stages")
    return dq, dk, dv


def tree_attn_bwd_noalloc(tree: Tree, params: AttnParams, q, k, v, o, lse, d_o, dq, dk, dv):
    """dta_tree_attn_bwd_noalloc on torch's current stream: the backward pass on
    the library-held scratch array; every tensor, outputs included, is the
    caller's, and the tree must have been prepared (Tree.prepare)."""
    import torch
    dt = torch.float32 if params.dtype == F32 else torch.bfloat16
    _check_tree_tokens(tree, q)
    T = q.shape[0]
    for name, t, heads in (("q", q, params.n_q_heads), ("k", k, params.n_kv_heads), ("v", v, params.n_kv_heads),
                           ("o", o, params.n_q_heads), ("d_o", d_o, params.n_q_heads),
                           ("dq", dq, params.n_q_heads), ("dk", dk, params.n_kv_heads),
                           ("dv", dv, params.n_kv_heads)):
        _check_tensor(t, name, (T, heads, params.head_dim), dt)
    _check_tensor(lse, "lse", (T, params.n_q_heads), torch.float32)
    st = load_library().dta_tree_attn_bwd_noalloc(tree.handle, C.byref(params), _ptr(q), _ptr(k), _ptr(v),
                                                  _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv),
                                                  _stream())
    _check(st, "dta_tree_attn_bwd_noalloc")


def tree_attn_fwd_segment(tree: Tree, params: AttnParams, t_begin: int, t_end: int, q, k, v, o, lse):
    """dta_tree_attn_fwd_segment on torch's current stream: fills rows
    [t_begin, t_end) of the full-size o and lse."""
    import torch
    dt = torch.float32 if params.dtype == F32 else torch.bfloat16
    _check_tree_tokens(tree, q)
    T = q.shape[0]
    _check_tensor(q, "q", (T, params.n_q_heads, params.head_dim), dt)
    _check_tensor(k, "k", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(v, "v", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(o, "o", q.shape, dt)
    _check_tensor(lse, "lse", (T, params.n_q_heads), torch.float32)
    st = load_library().dta_tree_attn_fwd_segment(tree.handle, C.byref(params), int(t_begin), int(t_end),
                                                  _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                                  C.c_void_p(0), 0, _stream())
    _check(st, "dta_tree_attn_fwd_segment")


def tree_attn_bwd_segment(tree: Tree, params: AttnParams, t_begin: int, t_end: int, q, k, v, o, lse, d_o,
                          dq, dk_acc, dv_acc, workspace):
    """dta_tree_attn_bwd_segment on torch's current stream: writes rows
    [t_begin, t_end) of dq and adds into the fp32 accumulators dk_acc, dv_acc."""
    import torch
    dt = torch.float32 if params.dtype == F32 else torch.bfloat16
    _check_tree_tokens(tree, q)
    T = q.shape[0]
    _check_tensor(q, "q", (T, params.n_q_heads, params.head_dim), dt)
    _check_tensor(k, "k", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(v, "v", (T, params.n_kv_heads, params.head_dim), dt)
    _check_tensor(o, "o", q.shape, dt)
    _check_tensor(d_o, "d_o", q.shape, dt)
    _check_tensor(lse, "lse", (T, params.n_q_heads), torch.float32)
    _check_tensor(dq, "dq", q.shape, dt)
    _check_tensor(dk_acc, "dk_acc", k.shape, torch.float32)
    _check_tensor(dv_acc, "dv_acc", v.shape, torch.float32)
    _check_workspace(workspace)
    ws_bytes = workspace.numel() * workspace.element_size()
    st = load_library().dta_tree_attn_bwd_segment(tree.handle, C.byref(params), int(t_begin), int(t_end),
                                                  _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                                  _ptr(dq), _ptr(dk_acc), _ptr(dv_acc), _ptr(workspace),
                                                  ws_bytes, _stream())
    _check(st, "dta_tree_attn_bwd_segment")


class Rollouts:
    """Owns a dta_rollouts_t*: the prefix tree of a set of token sequences."""

    def __init__(self, seqs):
        seqs = [np.ascontiguousarray(s, dtype=np.int32) for s in seqs]
        offs = np.zeros(len(seqs) + 1, dtype=np.int64)
        offs[1:] = np.cumsum([len(s) for s in seqs])
        toks = np.concatenate(seqs) if seqs else np.zeros(0, dtype=np.int32)
        toks = np.ascontiguousarray(toks, dtype=np.int32)
        h = C.c_void_p()
        st = load_library().dta_rollouts_build(toks.ctypes.data_as(C.POINTER(C.c_int32)),
                                               offs.ctypes.data_as(C.POINTER(C.c_int64)), len(seqs),
                                               C.byref(h))
        _check(st, "dta_rollouts_build")
        self._h = h

    def view(self) -> dict:
        out = _RolloutsView()
        _check(load_library().dta_rollouts_view(self._h, C.byref(out)), "dta_rollouts_view")
        arr = lambda p, k: np.ctypeslib.as_array(p, shape=(k,)).copy() if k else np.zeros(0, dtype=np.int64)
        return dict(parent=arr(out.parent, out.n_nodes), seg_len=arr(out.seg_len, out.n_nodes),
                    tokens=arr(out.tokens, out.n_tokens), seq_node=arr(out.seq_node, out.n_seqs),
                    order=arr(out.order, out.n_seqs), lcp=arr(out.lcp, out.n_seqs))

    def partition(self, k: int):
        """(group_begin [k+1], group_cost [k]) of dta_rollouts_partition."""
        gb = np.zeros(max(k, 0) + 1, dtype=np.int32)
        gc = np.zeros(max(k, 1), dtype=np.int64)
        st = load_library().dta_rollouts_partition(self._h, int(k), gb.ctypes.data_as(C.POINTER(C.c_int32)),
                                                   gc.ctypes.data_as(C.POINTER(C.c_int64)))
        _check(st, "dta_rollouts_partition")
        return gb, gc[:k]

    def destroy(self):
        if self._h:
            load_library().dta_rollouts_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


OP_FWD, OP_REFWD, OP_BWD, OP_FWD_NOGRAD = 0, 1, 2, 3


def tree_plan(tree: Tree, block: int = 0) -> dict:
    """dta_tree_plan as plain Python data: leaf_order, ops [(op, leaf, lo, hi)],
    call_ptr, calls [(op, node, t_begin, t_end)] and the counters."""
    lib = load_library()
    h = C.c_void_p()
    _check(lib.dta_tree_plan(tree.handle, int(block), C.byref(h)), "dta_tree_plan")
    try:
        v = _PlanView()
        _check(lib.dta_plan_view(h, C.byref(v)), "dta_plan_view")
        return dict(
            leaf_order=[int(v.leaf_order[i]) for i in range(v.n_leaves)],
            ops=[(v.ops[i].op, v.ops[i].leaf, int(v.ops[i].lo), int(v.ops[i].hi)) for i in range(v.n_ops)],
            call_ptr=[int(v.call_ptr[i]) for i in range(v.n_ops + 1)],
            calls=[(v.calls[i].op, v.calls[i].node, int(v.calls[i].t_begin), int(v.calls[i].t_end))
                   for i in range(v.n_calls)],
            n_fwd=int(v.n_fwd), n_fwd_nograd=int(v.n_fwd_nograd), n_chunks=int(v.n_chunks),
            max_stack_tokens=int(v.max_stack_tokens))
    finally:
        lib.dta_plan_destroy(h)
