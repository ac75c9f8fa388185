"""Thin ctypes binding over libdyspec.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
``include/dyspec.h``; torch is used for device memory and the current stream.  There is no
CPU fallback: if the library is missing or fails to load, importing callers get an error.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

from . import build as _build

F32, BF16, BF16_WAVE = 0, 1, 0x101
MAX_SEQ, MAX_NODES, MAX_BUILD_NODES, MAX_VOCAB = 64, 2048, 1024, 32768
WS_BUILD_TREE, WS_TREE_ATTN, WS_VERIFY = 0, 1, 2
EXPORTS = ("dyspec_init", "dyspec_mask_words", "dyspec_workspace_bytes", "dyspec_status_string",
           "dyspec_build_tree", "dyspec_build_tree_threshold", "dyspec_build_tree_threshold_workspace_bytes",
           "dyspec_dfs_reorder", "dyspec_tree_attn", "dyspec_tree_attn_static_scratch", "dyspec_tree_attn_layers",
           "dyspec_tree_attn_layers_workspace_bytes", "dyspec_verify", "dyspec_verify_bf16",
           "dyspec_probe_mfma_bf16", "dyspec_probe_clock", "dyspec_probe_hbm_read")


class DyspecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _Batch(ctypes.Structure):
    _fields_ = [("n_seq", ctypes.c_int32),
                ("node_offset", ctypes.POINTER(ctypes.c_int32)),
                ("prefix_len", ctypes.POINTER(ctypes.c_int32)),
                ("kv_offset", ctypes.POINTER(ctypes.c_int64))]


class _Tree(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("parent", "token", "sib_rank", "first_child", "next_sibling", "depth")]


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libdyspec.so (building it first only when nothing is built)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or _build.LIB
    if not os.path.exists(p):
        _build.build(force=True)
    # torch brings its own copy of the HIP runtime; it has to be the one in the process before
    # this library is mapped, or the two would run on separate runtimes and every pointer torch
    # hands over would be foreign to the kernels' launches
    import torch  # noqa: F401
    lib = ctypes.CDLL(p)
    V, I32, U64, SZ, F = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_float
    PB, PT = ctypes.POINTER(_Batch), ctypes.POINTER(_Tree)
    lib.dyspec_init.restype = I32
    lib.dyspec_init.argtypes = []
    lib.dyspec_mask_words.restype = I32
    lib.dyspec_mask_words.argtypes = [PB]
    lib.dyspec_workspace_bytes.restype = SZ
    lib.dyspec_workspace_bytes.argtypes = [I32, PB, I32, I32, I32, I32]
    lib.dyspec_status_string.restype = ctypes.c_char_p
    lib.dyspec_status_string.argtypes = [I32]
    lib.dyspec_build_tree.restype = I32
    lib.dyspec_build_tree.argtypes = [V, I32, PB, ctypes.POINTER(F), U64, PT, V, V, V, V, SZ, V]
    lib.dyspec_build_tree_threshold.restype = I32
    lib.dyspec_build_tree_threshold.argtypes = [V, I32, PB, ctypes.POINTER(F), ctypes.POINTER(ctypes.c_double), U64, PT,
                                                V, V, V, ctypes.POINTER(I32), V, SZ, V]
    lib.dyspec_build_tree_threshold_workspace_bytes.restype = SZ
    lib.dyspec_build_tree_threshold_workspace_bytes.argtypes = [PB]
    lib.dyspec_tree_attn.restype = I32
    lib.dyspec_tree_attn.argtypes = [V, V, V, V, V, V, PB, I32, I32, I32, I32, F, V, V, SZ, V]
    lib.dyspec_tree_attn_static_scratch.restype = I32
    lib.dyspec_tree_attn_static_scratch.argtypes = [V, V, V, V, V, V, PB, I32, I32, I32, I32, F, V, V]
    lib.dyspec_tree_attn_layers.restype = I32
    lib.dyspec_tree_attn_layers.argtypes = [V, V, V, V, V, V, PB, I32, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                            I32, I32, I32, I32, F, V, V, SZ, V]
    lib.dyspec_tree_attn_layers_workspace_bytes.restype = SZ
    lib.dyspec_tree_attn_layers_workspace_bytes.argtypes = [PB, I32, I32, I32, I32]
    lib.dyspec_verify.restype = I32
    lib.dyspec_verify.argtypes = [V, V, I32, PB, PT, ctypes.POINTER(F), ctypes.POINTER(F), U64, I32,
                                  V, V, V, V, V, V, V, SZ, V]
    lib.dyspec_verify_bf16.restype = I32
    lib.dyspec_verify_bf16.argtypes = lib.dyspec_verify.argtypes
    lib.dyspec_dfs_reorder.restype = I32
    lib.dyspec_dfs_reorder.argtypes = [PB, PT, PT, V, V, V]
    lib.dyspec_probe_mfma_bf16.restype = I32
    lib.dyspec_probe_mfma_bf16.argtypes = [I32, I32, ctypes.POINTER(ctypes.c_double), V, V]
    lib.dyspec_probe_clock.restype = I32
    lib.dyspec_probe_clock.argtypes = [I32, V, ctypes.POINTER(I32), V]
    lib.dyspec_probe_hbm_read.restype = I32
    lib.dyspec_probe_hbm_read.argtypes = [V, SZ, V, V]
    if path is None:
        _lib = lib
    return lib


def init() -> None:
    """dyspec_init on torch's current device: code loading and kernel attributes up front."""
    _check(load_library().dyspec_init(), "dyspec_init")


def status_string(status: int) -> str:
    return load_library().dyspec_status_string(status).decode()


@dataclass
class Batch:
    """Host description of a ragged batch (see dyspec_batch in include/dyspec.h)."""
    node_offset: np.ndarray      # int32 [n_seq+1]
    prefix_len: np.ndarray       # int32 [n_seq]
    kv_offset: np.ndarray        # int64 [n_seq+1]

    @staticmethod
    def from_sizes(n_nodes: Sequence[int], prefix_len: Optional[Sequence[int]] = None) -> "Batch":
        n_nodes = list(n_nodes)
        prefix_len = [0] * len(n_nodes) if prefix_len is None else list(prefix_len)
        no = np.zeros(len(n_nodes) + 1, dtype=np.int32)
        no[1:] = np.cumsum(n_nodes)
        kv = np.zeros(len(n_nodes) + 1, dtype=np.int64)
        kv[1:] = np.cumsum(prefix_len)
        return Batch(no, np.asarray(prefix_len, dtype=np.int32), kv)

    @property
    def n_seq(self) -> int:
        return int(self.prefix_len.shape[0])

    @property
    def total_nodes(self) -> int:
        return int(self.node_offset[-1])

    @property
    def total_prefix(self) -> int:
        return int(self.kv_offset[-1])

    def _memo(self) -> dict:
        """Per-content cache (C struct, mask words, workspace sizes): calls in a layer loop
        describe the same batch again and again."""
        key = (self.node_offset.tobytes(), self.prefix_len.tobytes(), self.kv_offset.tobytes())
        memo = self.__dict__.get("_memo_store")
        if memo is None or memo["key"] != key:
            memo = {"key": key}
            self.__dict__["_memo_store"] = memo
        return memo

    def _c(self) -> _Batch:
        memo = self._memo()
        c = memo.get("c")
        if c is None:
            no = np.ascontiguousarray(self.node_offset, dtype=np.int32)
            pl = np.ascontiguousarray(self.prefix_len, dtype=np.int32)
            kv = np.ascontiguousarray(self.kv_offset, dtype=np.int64)
            c = _Batch(self.n_seq,
                       no.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                       pl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                       kv.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)))
            memo["c"], memo["keep"] = c, (no, pl, kv)          # the struct points into these copies
        return c

    @property
    def mask_words(self) -> int:
        memo = self._memo()
        if "mask_words" not in memo:
            memo["mask_words"] = int(load_library().dyspec_mask_words(ctypes.byref(self._c())))
        return memo["mask_words"]


@dataclass
class Tree:
    """Device-resident packed token trees (see dyspec_tree in include/dyspec.h)."""
    parent: "torch.Tensor"
    token: "torch.Tensor"
    sib_rank: "torch.Tensor"
    first_child: "torch.Tensor"
    next_sibling: "torch.Tensor"
    depth: "torch.Tensor"

    def _c(self) -> _Tree:
        return _Tree(*[_ptr(getattr(self, n), "int32") for n in
                       ("parent", "token", "sib_rank", "first_child", "next_sibling", "depth")])

    @staticmethod
    def empty(total_nodes: int, device) -> "Tree":
        import torch
        return Tree(*[torch.empty(total_nodes, dtype=torch.int32, device=device) for _ in range(6)])


def _ptr(t, want: Optional[str] = None) -> int:
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("device tensor required")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor required")
    if want is not None and str(t.dtype) != "torch." + want:
        raise ValueError(f"expected {want}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream=None) -> int:
    import torch
    if stream is not None:
        return int(stream.cuda_stream)
    return int(torch._C._cuda_getCurrentRawStream(torch.cuda.current_device()))


def _temps(x, n_seq: int):
    a = np.ascontiguousarray(np.broadcast_to(np.asarray(x, dtype=np.float32), (n_seq,)))
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _check(status: int, where: str) -> None:
    if status != 0:
        raise DyspecError(status, where)


@dataclass
class BuiltTrees:
    tree: Tree
    est_value: "torch.Tensor"      # fp32 [sum N]
    anc_mask: "torch.Tensor"       # int64 view of u64 [sum N, mask_words]
    n_built: "torch.Tensor"        # int32 [n_seq]


def build_tree(draft_logits, batch: Batch, draft_temp, seed: int, stream=None, use_workspace: bool = True) -> BuiltTrees:
    """dyspec_build_tree: greedy token-tree construction (Algorithm 1) + ancestor mask.
    use_workspace=False passes no workspace (the slower form that recomputes row sums)."""
    import torch
    lib = load_library()
    dev = draft_logits.device
    total, V = batch.total_nodes, int(draft_logits.shape[1])
    if draft_logits.shape[0] != total:
        raise ValueError("draft_logits needs one row per tree node")
    tree = Tree.empty(total, dev)
    est = torch.empty(total, dtype=torch.float32, device=dev)
    mask = torch.empty((total, batch.mask_words), dtype=torch.int64, device=dev)
    nb = torch.empty(batch.n_seq, dtype=torch.int32, device=dev)
    cb, ct = batch._c(), tree._c()
    tarr, tptr = _temps(draft_temp, batch.n_seq)
    ws, ws_bytes = None, 0
    if use_workspace:
        ws_bytes = int(lib.dyspec_workspace_bytes(WS_BUILD_TREE, ctypes.byref(cb), V, 0, 0, 0))
        if ws_bytes:
            ws = torch.empty(ws_bytes // 8, dtype=torch.float64, device=dev)
    st = lib.dyspec_build_tree(_ptr(draft_logits, "float32"), V, ctypes.byref(cb), tptr, ctypes.c_uint64(seed),
                               ctypes.byref(ct), _ptr(est), _ptr(mask), _ptr(nb),
                               _ptr(ws) if ws is not None else None, ctypes.c_size_t(ws_bytes), _stream(stream))
    _check(st, "dyspec_build_tree")
    return BuiltTrees(tree, est, mask, nb)


def build_tree_threshold(draft_logits, batch: Batch, draft_temp, threshold, seed: int, stream=None):
    """dyspec_build_tree_threshold: level-by-level construction with a threshold (Algorithm 2)
    + ancestor mask.  Returns (BuiltTrees, levels expanded); the call waits for the tree."""
    import torch
    lib = load_library()
    dev = draft_logits.device
    total, V = batch.total_nodes, int(draft_logits.shape[1])
    if draft_logits.shape[0] != total:
        raise ValueError("draft_logits needs one row per tree node")
    tree = Tree.empty(total, dev)
    est = torch.empty(total, dtype=torch.float32, device=dev)
    mask = torch.empty((total, batch.mask_words), dtype=torch.int64, device=dev)
    nb = torch.empty(batch.n_seq, dtype=torch.int32, device=dev)
    cb, ct = batch._c(), tree._c()
    tarr, tptr = _temps(draft_temp, batch.n_seq)
    thr = np.ascontiguousarray(np.broadcast_to(np.asarray(threshold, dtype=np.float64), (batch.n_seq,)))
    ws_bytes = int(lib.dyspec_build_tree_threshold_workspace_bytes(ctypes.byref(cb)))
    ws = torch.empty(max(ws_bytes // 8, 1), dtype=torch.float64, device=dev)
    levels = ctypes.c_int32(0)
    st = lib.dyspec_build_tree_threshold(_ptr(draft_logits, "float32"), V, ctypes.byref(cb), tptr,
                                         thr.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), ctypes.c_uint64(seed),
                                         ctypes.byref(ct), _ptr(est), _ptr(mask), _ptr(nb), ctypes.byref(levels),
                                         _ptr(ws), ctypes.c_size_t(ws_bytes), _stream(stream))
    _check(st, "dyspec_build_tree_threshold")
    return BuiltTrees(tree, est, mask, nb), int(levels.value)


@dataclass
class ReorderedTrees:
    tree: Tree
    order: "torch.Tensor"          # int32 [sum N]: order[offset + new] = old local index
    anc_mask: "torch.Tensor"       # int64 view of u64 [sum N, mask_words]

    def gather_index(self, batch: "Batch"):
        """Global row indices: tensor[gather_index] puts token-aligned rows into the new order."""
        import torch
        off = torch.from_numpy(np.repeat(batch.node_offset[:-1], np.diff(batch.node_offset)).astype(np.int64))
        return self.order.long() + off.to(self.order.device)


def dfs_reorder(tree: Tree, batch: Batch, stream=None) -> ReorderedTrees:
    """dyspec_dfs_reorder: rename every tree's nodes in depth-first order (block-sparsity friendly)."""
    import torch
    lib = load_library()
    dev = tree.parent.device
    total = batch.total_nodes
    out = Tree.empty(total, dev)
    order = torch.empty(total, dtype=torch.int32, device=dev)
    mask = torch.empty((total, batch.mask_words), dtype=torch.int64, device=dev)
    cb, ci, co = batch._c(), tree._c(), out._c()
    _check(lib.dyspec_dfs_reorder(ctypes.byref(cb), ctypes.byref(ci), ctypes.byref(co), _ptr(order, "int32"),
                                  _ptr(mask, "int64"), _stream(stream)), "dyspec_dfs_reorder")
    return ReorderedTrees(out, order, mask)


_scratch_cache = {}


def _scratch(device, nbytes: int):
    """A zero-filled device buffer of at least nbytes, kept between calls (calls on one stream run
    in order, so consecutive layers can share it).  Tree attention wants the head of its workspace
    zero at the first call and leaves it zero, so the buffer is cleared once, here."""
    import torch
    key = str(device)
    buf = _scratch_cache.get(key)
    if buf is None or buf.numel() * 4 < nbytes:
        buf = torch.zeros((nbytes + 3) // 4, dtype=torch.float32, device=device)
        _scratch_cache[key] = buf
    return buf


class PreparedCall:
    """One library call with its arguments checked and marshalled once.  Calling the object issues
    the call again on the stream it was prepared for (the current one at that time unless given),
    with the same tensors: what a loop that repeats a call wants, e.g. a decode loop's layers,
    where the checks and conversions of the plain functions cost more host time per call than a
    short kernel runs.  The object keeps its tensors alive; `out` is what the plain function
    returns."""
    __slots__ = ("_fn", "_args", "_keep", "_where", "out")

    def __init__(self, fn, args, keep, where, out):
        self._fn, self._args, self._keep, self._where, self.out = fn, args, keep, where, out

    def __call__(self):
        st = self._fn(*self._args)
        if st != 0:
            raise DyspecError(st, self._where)
        return self.out


def tree_attn(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch: Batch, softmax_scale: float,
              out=None, dtype: Optional[int] = None, stream=None, use_workspace: bool = True,
              static_scratch: bool = False):
    """dyspec_tree_attn: one layer of tree-masked attention.  q/out [sum N, Hq, d].
    use_workspace=False passes no workspace (then the prefix is never split over workgroups).
    static_scratch=True calls dyspec_tree_attn_static_scratch instead (the library's own static
    array in place of a workspace; `out` must be given: this path allocates nothing)."""
    return tree_attn_call(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch, softmax_scale, out, dtype, stream,
                          use_workspace, static_scratch)()


def tree_attn_call(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch: Batch, softmax_scale: float,
                   out=None, dtype: Optional[int] = None, stream=None, use_workspace: bool = True,
                   static_scratch: bool = False) -> PreparedCall:
    """tree_attn's call, prepared: nothing is launched until the returned object is called."""
    import torch
    lib = load_library()
    total, Hq, d = q.shape
    Hkv = int(k_tree.shape[1])
    if dtype is None:
        dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
    if total != batch.total_nodes or k_tree.shape[0] != total or v_tree.shape != k_tree.shape:
        raise ValueError("q / k_tree / v_tree need one row per tree node")
    if batch.total_prefix > 0 and (k_prefix.shape[0] < batch.total_prefix or k_prefix.shape[1] != Hkv
                                   or k_prefix.shape[2] != d or v_prefix.shape != k_prefix.shape):
        raise ValueError("prefix K/V shape does not match the batch")
    if anc_mask.shape[0] != total or anc_mask.shape[1] != batch.mask_words:
        raise ValueError("ancestor mask shape does not match the batch")
    for t in (k_prefix, v_prefix, k_tree, v_tree):
        if t is not None and t.dtype != q.dtype:
            raise ValueError("q, k, v must share a dtype")
    if out is None:
        if static_scratch:
            raise ValueError("static_scratch=True needs the caller's `out` tensor")
        out = torch.empty_like(q)
    cb = batch._c()
    keep = (q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, out, batch, cb)
    if static_scratch:
        args = (_ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(anc_mask, "int64"),
                ctypes.byref(cb), int(Hq), Hkv, int(d), int(dtype), ctypes.c_float(softmax_scale), _ptr(out), _stream(stream))
        return PreparedCall(lib.dyspec_tree_attn_static_scratch, args, keep, "dyspec_tree_attn_static_scratch", out)
    ws, ws_bytes = None, 0
    if use_workspace and dtype == BF16:
        memo, wkey = batch._memo(), ("ws_attn", int(Hq), Hkv, int(d))
        if wkey not in memo:
            memo[wkey] = int(lib.dyspec_workspace_bytes(WS_TREE_ATTN, ctypes.byref(cb), 0, int(Hq), Hkv, int(d)))
        ws_bytes = memo[wkey]
        if ws_bytes:
            ws = _scratch(q.device, ws_bytes)
    args = (_ptr(q), _ptr(k_prefix), _ptr(v_prefix), _ptr(k_tree), _ptr(v_tree), _ptr(anc_mask, "int64"),
            ctypes.byref(cb), int(Hq), Hkv, int(d), int(dtype), ctypes.c_float(softmax_scale), _ptr(out),
            _ptr(ws) if ws is not None else None, ctypes.c_size_t(ws_bytes), _stream(stream))
    return PreparedCall(lib.dyspec_tree_attn, args, keep + (ws,), "dyspec_tree_attn", out)


def tree_attn_layers(q, k_prefix, v_prefix, k_tree, v_tree, anc_mask, batch: Batch, softmax_scale: float,
                     out=None, dtype: Optional[int] = None, stream=None, use_workspace: bool = True):
    """dyspec_tree_attn_layers: tree-masked attention of L stacked layers in one call.
    q/out [L, sum N, Hq, d], k_prefix/v_prefix [L, kv rows, Hkv, d], k_tree/v_tree [L, sum N, Hkv, d];
    the leading dimension may be strided, the rest is dense."""
    import torch
    lib = load_library()
    L, total, Hq, d = q.shape
    Hkv = int(k_tree.shape[2])
    if dtype is None:
        dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
    if total != batch.total_nodes or tuple(k_tree.shape) != (L, total, Hkv, d) or v_tree.shape != k_tree.shape:
        raise ValueError("q / k_tree / v_tree need one row per tree node and layer")
    if batch.total_prefix > 0 and (k_prefix.shape[0] != L or k_prefix.shape[1] < batch.total_prefix or k_prefix.shape[2] != Hkv
                                   or k_prefix.shape[3] != d or v_prefix.shape != k_prefix.shape):
        raise ValueError("prefix K/V shape does not match the batch")
    if anc_mask.shape[0] != total or anc_mask.shape[1] != batch.mask_words:
        raise ValueError("ancestor mask shape does not match the batch")
    if out is None:
        out = torch.empty_like(q)
    for t in (q, out, k_prefix, v_prefix, k_tree, v_tree):
        if t is None:
            continue
        if t.dtype != q.dtype:
            raise ValueError("q, k, v, out must share a dtype")
        if not t.is_cuda or not t[0].is_contiguous():
            raise ValueError("device tensors with dense layers required")
    if out.stride(0) != q.stride(0) or (k_prefix is not None and v_prefix.stride(0) != k_prefix.stride(0)) \
            or v_tree.stride(0) != k_tree.stride(0):
        raise ValueError("q/out, k_prefix/v_prefix and k_tree/v_tree must share their layer strides")
    cb = batch._c()
    ws, ws_bytes = None, 0
    if use_workspace and dtype == BF16:
        ws_bytes = int(lib.dyspec_tree_attn_layers_workspace_bytes(ctypes.byref(cb), int(L), int(Hq), Hkv, int(d)))
        if ws_bytes:
            ws = _scratch(q.device, ws_bytes)
    kp_stride = int(k_prefix.stride(0)) if k_prefix is not None else 0
    base = lambda t: 0 if t is None else t.data_ptr()          # the layer dimension may be strided
    st = lib.dyspec_tree_attn_layers(base(q), base(k_prefix), base(v_prefix), base(k_tree), base(v_tree),
                                     _ptr(anc_mask, "int64"), ctypes.byref(cb), int(L), int(q.stride(0)), kp_stride,
                                     int(k_tree.stride(0)), int(Hq), Hkv, int(d), int(dtype),
                                     ctypes.c_float(softmax_scale), base(out), _ptr(ws) if ws is not None else None,
                                     ctypes.c_size_t(ws_bytes), _stream(stream))
    _check(st, "dyspec_tree_attn_layers")
    return out


@dataclass
class VerifyOutput:
    row_stats: "torch.Tensor"        # fp32 [sum N, 4]
    accept_ratio: "torch.Tensor"     # fp32 [sum N]; -1 / -2 mark children the walk did not test
    accepted_nodes: "torch.Tensor"   # int32 [sum N]
    n_accepted: "torch.Tensor"       # int32 [n_seq]
    final_token: "torch.Tensor"      # int32 [n_seq]
    min_margin: "torch.Tensor"       # fp32 [n_seq]

    @staticmethod
    def empty(batch: Batch, device) -> "VerifyOutput":
        import torch
        t, s = batch.total_nodes, batch.n_seq
        f = lambda *sh: torch.empty(sh, dtype=torch.float32, device=device)
        i = lambda *sh: torch.empty(sh, dtype=torch.int32, device=device)
        return VerifyOutput(f(t, 4), f(t), i(t), i(s), i(s), f(s))


def verify(draft_logits, target_logits, batch: Batch, tree: Tree, draft_temp, target_temp, seed: int,
           emit_bonus: bool = True, out: Optional[VerifyOutput] = None, stream=None) -> VerifyOutput:
    """dyspec_verify / dyspec_verify_bf16 (by the tables' dtype): per-row vocabulary softmax + tree
    rejection sampling (Algorithm 3)."""
    return verify_call(draft_logits, target_logits, batch, tree, draft_temp, target_temp, seed, emit_bonus, out, stream)()


def verify_call(draft_logits, target_logits, batch: Batch, tree: Tree, draft_temp, target_temp, seed: int,
                emit_bonus: bool = True, out: Optional[VerifyOutput] = None, stream=None) -> PreparedCall:
    """verify's call, prepared: nothing is launched until the returned object is called."""
    import torch
    lib = load_library()
    total, V = batch.total_nodes, int(draft_logits.shape[1])
    if draft_logits.shape[0] != total or target_logits.shape != draft_logits.shape:
        raise ValueError("logit tables need one row per tree node")
    if draft_logits.dtype != target_logits.dtype or draft_logits.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("logit tables must both be float32 or both be bfloat16")
    bf16 = draft_logits.dtype == torch.bfloat16
    entry = lib.dyspec_verify_bf16 if bf16 else lib.dyspec_verify
    if out is None:
        out = VerifyOutput.empty(batch, draft_logits.device)
    cb, ct = batch._c(), tree._c()
    da, dp = _temps(draft_temp, batch.n_seq)
    ta, tp = _temps(target_temp, batch.n_seq)
    args = (_ptr(draft_logits), _ptr(target_logits), V, ctypes.byref(cb), ctypes.byref(ct), dp, tp,
            ctypes.c_uint64(seed), int(bool(emit_bonus)), _ptr(out.row_stats), _ptr(out.accept_ratio),
            _ptr(out.accepted_nodes), _ptr(out.n_accepted), _ptr(out.final_token), _ptr(out.min_margin), None, 0,
            _stream(stream))
    keep = (draft_logits, target_logits, batch, tree, cb, ct, da, ta, out)
    return PreparedCall(entry, args, keep, "dyspec_verify_bf16" if bf16 else "dyspec_verify", out)


def probe_mfma_bf16(iterations: int, sink, stream=None, random_operands: bool = False) -> float:
    """dyspec_probe_mfma_bf16: launches the MFMA-only loop, returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _check(load_library().dyspec_probe_mfma_bf16(int(iterations), int(bool(random_operands)), ctypes.byref(flops),
                                                 _ptr(sink, "float32"), _stream(stream)), "dyspec_probe_mfma_bf16")
    return float(flops.value)


def probe_clock(iterations: int, counters, stream=None) -> int:
    """dyspec_probe_clock: launches the sleeping wave; counters (int64[2], device) receives shader
    cycles and wall clock ticks once it ends.  Returns the wall clock rate in kHz."""
    khz = ctypes.c_int32(0)
    _check(load_library().dyspec_probe_clock(int(iterations), _ptr(counters, "int64"), ctypes.byref(khz), _stream(stream)),
           "dyspec_probe_clock")
    return int(khz.value)


def probe_hbm_read(src, sink, stream=None) -> int:
    """dyspec_probe_hbm_read: launches one streaming read of src, returns the bytes read."""
    nbytes = (src.numel() * src.element_size()) // 16 * 16
    _check(load_library().dyspec_probe_hbm_read(_ptr(src), ctypes.c_size_t(nbytes), _ptr(sink, "float32"),
                                                _stream(stream)), "dyspec_probe_hbm_read")
    return nbytes
