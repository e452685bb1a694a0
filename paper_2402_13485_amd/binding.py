"""Thin Python binding of the C ABI in ``include/propd.h``.

Argument marshalling only: every step of the verification path runs in the HIP
kernels of ``libpropd.so``.  PyTorch tensors supply device memory and the current
stream; nothing here computes on them.  There is no CPU fallback: if the library
is missing or cannot be loaded, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpropd.so")

PROPD_F32, PROPD_BF16 = 0, 1
WS_TREE_ATTENTION, WS_EARLY_PRUNE, WS_ACCEPT_PATH = 0, 1, 2
MAX_TREE = 128
MAX_PAYLOADS = 8

EXPORTS = ("propd_tree_mask", "propd_validate_tree", "propd_tree_attention", "propd_early_prune", "propd_accept_path",
           "propd_accept_path_static", "propd_early_prune_prob", "propd_commit_path", "propd_workspace_bytes", "propd_status_string",
           "propd_controller_bytes", "propd_controller_init", "propd_controller_observe_time",
           "propd_controller_observe_hit", "propd_controller_fit", "propd_controller_build_tree",
           "propd_controller_best_size")


class _Tree(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T_max", ctypes.c_int32),
                ("n_nodes", ctypes.c_void_p), ("parent", ctypes.c_void_p),
                ("token", ctypes.c_void_p), ("depth", ctypes.c_void_p), ("anc", ctypes.c_void_p)]


class _TreeOut(ctypes.Structure):
    _fields_ = [("n_nodes", ctypes.c_void_p), ("parent", ctypes.c_void_p),
                ("token", ctypes.c_void_p), ("depth", ctypes.c_void_p), ("anc", ctypes.c_void_p)]


class _Payload(ctypes.Structure):
    _fields_ = [("src", ctypes.c_void_p), ("dst", ctypes.c_void_p), ("row_bytes", ctypes.c_size_t),
                ("outer", ctypes.c_int64), ("stride_b", ctypes.c_int64),
                ("stride_outer", ctypes.c_int64), ("stride_t", ctypes.c_int64)]


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    """Load libpropd.so (built in-tree by ``build.py``); raise if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2402_13485_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.propd_tree_mask.restype = ctypes.c_int
    lib.propd_tree_mask.argtypes = [i32, i32, vp, vp, vp, vp, vp]
    lib.propd_validate_tree.restype = ctypes.c_int
    lib.propd_validate_tree.argtypes = [ctypes.POINTER(_Tree), vp, vp]
    lib.propd_tree_attention.restype = ctypes.c_int
    lib.propd_tree_attention.argtypes = [ctypes.POINTER(_Tree), ctypes.c_int, i32, i32,
                                         ctypes.c_float, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.propd_early_prune.restype = ctypes.c_int
    lib.propd_early_prune.argtypes = [ctypes.POINTER(_Tree), ctypes.c_int, i32, i32, i32, vp, vp,
                                      vp, vp, vp, vp, vp, ctypes.POINTER(_TreeOut), vp, i32,
                                      ctypes.POINTER(_Payload), vp, sz, vp]
    lib.propd_early_prune_prob.restype = ctypes.c_int
    lib.propd_early_prune_prob.argtypes = [ctypes.POINTER(_Tree), ctypes.c_int, i32, i32, ctypes.c_int,
                                           ctypes.c_float, i32, vp, vp, vp, vp, vp, vp, vp,
                                           ctypes.POINTER(_TreeOut), vp, i32,
                                           ctypes.POINTER(_Payload), vp, sz, vp]
    lib.propd_accept_path.restype = ctypes.c_int
    lib.propd_accept_path.argtypes = [ctypes.POINTER(_Tree), ctypes.c_int, i32, vp, vp, vp, i32, vp,
                                      vp, sz, vp]
    lib.propd_accept_path_static.restype = ctypes.c_int
    lib.propd_accept_path_static.argtypes = [ctypes.POINTER(_Tree), ctypes.c_int, i32, vp, vp, vp, i32,
                                             vp, vp]
    lib.propd_commit_path.restype = ctypes.c_int
    lib.propd_commit_path.argtypes = [ctypes.POINTER(_Tree), ctypes.c_int, i32, i32, vp, vp, i32, vp,
                                      vp, vp, vp, vp, i32, vp, vp, i32, vp]
    lib.propd_workspace_bytes.restype = sz
    lib.propd_workspace_bytes.argtypes = [ctypes.c_int, i32, i32, i32, i32, i32, i32, i32]
    dbl, pd = ctypes.c_double, ctypes.POINTER(ctypes.c_double)
    lib.propd_controller_bytes.restype = sz
    lib.propd_controller_bytes.argtypes = [i32, i32, i32]
    lib.propd_controller_init.restype = ctypes.c_int
    lib.propd_controller_init.argtypes = [vp, sz, vp, i32, i32, i32, dbl, dbl, vp]
    lib.propd_controller_observe_time.restype = ctypes.c_int
    lib.propd_controller_observe_time.argtypes = [vp, i32, dbl, dbl]
    lib.propd_controller_observe_hit.restype = ctypes.c_int
    lib.propd_controller_observe_hit.argtypes = [vp, i32, i32]
    lib.propd_controller_fit.restype = ctypes.c_int
    lib.propd_controller_fit.argtypes = [vp, dbl, pd, pd]
    lib.propd_controller_build_tree.restype = ctypes.c_int
    lib.propd_controller_build_tree.argtypes = [vp, i32, ctypes.POINTER(i32), vp, vp, vp, vp, pd]
    lib.propd_controller_best_size.restype = ctypes.c_int
    lib.propd_controller_best_size.argtypes = [vp, dbl, ctypes.POINTER(i32), vp, pd, pd]
    lib.propd_status_string.restype = ctypes.c_char_p
    lib.propd_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def to_device(a: "np.ndarray") -> torch.Tensor:
    """numpy -> GPU tensor.  uint16 arrays are bf16 bit patterns; uint64 travels as int64."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> "np.ndarray":
    """GPU tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class PropdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load_library().propd_status_string(code).decode()
        super().__init__(f"{where}: {msg} (status {code})")


def _check(code: int, where: str) -> None:
    if code != 0:
        raise PropdError(code, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: need a contiguous {dtype} tensor in GPU memory")
    return t


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return PROPD_BF16
    if t.dtype == torch.float32:
        return PROPD_F32
    raise TypeError(f"tensor dtype must be bfloat16 or float32, got {t.dtype}")


@dataclass
class Tree:
    """Device-resident batch of token trees (fields as in ``propd_tree``)."""
    n_nodes: torch.Tensor                 # int32 [B]
    parent: torch.Tensor                  # int32 [B,T_max]
    token: Optional[torch.Tensor] = None  # int32 [B,T_max]
    depth: Optional[torch.Tensor] = None  # int32 [B,T_max]
    anc: Optional[torch.Tensor] = None    # int64 [B,T_max,2] holding the uint64 bit sets

    @property
    def B(self) -> int:
        return self.parent.shape[0]

    @property
    def T_max(self) -> int:
        return self.parent.shape[1]

    def _c(self) -> _Tree:
        return _Tree(self.B, self.T_max, _ptr(self.n_nodes), _ptr(self.parent), _ptr(self.token),
                     _ptr(self.depth), _ptr(self.anc))


def workspace_bytes(which: int, B: int, T_max: int, H: int = 0, d: int = 0, L_max: int = 0,
                    hidden: int = 0, vocab: int = 0) -> int:
    return int(load_library().propd_workspace_bytes(which, B, T_max, H, d, L_max, hidden, vocab))


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    if workspace is not None:
        if workspace.numel() * workspace.element_size() < nbytes:
            raise ValueError("workspace tensor too small")
        return workspace
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def propd_tree_mask(n_nodes: torch.Tensor, parent: torch.Tensor):
    """-> (depth int32 [B,T_max], anc int64 [B,T_max,2])"""
    _dev(n_nodes, torch.int32, "n_nodes")
    _dev(parent, torch.int32, "parent")
    B, T_max = parent.shape
    depth = torch.empty((B, T_max), dtype=torch.int32, device=parent.device)
    anc = torch.empty((B, T_max, 2), dtype=torch.int64, device=parent.device)
    _check(load_library().propd_tree_mask(B, T_max, _ptr(n_nodes), _ptr(parent), _ptr(depth),
                                          _ptr(anc), _stream()), "propd_tree_mask")
    return depth, anc


TREE_BAD_SIZE, TREE_BAD_PARENT, TREE_BAD_DEPTH, TREE_BAD_MASK = 1, 2, 4, 8


def propd_validate_tree(tree: "Tree") -> torch.Tensor:
    """-> int32 [B] of TREE_BAD_* flags per sequence (0 = consistent); no synchronisation."""
    flags = torch.empty(tree.B, dtype=torch.int32, device=tree.n_nodes.device)
    c_tree = tree._c()
    _check(load_library().propd_validate_tree(ctypes.byref(c_tree), _ptr(flags), _stream()),
           "propd_validate_tree")
    return flags


def propd_tree_attention(tree: Tree, q, k_cache, v_cache, k_tree, v_tree, seq_lens, scale: float,
                         out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    dt = _dt(q)
    B, H, T_max, d = q.shape
    L_max = k_cache.shape[2]
    for name, t, shape in (("q", q, (B, H, T_max, d)), ("k_cache", k_cache, (B, H, L_max, d)),
                           ("v_cache", v_cache, (B, H, L_max, d)),
                           ("k_tree", k_tree, (B, H, T_max, d)),
                           ("v_tree", v_tree, (B, H, T_max, d))):
        _dev(t, q.dtype, name)
        if tuple(t.shape) != shape:
            raise ValueError(f"{name}: expected shape {shape}, got {tuple(t.shape)}")
    _dev(seq_lens, torch.int32, "seq_lens")
    if tree.B != B or tree.T_max != T_max:
        raise ValueError("tree and q disagree on B or T_max")
    if out is None:
        out = torch.empty_like(q)
    ws = _workspace(workspace_bytes(WS_TREE_ATTENTION, B, T_max, H, d, L_max), q.device, workspace)
    c_tree = tree._c()
    _check(load_library().propd_tree_attention(
        ctypes.byref(c_tree), dt, H, d, scale, _ptr(q), _ptr(k_cache) if L_max else None,
        _ptr(v_cache) if L_max else None, _ptr(k_tree), _ptr(v_tree), _ptr(seq_lens), L_max,
        _ptr(out), _ptr(ws), ws.numel() * ws.element_size(), _stream()), "propd_tree_attention")
    return out


@dataclass
class PruneResult:
    keep_bits: torch.Tensor   # int64 [B,2]
    new_index: torch.Tensor   # int32 [B,T_max]
    orig_index: torch.Tensor  # int32 [B,T_max]
    n_kept: torch.Tensor      # int32 [B]
    cu_nodes: torch.Tensor    # int32 [B+1]
    tree: Tree                # compacted tree
    rank: Optional[torch.Tensor]
    payloads: list
    log_marginal: Optional[torch.Tensor] = None   # float32 [B,T_max], probability criterion only


def propd_early_prune(tree: Tree, hidden_states: torch.Tensor, head_weight: torch.Tensor,
                      top_k: int, payloads: Sequence[torch.Tensor] = (),
                      payload_out: Optional[Sequence[torch.Tensor]] = None,
                      want_rank: bool = False,
                      workspace: Optional[torch.Tensor] = None) -> PruneResult:
    """``payloads`` are tensors shaped [B,T_max,C] or [B,outer,T_max,C] to narrow to survivors."""
    return _early_prune(("topk", top_k), tree, hidden_states, head_weight, payloads, payload_out,
                        want_rank, workspace)


def propd_early_prune_prob(tree: Tree, hidden_states: torch.Tensor, head_weight: torch.Tensor,
                           threshold: Optional[float] = None, keep_count: Optional[int] = None,
                           payloads: Sequence[torch.Tensor] = (),
                           payload_out: Optional[Sequence[torch.Tensor]] = None,
                           want_log_marginal: bool = False,
                           workspace: Optional[torch.Tensor] = None) -> PruneResult:
    """Probability-based criterion: give exactly one of ``threshold`` (a probability) and
    ``keep_count`` (sequences kept per tree)."""
    if (threshold is None) == (keep_count is None):
        raise ValueError("give exactly one of threshold and keep_count")
    crit = ("threshold", float(threshold)) if keep_count is None else ("rank", int(keep_count))
    return _early_prune(crit, tree, hidden_states, head_weight, payloads, payload_out,
                        want_log_marginal, workspace)


def _early_prune(crit, tree, hidden_states, head_weight, payloads, payload_out, want_extra,
                 workspace) -> PruneResult:
    want_rank = want_extra and crit[0] == "topk"
    dt = _dt(hidden_states)
    B, T_max, hidden = hidden_states.shape
    vocab = head_weight.shape[0]
    _dev(hidden_states, hidden_states.dtype, "hidden_states")
    _dev(head_weight, hidden_states.dtype, "head_weight")
    if tuple(head_weight.shape) != (vocab, hidden):
        raise ValueError("head_weight must be [vocab, hidden]")
    if tree.B != B or tree.T_max != T_max:
        raise ValueError("tree and hidden_states disagree on B or T_max")
    dev = hidden_states.device
    i32 = dict(dtype=torch.int32, device=dev)
    res = PruneResult(
        keep_bits=torch.empty((B, 2), dtype=torch.int64, device=dev),
        new_index=torch.empty((B, T_max), **i32), orig_index=torch.empty((B, T_max), **i32),
        n_kept=torch.empty(B, **i32), cu_nodes=torch.empty(B + 1, **i32),
        tree=Tree(n_nodes=torch.empty(B, **i32), parent=torch.empty((B, T_max), **i32),
                  token=torch.empty((B, T_max), **i32), depth=torch.empty((B, T_max), **i32),
                  anc=torch.empty((B, T_max, 2), dtype=torch.int64, device=dev)),
        rank=torch.empty((B, T_max), **i32) if want_rank else None, payloads=[])
    descs = (_Payload * max(len(payloads), 1))()
    for n, src in enumerate(payloads):
        if not src.is_cuda or not src.is_contiguous() or src.dim() not in (3, 4):
            raise TypeError("payload: need a contiguous GPU tensor [B,T_max,C] or [B,outer,T_max,C]")
        outer = 1 if src.dim() == 3 else src.shape[1]
        if src.shape[0] != B or src.shape[-2] != T_max:
            raise ValueError("payload shape does not match the tree")
        dst = payload_out[n] if payload_out is not None else torch.empty_like(src)
        if dst.shape != src.shape or dst.dtype != src.dtype or not dst.is_contiguous():
            raise ValueError("payload_out must match the payload")
        row_bytes = src.shape[-1] * src.element_size()
        descs[n] = _Payload(src.data_ptr(), dst.data_ptr(), row_bytes, outer,
                            outer * T_max * row_bytes, T_max * row_bytes, row_bytes)
        res.payloads.append(dst)
    t_out = _TreeOut(_ptr(res.tree.n_nodes), _ptr(res.tree.parent), _ptr(res.tree.token),
                     _ptr(res.tree.depth), _ptr(res.tree.anc))
    ws = _workspace(workspace_bytes(WS_EARLY_PRUNE, B, T_max, hidden=hidden, vocab=vocab), dev,
                    workspace)
    c_tree = tree._c()
    if crit[0] == "topk":
        _check(load_library().propd_early_prune(
            ctypes.byref(c_tree), dt, hidden, vocab, crit[1], _ptr(hidden_states), _ptr(head_weight),
            _ptr(res.keep_bits), _ptr(res.new_index), _ptr(res.orig_index), _ptr(res.n_kept),
            _ptr(res.cu_nodes), ctypes.byref(t_out), _ptr(res.rank), len(payloads), descs, _ptr(ws),
            ws.numel() * ws.element_size(), _stream()), "propd_early_prune")
    else:
        if want_extra:
            res.log_marginal = torch.empty((B, T_max), dtype=torch.float32, device=dev)
        mode = 0 if crit[0] == "threshold" else 1
        _check(load_library().propd_early_prune_prob(
            ctypes.byref(c_tree), dt, hidden, vocab, mode, crit[1] if mode == 0 else 0.0,
            crit[1] if mode == 1 else 0, _ptr(hidden_states), _ptr(head_weight),
            _ptr(res.keep_bits), _ptr(res.new_index), _ptr(res.orig_index), _ptr(res.n_kept),
            _ptr(res.cu_nodes), ctypes.byref(t_out), _ptr(res.log_marginal), len(payloads), descs,
            _ptr(ws), ws.numel() * ws.element_size(), _stream()), "propd_early_prune_prob")
    return res


def propd_accept_path(tree: Tree, logits: torch.Tensor, path_stride: Optional[int] = None,
                      workspace: Optional[torch.Tensor] = None):
    """-> (accept_len int32 [B], accept_path int32 [B,path_stride], next_token int32 [B])"""
    dt = _dt(logits)
    B, T_max, vocab = logits.shape
    _dev(logits, logits.dtype, "logits")
    if tree.B != B or tree.T_max != T_max:
        raise ValueError("tree and logits disagree on B or T_max")
    if path_stride is None:
        path_stride = T_max
    dev = logits.device
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty((B, path_stride), dtype=torch.int32, device=dev)
    next_token = torch.empty(B, dtype=torch.int32, device=dev)
    ws = _workspace(workspace_bytes(WS_ACCEPT_PATH, B, T_max, vocab=vocab), dev, workspace)
    c_tree = tree._c()
    _check(load_library().propd_accept_path(
        ctypes.byref(c_tree), dt, vocab, _ptr(logits), _ptr(accept_len), _ptr(path), path_stride,
        _ptr(next_token), _ptr(ws), ws.numel() * ws.element_size(), _stream()),
        "propd_accept_path")
    return accept_len, path, next_token


STATIC_ACCEPT_MAX_NODES = 8192


def propd_accept_path_static(tree: Tree, logits: torch.Tensor, accept_len: torch.Tensor,
                             accept_path: torch.Tensor, next_token: torch.Tensor) -> None:
    """The allocation-free form of ``propd_accept_path``: the caller passes every output
    (int32 [B], [B,path_stride], [B]); the library's own fixed device array is the scratch."""
    dt = _dt(logits)
    B, T_max, vocab = logits.shape
    _dev(logits, logits.dtype, "logits")
    for t, name in ((accept_len, "accept_len"), (accept_path, "accept_path"), (next_token, "next_token")):
        _dev(t, torch.int32, name)
    if tree.B != B or tree.T_max != T_max or accept_len.numel() != B or next_token.numel() != B \
            or accept_path.dim() != 2 or accept_path.shape[0] != B:
        raise ValueError("accept_path_static: shapes disagree")
    c_tree = tree._c()
    _check(load_library().propd_accept_path_static(
        ctypes.byref(c_tree), dt, vocab, _ptr(logits), _ptr(accept_len), _ptr(accept_path),
        accept_path.shape[1], _ptr(next_token), _stream()), "propd_accept_path_static")


def propd_commit_path(tree: Tree, accept_len: torch.Tensor, accept_path: torch.Tensor,
                      next_token: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor,
                      k_cache: torch.Tensor, v_cache: torch.Tensor, seq_lens: torch.Tensor,
                      out_stride: Optional[int] = None) -> torch.Tensor:
    """Appends the accepted nodes' K/V rows to the caches IN PLACE, advances ``seq_lens`` in
    place and returns the step's tokens, int32 [B,out_stride], -1 padded."""
    dt = _dt(k_tree)
    B, H, T_max, d = k_tree.shape
    L_max = k_cache.shape[2]
    for t, name in ((k_tree, "k_tree"), (v_tree, "v_tree"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _dev(t, k_tree.dtype, name)
    for t, name in ((accept_len, "accept_len"), (accept_path, "accept_path"),
                    (next_token, "next_token"), (seq_lens, "seq_lens")):
        _dev(t, torch.int32, name)
    if tuple(v_tree.shape) != (B, H, T_max, d) or tuple(k_cache.shape) != (B, H, L_max, d) or \
            tuple(v_cache.shape) != (B, H, L_max, d) or tree.B != B or tree.T_max != T_max:
        raise ValueError("commit_path: tensor shapes disagree")
    path_stride = accept_path.shape[1]
    if out_stride is None:
        out_stride = path_stride
    out = torch.empty((B, out_stride), dtype=torch.int32, device=k_tree.device)
    c_tree = tree._c()
    _check(load_library().propd_commit_path(
        ctypes.byref(c_tree), dt, H, d, _ptr(accept_len), _ptr(accept_path), path_stride,
        _ptr(next_token), _ptr(k_tree), _ptr(v_tree), _ptr(k_cache), _ptr(v_cache), L_max,
        _ptr(seq_lens), _ptr(out), out_stride, _stream()), "propd_commit_path")
    return out


class Controller:
    """Host-side tree-size controller (``propd_controller_*``).  The state is a numpy buffer this
    object owns; every method is one C call with host arrays."""

    def __init__(self, sizes, n_heads: int, k_max: int, alpha: float, lam: float,
                 hit_rate_init=None):
        lib = load_library()
        self.sizes = np.ascontiguousarray(sizes, dtype=np.int32)
        self.n_heads, self.k_max = int(n_heads), int(k_max)
        nbytes = lib.propd_controller_bytes(len(self.sizes), n_heads, k_max)
        if nbytes == 0:
            raise ValueError("controller: dimensions out of range")
        self._state = np.zeros(nbytes // 8 + 1, dtype=np.float64)  # 8-byte aligned
        init = None
        if hit_rate_init is not None:
            init = np.ascontiguousarray(hit_rate_init, dtype=np.float64).reshape(n_heads, k_max)
        _check(lib.propd_controller_init(self._state.ctypes.data, self._state.nbytes,
                                         self.sizes.ctypes.data, len(self.sizes), n_heads, k_max,
                                         alpha, lam, None if init is None else init.ctypes.data),
               "propd_controller_init")

    def observe_time(self, size: int, t: float, now: float) -> None:
        _check(load_library().propd_controller_observe_time(self._state.ctypes.data, size, t, now),
               "propd_controller_observe_time")

    def observe_hit(self, head: int, rank: int) -> None:
        _check(load_library().propd_controller_observe_hit(self._state.ctypes.data, head, rank),
               "propd_controller_observe_hit")

    def fit(self, now: float):
        b0, b1 = ctypes.c_double(), ctypes.c_double()
        _check(load_library().propd_controller_fit(self._state.ctypes.data, now, ctypes.byref(b0),
                                                   ctypes.byref(b1)), "propd_controller_fit")
        return b0.value, b1.value

    def build_tree(self, size: int):
        """-> dict(parent, depth, choice int32 [n], node_value float64 [n], expected_len)"""
        n = ctypes.c_int32()
        parent, depth, choice = (np.full(size, -9, np.int32) for _ in range(3))
        value = np.zeros(size, np.float64)
        total = ctypes.c_double()
        _check(load_library().propd_controller_build_tree(
            self._state.ctypes.data, size, ctypes.byref(n), parent.ctypes.data, depth.ctypes.data,
            choice.ctypes.data, value.ctypes.data, ctypes.byref(total)), "propd_controller_build_tree")
        k = n.value
        return dict(parent=parent[:k], depth=depth[:k], choice=choice[:k], node_value=value[:k],
                    expected_len=total.value)

    def best_size(self, now: float):
        """-> (best size, speed per candidate size, (beta0, beta1))"""
        best = ctypes.c_int32()
        speed = np.zeros(len(self.sizes), np.float64)
        b0, b1 = ctypes.c_double(), ctypes.c_double()
        _check(load_library().propd_controller_best_size(
            self._state.ctypes.data, now, ctypes.byref(best), speed.ctypes.data, ctypes.byref(b0),
            ctypes.byref(b1)), "propd_controller_best_size")
        return best.value, speed, (b0.value, b1.value)
