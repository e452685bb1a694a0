"""ctypes front end of the CPU oracle (``propd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module and
this module never imports the product package.

Arrays are numpy; bf16 tensors are ``uint16`` bit patterns, fp32 tensors are
``float32``.  Attention results come back in float64, not rounded.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "propd_oracle.c")
_LIB = os.path.join(_HERE, "libpropd_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"tensor must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the input (code {rc})")


def threads() -> int:
    return int(lib().propd_oracle_threads())


def set_threads(n: int) -> None:
    lib().propd_oracle_set_threads(ctypes.c_int(int(n)))


def tree_mask(n_nodes, parent):
    """-> (depth int32 [B,T_max], anc uint64 [B,T_max,2])"""
    parent = _c(parent, np.int32)
    n_nodes = _c(n_nodes, np.int32)
    B, T_max = parent.shape
    depth = np.empty((B, T_max), dtype=np.int32)
    anc = np.empty((B, T_max, 2), dtype=np.uint64)
    _check(lib().propd_oracle_tree_mask(B, T_max, _p(n_nodes), _p(parent), _p(depth), _p(anc)),
           "tree_mask")
    return depth, anc


def _attn_common(n_nodes, parent, seq_lens, q, k_cache, v_cache, k_tree, v_tree):
    q = np.ascontiguousarray(q)
    code = _dtype_code(q)
    ts = [np.ascontiguousarray(t) for t in (k_cache, v_cache, k_tree, v_tree)]
    for t in ts:
        if t.dtype != q.dtype:
            raise TypeError("mixed tensor dtypes")
    B, H, T_max, d = q.shape
    L_max = ts[0].shape[2]
    assert ts[0].shape == (B, H, L_max, d) and ts[1].shape == (B, H, L_max, d)
    assert ts[2].shape == (B, H, T_max, d) and ts[3].shape == (B, H, T_max, d)
    return (B, H, T_max, d, L_max, code, _c(n_nodes, np.int32), _c(parent, np.int32),
            _c(seq_lens, np.int32), q, ts)


def tree_attention(n_nodes, parent, seq_lens, q, k_cache, v_cache, k_tree, v_tree, scale,
                   fill=np.nan):
    """-> float64 [B,H,T_max,d]; rows i >= n_nodes[b] hold ``fill``."""
    B, H, T_max, d, L_max, code, n_nodes, parent, seq_lens, q, ts = _attn_common(
        n_nodes, parent, seq_lens, q, k_cache, v_cache, k_tree, v_tree)
    out = np.full((B, H, T_max, d), fill, dtype=np.float64)
    _check(lib().propd_oracle_tree_attention(
        B, H, T_max, d, L_max, code, ctypes.c_double(scale), _p(n_nodes), _p(parent),
        _p(seq_lens), _p(q), _p(ts[0]), _p(ts[1]), _p(ts[2]), _p(ts[3]), _p(out)),
        "tree_attention")
    return out


def tree_attention_rows(n_nodes, parent, seq_lens, q, k_cache, v_cache, k_tree, v_tree, scale,
                        rows):
    """Selected (b, h, i) rows only -> float64 [n_rows, d]."""
    B, H, T_max, d, L_max, code, n_nodes, parent, seq_lens, q, ts = _attn_common(
        n_nodes, parent, seq_lens, q, k_cache, v_cache, k_tree, v_tree)
    rows = _c(rows, np.int32).reshape(-1, 3)
    out = np.empty((rows.shape[0], d), dtype=np.float64)
    _check(lib().propd_oracle_tree_attention_rows(
        B, H, T_max, d, L_max, code, ctypes.c_double(scale), _p(n_nodes), _p(parent),
        _p(seq_lens), _p(q), _p(ts[0]), _p(ts[1]), _p(ts[2]), _p(ts[3]),
        ctypes.c_int64(rows.shape[0]), _p(rows), _p(out)), "tree_attention_rows")
    return out


def validate_tree(n_nodes, parent, depth=None, anc=None):
    """Flags per sequence for the debug check of a tree (Section 2: node 0 is the root, every
    other node hangs below an earlier node; the mask row of a node is its root path):
    1 size outside [1, T_max], 2 parent array not topological, 4 depth wrong, 8 mask wrong.
    depth and the mask are compared with what the parent pointers give, every climb stopping
    at a pointer that does not lead towards the root."""
    n_nodes, parent = np.asarray(n_nodes), np.asarray(parent)
    B, T_max = parent.shape
    flags = np.zeros(B, np.int32)
    for b in range(B):
        T_raw = int(n_nodes[b])
        if T_raw < 1 or T_raw > T_max:
            flags[b] |= 1
        T = min(max(T_raw, 1), T_max)
        for i in range(T):
            p = int(parent[b, i])
            if (p != -1) if i == 0 else not (0 <= p < i):
                flags[b] |= 2
            path, x = [], i
            while 0 <= x < T and len(path) < T:
                path.append(x)
                up = int(parent[b, x])
                x = up if up < x else -1
            if depth is not None and int(depth[b, i]) != len(path) - 1:
                flags[b] |= 4
            if anc is not None:
                lo = sum(1 << x for x in path if x < 64)
                hi = sum(1 << (x - 64) for x in path if x >= 64)
                if int(anc[b, i, 0]) != lo or int(anc[b, i, 1]) != hi:
                    flags[b] |= 8
    return flags


def early_head_rank(n_nodes, parent, token, hidden_states, head_weight, top_k):
    """-> (rank int32 [B,T_max], margin float64 [B,T_max]); head_weight is [V, Hd]."""
    hidden_states = np.ascontiguousarray(hidden_states)
    head_weight = np.ascontiguousarray(head_weight)
    code = _dtype_code(hidden_states)
    if head_weight.dtype != hidden_states.dtype:
        raise TypeError("mixed tensor dtypes")
    B, T_max, Hd = hidden_states.shape
    V = head_weight.shape[0]
    assert head_weight.shape == (V, Hd)
    n_nodes, parent, token = _c(n_nodes, np.int32), _c(parent, np.int32), _c(token, np.int32)
    rank = np.empty((B, T_max), dtype=np.int32)
    margin = np.empty((B, T_max), dtype=np.float64)
    _check(lib().propd_oracle_early_head_rank(
        B, T_max, Hd, V, code, int(top_k), _p(n_nodes), _p(parent), _p(token),
        _p(hidden_states), _p(head_weight), _p(rank), _p(margin)), "early_head_rank")
    return rank, margin


def early_head_logprob(n_nodes, parent, token, hidden_states, head_weight):
    """-> (logq, logm) float64 [B,T_max]: log of the head's predicted probability of every node's
    token given its parent, and its sum along the root path (the sequence's log marginal)."""
    hidden_states = np.ascontiguousarray(hidden_states)
    head_weight = np.ascontiguousarray(head_weight)
    code = _dtype_code(hidden_states)
    if head_weight.dtype != hidden_states.dtype:
        raise TypeError("mixed tensor dtypes")
    B, T_max, Hd = hidden_states.shape
    V = head_weight.shape[0]
    assert head_weight.shape == (V, Hd)
    n_nodes, parent, token = _c(n_nodes, np.int32), _c(parent, np.int32), _c(token, np.int32)
    logq = np.empty((B, T_max), dtype=np.float64)
    logm = np.empty((B, T_max), dtype=np.float64)
    _check(lib().propd_oracle_early_head_logprob(
        B, T_max, Hd, V, code, _p(n_nodes), _p(parent), _p(token), _p(hidden_states),
        _p(head_weight), _p(logq), _p(logm)), "early_head_logprob")
    return logq, logm


def prob_fail_flags(n_nodes, logm, threshold=None, keep_count=None):
    """The probability-based decision (Section 4.1): a sequence goes when its marginal is below
    `threshold`, or (keep_count given) when it is not among the `keep_count` most probable
    sequences of its tree (equal marginals: the lower node index first).  Returns an int32
    [B,T_max] array, 1 = pruned by the criterion, 0 = kept; the root is always 0.  Shaped as a
    `rank` for prune_compact(..., top_k=1), which then removes what hangs below a pruned node
    (nothing more: marginals never grow along a path)."""
    logm = np.asarray(logm, np.float64)
    B, T_max = logm.shape
    fail = np.zeros((B, T_max), np.int32)
    log_thr = -np.inf if not threshold else float(np.log(threshold))
    for b in range(B):
        T = int(n_nodes[b])
        for i in range(1, T):
            if keep_count is None:
                fail[b, i] = 0 if logm[b, i] >= log_thr else 1
            else:
                ahead = sum(1 for j in range(T)
                            if logm[b, j] > logm[b, i] or (logm[b, j] == logm[b, i] and j < i))
                fail[b, i] = 0 if ahead < keep_count else 1
    return fail


def prune_compact(n_nodes, parent, token, rank, top_k):
    """-> dict with keep_bits, new_index, orig_index, n_kept, cu_nodes and the compacted tree."""
    n_nodes, parent = _c(n_nodes, np.int32), _c(parent, np.int32)
    token, rank = _c(token, np.int32), _c(rank, np.int32)
    B, T_max = parent.shape
    out = dict(
        keep_bits=np.empty((B, 2), np.uint64), new_index=np.empty((B, T_max), np.int32),
        orig_index=np.empty((B, T_max), np.int32), n_kept=np.empty(B, np.int32),
        cu_nodes=np.empty(B + 1, np.int32), parent=np.empty((B, T_max), np.int32),
        token=np.empty((B, T_max), np.int32), depth=np.empty((B, T_max), np.int32),
        anc=np.empty((B, T_max, 2), np.uint64))
    _check(lib().propd_oracle_prune_compact(
        B, T_max, int(top_k), _p(n_nodes), _p(parent), _p(token), _p(rank),
        _p(out["keep_bits"]), _p(out["new_index"]), _p(out["orig_index"]), _p(out["n_kept"]),
        _p(out["cu_nodes"]), _p(out["parent"]), _p(out["token"]), _p(out["depth"]),
        _p(out["anc"])), "prune_compact")
    return out


def gather_rows(src: np.ndarray, orig_index, n_kept, fill_from: Optional[np.ndarray] = None):
    """src [B, (outer,) T_max, cols] -> same shape, survivors first; the rest from ``fill_from``."""
    src = np.ascontiguousarray(src)
    if src.ndim == 3:
        B, T_max, cols = src.shape
        outer = 1
    else:
        B, outer, T_max, cols = src.shape
    dst = np.zeros_like(src) if fill_from is None else np.ascontiguousarray(fill_from).copy()
    row_bytes = cols * src.itemsize
    _check(lib().propd_oracle_gather_rows(
        B, ctypes.c_int64(outer), T_max, ctypes.c_int64(row_bytes),
        ctypes.c_int64(outer * T_max * row_bytes), ctypes.c_int64(T_max * row_bytes),
        ctypes.c_int64(row_bytes), _p(_c(orig_index, np.int32)), _p(_c(n_kept, np.int32)),
        _p(src), _p(dst)), "gather_rows")
    return dst


def accept_path(n_nodes, parent, token, logits, path_stride: Optional[int] = None):
    """-> (accept_len int32 [B], accept_path int32 [B,path_stride], next_token int32 [B])"""
    logits = np.ascontiguousarray(logits)
    code = _dtype_code(logits)
    B, T_max, V = logits.shape
    if path_stride is None:
        path_stride = T_max
    n_nodes, parent, token = _c(n_nodes, np.int32), _c(parent, np.int32), _c(token, np.int32)
    accept_len = np.empty(B, np.int32)
    path = np.empty((B, path_stride), np.int32)
    next_token = np.empty(B, np.int32)
    _check(lib().propd_oracle_accept_path(
        B, T_max, V, code, _p(n_nodes), _p(parent), _p(token), _p(logits), _p(accept_len),
        _p(path), int(path_stride), _p(next_token)), "accept_path")
    return accept_len, path, next_token


def commit_path(n_nodes, token, accept_len, accept_path_, next_token, k_tree, v_tree, k_cache,
                v_cache, seq_lens, out_stride: Optional[int] = None):
    """Appends the accepted nodes' K/V rows to copies of the caches.
    -> (k_cache, v_cache, seq_lens, out_tokens [B,out_stride])"""
    k_tree, v_tree = np.ascontiguousarray(k_tree), np.ascontiguousarray(v_tree)
    k_cache, v_cache = np.array(k_cache, copy=True, order="C"), np.array(v_cache, copy=True, order="C")
    B, H, T_max, d = k_tree.shape
    L_max = k_cache.shape[2]
    n_nodes, token = _c(n_nodes, np.int32), _c(token, np.int32)
    accept_len, path = _c(accept_len, np.int32), _c(accept_path_, np.int32)
    next_token = _c(next_token, np.int32)
    seq = np.array(seq_lens, dtype=np.int32, copy=True)
    if out_stride is None:
        out_stride = path.shape[1]
    out = np.empty((B, out_stride), np.int32)
    _check(lib().propd_oracle_commit_path(
        B, H, d, T_max, L_max, k_tree.dtype.itemsize, _p(n_nodes), _p(token), _p(accept_len),
        _p(path), int(path.shape[1]), _p(next_token), _p(k_tree), _p(v_tree), _p(k_cache),
        _p(v_cache), _p(seq), _p(out), int(out_stride)), "commit_path")
    return k_cache, v_cache, seq, out
