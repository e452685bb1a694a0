"""Seeded synthetic inputs shaped like the paper's verification workloads.

The paper evaluates on Vicuna 7b/13b/33b with prompts from three public
conversation sets (Section 5.1); neither the weights, the trained heads nor the
prompts are available to this build, so every tensor here is a seeded random
stand-in that keeps only shapes, dtypes, value distributions and tree structure.

This module serves both the CPU oracle and the HIP path and therefore holds no
verification arithmetic: it draws random tensors, builds token trees and decides
which token ids to place where.  It imports neither of the two.

Random streams: ``numpy.random.PCG64(20240213 + 1000*config + stream)``.
bf16 tensors are fp32 draws rounded once (round-to-nearest-even) to bf16 and are
carried as ``uint16`` bit patterns so that both sides see identical bits.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass, field
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20240213
MAX_TREE = 128

# --------------------------------------------------------------------------
# random streams and bf16 bit handling
# --------------------------------------------------------------------------


def rng_for(config: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + stream))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal_f32(rng: np.random.Generator, shape, sigma: float = 1.0) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    return out


def normal_bf16(rng: np.random.Generator, shape, sigma: float = 1.0,
                chunk: int = 1 << 24) -> np.ndarray:
    """N(0, sigma^2) rounded to bf16, generated in chunks to bound peak memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = f32_to_bf16_bits(normal_f32(rng, e - s, sigma))
    return out.reshape(shape)


BF16_NAN = np.uint16(0x7FC0)

# --------------------------------------------------------------------------
# token trees
# --------------------------------------------------------------------------


@dataclass
class TreeShape:
    """A prefix-closed set of child-rank tuples in breadth-first order."""
    ranks: List[Tuple[int, ...]]
    parent: np.ndarray  # int32 [T], parent[0] = -1, parent[i] < i
    depth: np.ndarray   # int32 [T]
    score: List[Fraction] = field(default_factory=list)

    @property
    def T(self) -> int:
        return len(self.ranks)


def rank_product_tree(T: int, D: int, R: int = 10) -> TreeShape:
    """Root plus the T-1 best child-rank tuples of length <= D.

    A node is the tuple of child ranks on its root path; rank r has weight
    p_r = (1/(r+1)) / H_R with H_R = sum_{r<R} 1/(r+1); a tuple scores the
    product of its weights (the node value of Section 4.2.2, under which the
    best T-node prefix-closed tree is exactly the T highest-scoring tuples).
    Scores are compared exactly (rationals); equal scores are ordered by shorter
    depth, then lexicographically.  Nodes are stored sorted by (depth, tuple),
    which is breadth-first and makes every parent index smaller than its
    children's.
    """
    if T < 1:
        raise ValueError("T >= 1")
    H_R = sum(Fraction(1, r + 1) for r in range(R))
    p = [Fraction(1, r + 1) / H_R for r in range(R)]
    chosen: Dict[Tuple[int, ...], Fraction] = {(): Fraction(1)}
    # max-heap on (score, -len, tuple-lexicographic reversed) via negation
    heap: List[Tuple[Fraction, int, Tuple[int, ...]]] = []

    def push(t: Tuple[int, ...], s: Fraction) -> None:
        heapq.heappush(heap, (-s, len(t), t))

    if D >= 1:
        push((0,), p[0])
    while len(chosen) < T and heap:
        neg, _, t = heapq.heappop(heap)
        s = -neg
        chosen[t] = s
        # next sibling
        if t[-1] + 1 < R:
            push(t[:-1] + (t[-1] + 1,), s / p[t[-1]] * p[t[-1] + 1])
        # first child
        if len(t) < D:
            push(t + (0,), s * p[0])
    if len(chosen) < T:
        raise ValueError(f"tree with depth<={D}, ranks<{R} has only {len(chosen)} nodes")
    ranks = sorted(chosen.keys(), key=lambda t: (len(t), t))
    index = {t: i for i, t in enumerate(ranks)}
    parent = np.array([-1 if not t else index[t[:-1]] for t in ranks], dtype=np.int32)
    depth = np.array([len(t) for t in ranks], dtype=np.int32)
    return TreeShape(ranks, parent, depth, [chosen[t] for t in ranks])


def chain_tree(T: int) -> TreeShape:
    ranks = [tuple([0] * i) for i in range(T)]
    return TreeShape(ranks, np.arange(-1, T - 1, dtype=np.int32), np.arange(T, dtype=np.int32))


def star_tree(T: int) -> TreeShape:
    ranks = [()] + [(i,) for i in range(T - 1)]
    parent = np.zeros(T, dtype=np.int32)
    parent[0] = -1
    depth = np.ones(T, dtype=np.int32)
    depth[0] = 0
    return TreeShape(ranks, parent, depth)


def random_tree(rng: np.random.Generator, T: int, max_depth: Optional[int] = None) -> TreeShape:
    """Random topologically ordered tree (parent[i] < i), re-sorted breadth-first."""
    par = [-1]
    dep = [0]
    for i in range(1, T):
        while True:
            p = int(rng.integers(0, i))
            if max_depth is None or dep[p] < max_depth:
                break
        par.append(p)
        dep.append(dep[p] + 1)
    # give every node its rank tuple, then sort (depth, tuple)
    nchild = [0] * T
    tup: List[Tuple[int, ...]] = [()] * T
    for i in range(1, T):
        tup[i] = tup[par[i]] + (nchild[par[i]],)
        nchild[par[i]] += 1
    ranks = sorted(tup, key=lambda t: (len(t), t))
    index = {t: i for i, t in enumerate(ranks)}
    parent = np.array([-1 if not t else index[t[:-1]] for t in ranks], dtype=np.int32)
    depth = np.array([len(t) for t in ranks], dtype=np.int32)
    return TreeShape(ranks, parent, depth)


def pad_trees(shapes: Sequence[TreeShape], T_max: int):
    """Stack per-sequence trees into padded [B, T_max] arrays (padding = -1)."""
    B = len(shapes)
    n_nodes = np.array([s.T for s in shapes], dtype=np.int32)
    if n_nodes.max() > T_max:
        raise ValueError("tree larger than T_max")
    parent = np.full((B, T_max), -1, dtype=np.int32)
    depth = np.full((B, T_max), -1, dtype=np.int32)
    for b, s in enumerate(shapes):
        parent[b, : s.T] = s.parent
        depth[b, : s.T] = s.depth
    return n_nodes, parent, depth


def children_lists(parent_row: np.ndarray, T: int) -> List[List[int]]:
    ch: List[List[int]] = [[] for _ in range(T)]
    for c in range(1, T):
        ch[int(parent_row[c])].append(c)
    return ch


def draw_tokens(rng: np.random.Generator, n_nodes: np.ndarray, parent: np.ndarray,
                vocab: int) -> np.ndarray:
    """Random token ids, distinct among siblings (a trie never repeats a child)."""
    B, T_max = parent.shape
    token = np.full((B, T_max), -1, dtype=np.int32)
    for b in range(B):
        T = int(n_nodes[b])
        token[b, 0] = rng.integers(0, vocab)
        for kids in children_lists(parent[b], T):
            if kids:
                if len(kids) > vocab:
                    raise ValueError("more siblings than vocabulary entries")
                token[b, kids] = rng.choice(vocab, size=len(kids), replace=False)
    return token


# --------------------------------------------------------------------------
# token placement for the early-pruning pass
# --------------------------------------------------------------------------


def place_prune_tokens(rng: np.random.Generator, n_nodes: np.ndarray, parent: np.ndarray,
                       hidden: np.ndarray, head_weight: np.ndarray, top_k: int,
                       tau: float, p_pass: float = 0.5):
    """Choose each child's token id so that a chosen share passes the top-k test.

    ``hidden`` [B, T_max, Hd] and ``head_weight`` [V, Hd] are float arrays holding
    exactly the values the two implementations will see.  For every parent the
    early-head scores are formed here only to decide *which ids to hand out*:
    a passing child gets a sibling-unused id whose score lies at least ``tau``
    above the k-th largest-but-one boundary, a failing child one at least
    ``tau`` below it, so that the pass/fail decision does not depend on
    summation order.  Returns (token, wanted_pass) with wanted_pass[b, c] in
    {0, 1} for children and -1 elsewhere.
    """
    B, T_max = parent.shape
    V = head_weight.shape[0]
    W64 = np.ascontiguousarray(head_weight, dtype=np.float64)
    token = np.full((B, T_max), -1, dtype=np.int32)
    wanted = np.full((B, T_max), -1, dtype=np.int8)
    for b in range(B):
        T = int(n_nodes[b])
        token[b, 0] = rng.integers(0, V)
        kids_of = children_lists(parent[b], T)
        par_idx = [p for p in range(T) if kids_of[p]]
        if not par_idx:
            continue
        z_all = np.ascontiguousarray(hidden[b, par_idx], dtype=np.float64) @ W64.T
        for row, p in enumerate(par_idx):
            z = z_all[row]
            order = np.argsort(-z, kind="stable")
            kk = min(top_k, V)
            # boundary values: smallest score inside the list, largest outside
            z_in = z[order[kk - 1]]
            z_out = z[order[kk]] if kk < V else -np.inf
            ok_pass = [int(v) for v in order[:kk] if z[v] - z_out >= tau]
            ok_fail = [int(v) for v in order[kk:] if z_in - z[v] >= tau]
            rng.shuffle(ok_pass)
            # failing ids: a bounded random sample keeps this cheap for big V
            if len(ok_fail) > 4 * len(kids_of[p]) + 8:
                pick = rng.choice(len(ok_fail), size=4 * len(kids_of[p]) + 8, replace=False)
                ok_fail = [ok_fail[i] for i in pick]
            else:
                rng.shuffle(ok_fail)
            for c in kids_of[p]:
                want = bool(rng.random() < p_pass)
                if want and ok_pass:
                    token[b, c] = ok_pass.pop()
                    wanted[b, c] = 1
                elif ok_fail:
                    token[b, c] = ok_fail.pop()
                    wanted[b, c] = 0
                elif ok_pass:
                    token[b, c] = ok_pass.pop()
                    wanted[b, c] = 1
                else:
                    raise ValueError("no token id with the requested margin is left")
    return token, wanted


# --------------------------------------------------------------------------
# final logits with a planted accepted chain
# --------------------------------------------------------------------------


def plant_accept_chain(rng: np.random.Generator, logits: np.ndarray, n_nodes: np.ndarray,
                       parent: np.ndarray, token: np.ndarray, geometric_p: float = 0.45):
    """Overwrite entries of float ``logits`` [B, T_max, V] so that a chosen chain is accepted.

    Per sequence: pick a random leaf, cut its root path after a
    Geometric(p)-distributed number of steps, and along the kept chain raise the
    logit of the next node's token to (row maximum + 1) at each chain node.  At
    the chain's end the raised id is one that no child of that node carries, so
    the chain stops there.  Returns the list of planted chains (node indices).
    """
    B, T_max, V = logits.shape
    chains = []
    for b in range(B):
        T = int(n_nodes[b])
        kids_of = children_lists(parent[b], T)
        leaves = [i for i in range(T) if not kids_of[i]]
        leaf = int(leaves[int(rng.integers(0, len(leaves)))])
        path = []
        x = leaf
        while x >= 0:
            path.append(x)
            x = int(parent[b, x])
        path.reverse()
        steps = int(rng.geometric(geometric_p)) - 1
        chain = path[: min(len(path), steps + 1)]
        for a, node in enumerate(chain):
            row = logits[b, node]
            top = float(row.max()) + 1.0
            if a + 1 < len(chain):
                row[token[b, chain[a + 1]]] = top
            else:
                used = {int(token[b, c]) for c in kids_of[node]}
                free = [v for v in range(V) if v not in used] if len(used) * 2 >= V else None
                if free is None:
                    while True:
                        v = int(rng.integers(0, V))
                        if v not in used:
                            break
                    row[v] = top
                elif free:
                    row[free[int(rng.integers(0, len(free)))]] = top
        chains.append(chain)
    return chains


# --------------------------------------------------------------------------
# workload descriptions (the five benchmark configurations)
# --------------------------------------------------------------------------


@dataclass
class Workload:
    index: int
    name: str
    dtype: str          # "f32" or "bf16"
    B: int
    H: int
    d: int
    T_max: int
    hidden: int
    vocab: int
    top_k: int          # 0 = no pruning in this workload
    tau: float


WORKLOADS = {
    1: Workload(1, "c1_tiny_f32", "f32", 1, 1, 64, 16, 64, 256, 4, 1e-5),
    2: Workload(2, "c2_7b_b1_t64", "bf16", 1, 32, 128, 64, 4096, 32000, 0, 1e-3),
    3: Workload(3, "c3_7b_b4_prune", "bf16", 4, 32, 128, 64, 4096, 32000, 10, 1e-3),
    4: Workload(4, "c4_13b_b16_t128", "bf16", 16, 40, 128, 128, 5120, 32000, 8, 1e-3),
    5: Workload(5, "c5_ragged_b32", "bf16", 32, 32, 128, 128, 4096, 32000, 10, 1e-3),
}

_TREE_DEPTH = {16: 3, 32: 4, 64: 4, 96: 5, 128: 5}


def workload_seq_lens(w: Workload) -> np.ndarray:
    rng = rng_for(w.index, 0)
    if w.index == 1:
        return np.full(w.B, 128, dtype=np.int32)
    if w.index == 2:
        return np.full(w.B, 1024, dtype=np.int32)
    if w.index == 3:
        return rng.integers(512, 2049, size=w.B).astype(np.int32)
    if w.index == 4:
        return np.full(w.B, 4096, dtype=np.int32)
    if w.index == 5:
        u = rng.uniform(np.log(512.0), np.log(8192.0), size=w.B)
        return np.rint(np.exp(u)).astype(np.int32)
    raise ValueError(w.index)


def workload_trees(w: Workload) -> List[TreeShape]:
    rng = rng_for(w.index, 1)
    if w.index == 5:
        sizes = rng.choice([16, 32, 64, 96, 128], size=w.B)
    else:
        sizes = [w.T_max] * w.B
    cache: Dict[int, TreeShape] = {}
    out = []
    for T in sizes:
        T = int(T)
        if T not in cache:
            cache[T] = rank_product_tree(T, _TREE_DEPTH[T])
        out.append(cache[T])
    return out


def _tensor(rng, shape, dtype: str, sigma: float = 1.0):
    return normal_f32(rng, shape, sigma) if dtype == "f32" else normal_bf16(rng, shape, sigma)


def as_float(x: np.ndarray) -> np.ndarray:
    """View a generated tensor (fp32 array or bf16 bit patterns) as float32 values."""
    return bf16_bits_to_f32(x) if x.dtype == np.uint16 else x


def from_float(x: np.ndarray, dtype: str) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32) if dtype == "f32" else f32_to_bf16_bits(x)


def poison_padding(x: np.ndarray, valid: np.ndarray) -> None:
    """Overwrite rows at or beyond valid[b] with NaN, in place.

    x is [B, ..., rows, cols]; rows >= valid[b] are never data, and NaN there
    makes any implementation that lets them leak into a result fail loudly.
    """
    nan = BF16_NAN if x.dtype == np.uint16 else np.float32(np.nan)
    for b in range(x.shape[0]):
        x[b][..., int(valid[b]):, :] = nan


def make_attention_inputs(w: Workload, seq_lens: Optional[np.ndarray] = None,
                          L_max: Optional[int] = None, poison: bool = True,
                          B: Optional[int] = None, H: Optional[int] = None,
                          trees: Optional[List[TreeShape]] = None):
    """q, KV cache and tree K/V for one workload (optionally reduced in B / H)."""
    B = w.B if B is None else B
    H = w.H if H is None else H
    if seq_lens is None:
        seq_lens = workload_seq_lens(w)[:B]
    if trees is None:
        trees = workload_trees(w)[:B]
    n_nodes, parent, depth = pad_trees(trees, w.T_max)
    if L_max is None:
        L_max = int(seq_lens.max())
    rng = rng_for(w.index, 2)
    q = _tensor(rng, (B, H, w.T_max, w.d), w.dtype)
    k_tree = _tensor(rng, (B, H, w.T_max, w.d), w.dtype)
    v_tree = _tensor(rng, (B, H, w.T_max, w.d), w.dtype)
    k_cache = _tensor(rng, (B, H, L_max, w.d), w.dtype)
    v_cache = _tensor(rng, (B, H, L_max, w.d), w.dtype)
    if poison:
        poison_padding(k_cache, seq_lens)
        poison_padding(v_cache, seq_lens)
        for t in (q, k_tree, v_tree):
            poison_padding(t, n_nodes)
    return dict(B=B, H=H, d=w.d, T_max=w.T_max, L_max=L_max, dtype=w.dtype,
                scale=float(1.0 / np.sqrt(w.d)), seq_lens=seq_lens.astype(np.int32),
                n_nodes=n_nodes, parent=parent, depth=depth,
                q=q, k_cache=k_cache, v_cache=v_cache, k_tree=k_tree, v_tree=v_tree)


def make_prune_inputs(w: Workload, B: Optional[int] = None,
                      trees: Optional[List[TreeShape]] = None,
                      hidden: Optional[int] = None, vocab: Optional[int] = None,
                      top_k: Optional[int] = None, p_pass: float = 0.5):
    """Early-layer hidden states, head weight [V, Hd] and margin-guarded tokens."""
    B = w.B if B is None else B
    Hd = w.hidden if hidden is None else hidden
    V = w.vocab if vocab is None else vocab
    k = w.top_k if top_k is None else top_k
    if trees is None:
        trees = workload_trees(w)[:B]
    n_nodes, parent, depth = pad_trees(trees, w.T_max)
    rng = rng_for(w.index, 3)
    hidden_states = _tensor(rng, (B, w.T_max, Hd), w.dtype)
    head_weight = _tensor(rng, (V, Hd), w.dtype, 0.02)
    token, wanted = place_prune_tokens(rng, n_nodes, parent, as_float(hidden_states),
                                       as_float(head_weight), k, w.tau, p_pass)
    poison_padding(hidden_states, n_nodes)
    return dict(B=B, T_max=w.T_max, hidden=Hd, vocab=V, top_k=k, dtype=w.dtype,
                n_nodes=n_nodes, parent=parent, depth=depth, token=token,
                wanted_pass=wanted, hidden_states=hidden_states, head_weight=head_weight)


def make_accept_inputs(w: Workload, n_nodes: np.ndarray, parent: np.ndarray,
                       token: np.ndarray, vocab: Optional[int] = None):
    """Final-layer logits [B, T_max, V] with one planted accepted chain per sequence."""
    V = w.vocab if vocab is None else vocab
    B, T_max = parent.shape
    rng = rng_for(w.index, 4)
    vals = as_float(_tensor(rng, (B, T_max, V), w.dtype)).copy()
    chains = plant_accept_chain(rng, vals, n_nodes, parent, token)
    logits = from_float(vals, w.dtype)
    poison_padding(logits, n_nodes)
    return dict(vocab=V, logits=logits, chains=chains)
