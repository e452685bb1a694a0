"""CPU oracle of the dynamic token-tree generation controller (Section 4.2).

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and by the smoke check / the benchmark's CPU
leg if they ever need it).  The product package never imports this module and this module never
imports the product package.  Plain numpy, float64, the paper's steps in the paper's order.

Notation (Section 4.2): T_perf^i running mean of the iteration time at tree size i, o_i time since
its last update, W_i = exp(-lambda o_i), T_est^i = i beta_1 + beta_0; P_i^k running frequency of
"the true token was within the top-k of head i", p_i^k = P_i^k - P_i^(k-1) the accuracy of the
k-th ranked token of head i; a node reached by choosing rank k_j at head j, j = 0..n, is worth
l = prod_j p_j^(k_j); the root is the token already fixed and is worth 1 (the worked example of
Section 4.2.2 adds up to its printed total only with the root counted as 1).

Pins (tests/test_oracle_controller.py): the three values printed in Section 4.2.2; numpy.polyfit
and exact recovery of a line for the regression; closed form of the running mean under a constant
input; brute force over every prefix-closed node set for the best tree of a size.
"""
from __future__ import annotations

import itertools
import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


class Controller:
    """State of Section 4.2: one T_perf / last-update pair per candidate size, one P table."""

    def __init__(self, sizes: Sequence[int], n_heads: int, k_max: int, alpha: float, lam: float,
                 hit_rate_init: Optional[np.ndarray] = None):
        self.sizes = [int(s) for s in sizes]
        self.n_heads, self.k_max = int(n_heads), int(k_max)
        self.alpha, self.lam = float(alpha), float(lam)
        self.t_perf = {s: None for s in self.sizes}      # None: never observed
        self.last = {s: None for s in self.sizes}
        self.P = np.zeros((n_heads, k_max), np.float64)   # P[i, k-1] = P_i^k
        if hit_rate_init is not None:
            self.P[:] = np.asarray(hit_rate_init, np.float64).reshape(n_heads, k_max)

    # ---- Section 4.2.1, "Update average iteration time"
    def observe_time(self, size: int, t: float, now: float) -> None:
        if self.t_perf[size] is None:
            self.t_perf[size] = float(t)                  # reading: the first sample starts the mean
        else:
            self.t_perf[size] = (1.0 - self.alpha) * self.t_perf[size] + self.alpha * float(t)
        self.last[size] = float(now)

    # ---- Section 4.2.1, "Weighted regression" and "Solve the regression model"
    def fit(self, now: float) -> Tuple[float, float]:
        xs, ys, ws = [], [], []
        for s in self.sizes:
            if self.t_perf[s] is not None:
                xs.append(float(s))
                ys.append(self.t_perf[s])
                ws.append(math.exp(-self.lam * (float(now) - self.last[s])))
        return weighted_line_fit(xs, ys, ws)

    # ---- Section 4.2.2, running top-k hit frequency of a head
    def observe_hit(self, head: int, rank: int) -> None:
        """rank: 0-based position of the true token in the head's list, or -1 when absent."""
        for k in range(1, self.k_max + 1):
            hit = 1.0 if 0 <= rank < k else 0.0
            self.P[head, k - 1] = (1.0 - self.alpha) * self.P[head, k - 1] + self.alpha * hit

    def rank_accuracy(self) -> np.ndarray:
        """p[i, k-1] = P_i^k - P_i^(k-1), with P_i^0 = 0."""
        p = self.P.copy()
        p[:, 1:] -= self.P[:, :-1]
        return p

    # ---- Section 4.2.3
    def best_size(self, now: float):
        beta0, beta1 = self.fit(now)
        p = self.rank_accuracy()
        speeds = []
        for s in self.sizes:
            t_est = beta0 + beta1 * s
            speeds.append(expected_length(p, s) / t_est if t_est > 0.0 else 0.0)
        best = max(range(len(self.sizes)), key=lambda j: (speeds[j], -self.sizes[j]))
        return self.sizes[best], speeds, (beta0, beta1)


def weighted_line_fit(x, y, w) -> Tuple[float, float]:
    """(beta0, beta1) minimising sum_i w_i (y_i - beta0 - beta1 x_i)^2: the normal equations of
    Section 4.2.1 written out.  With fewer than two distinct abscissae the slope is undetermined
    and taken as 0 (beta0 = weighted mean)."""
    x, y, w = (np.asarray(a, np.float64) for a in (x, y, w))
    if x.size == 0:
        raise ValueError("no observation")
    sw, sx, sy = w.sum(), (w * x).sum(), (w * y).sum()
    sxx, sxy = (w * x * x).sum(), (w * x * y).sum()
    den = sw * sxx - sx * sx
    if not den > 1e-12 * sw * sxx:
        return sy / sw, 0.0
    beta1 = (sw * sxy - sx * sy) / den
    beta0 = (sy - beta1 * sx) / sw
    return float(beta0), float(beta1)


def all_nodes(p: np.ndarray) -> List[Tuple[float, Tuple[int, ...]]]:
    """Every candidate sequence (k_0, .., k_n), n < n_heads, with its value prod_j p[j, k_j]."""
    n_heads, k_max = p.shape
    out = []
    for depth in range(1, n_heads + 1):
        for ks in itertools.product(range(k_max), repeat=depth):
            v = 1.0
            for j, k in enumerate(ks):
                v *= p[j, k]
            out.append((v, ks))
    return out


def best_tree(p: np.ndarray, size: int) -> List[Tuple[int, ...]]:
    """The `size - 1` most valuable candidate sequences (the root is the size-th node).  Values
    never grow along a path (every p is at most 1), so with ties broken towards the shorter
    sequence the chosen set is closed under taking prefixes, i.e. a tree."""
    nodes = all_nodes(p)
    nodes.sort(key=lambda vk: (-vk[0], len(vk[1]), vk[1]))
    return [ks for _, ks in nodes[: max(size - 1, 0)]]


def expected_length(p: np.ndarray, size: int) -> float:
    """l(size): 1 for the root plus the values of the best tree's other nodes."""
    total = 1.0
    for ks in best_tree(p, size):
        v = 1.0
        for j, k in enumerate(ks):
            v *= p[j, k]
        total += v
    return total


def tree_value(p: np.ndarray, seqs) -> float:
    """Estimated acceptance length of a given tree: root + the value of every listed sequence."""
    total = 1.0
    for ks in seqs:
        v = 1.0
        for j, k in enumerate(ks):
            v *= p[j, k]
        total += v
    return total
