"""Pins of the oracle of the dynamic token-tree controller (Section 4.2), CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import tree_controller as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "controller_worked_example.txt")
LETTER = {"b": (0, 0), "c": (0, 1), "d": (1, 0), "e": (1, 1)}  # letter -> (head, rank)


def load_example():
    p, values, tree = [], {}, None
    for line in open(GOLDEN):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "p":
            p.append([float(x) for x in f[1:]])
        elif f[0] == "value":
            values[f[1]] = float(f[2])
        elif f[0] == "tree":
            tree = (f[1].split(","), float(f[2]))
    return np.array(p), values, tree


def seq_of(word):
    """'abe' -> ranks along the path below the root 'a'."""
    return tuple(LETTER[ch][1] for ch in word[1:])


def prefixes(words):
    out = set()
    for w in words:
        for n in range(2, len(w) + 1):
            out.add(seq_of(w[:n]))
    return sorted(out)


def test_worked_example_of_section_4_2_2():
    p, values, (words, total) = load_example()
    for word, v in values.items():
        ks = seq_of(word)
        got = np.prod([p[j, k] for j, k in enumerate(ks)])
        assert got == pytest.approx(v, abs=1e-12), word
    assert oc.tree_value(p, prefixes(words)) == pytest.approx(total, abs=1e-12)
    # the same tree is also the best one of its size under these accuracies
    assert sorted(oc.best_tree(p, 4)) == prefixes(words)
    assert oc.expected_length(p, 4) == pytest.approx(total, abs=1e-12)


def test_rank_accuracy_is_the_difference_of_cumulative_rates():
    c = oc.Controller([8], n_heads=2, k_max=3, alpha=0.5, lam=0.0,
                      hit_rate_init=[[0.6, 0.7, 0.75], [0.3, 0.4, 0.4]])
    np.testing.assert_allclose(c.rank_accuracy(), [[0.6, 0.1, 0.05], [0.3, 0.1, 0.0]], atol=1e-15)


def test_hit_rate_running_mean():
    alpha = 0.2
    c = oc.Controller([8], n_heads=1, k_max=3, alpha=alpha, lam=0.0)
    ranks = [0, 2, -1, 1, 1, 0, 5, 2]
    for r in ranks:
        c.observe_hit(0, r)
    # closed form: P^k = sum_j alpha (1-alpha)^(n-1-j) 1[rank_j < k]
    n = len(ranks)
    for k in (1, 2, 3):
        want = sum(alpha * (1 - alpha) ** (n - 1 - j) for j, r in enumerate(ranks) if 0 <= r < k)
        assert c.P[0, k - 1] == pytest.approx(want, abs=1e-15)
    assert (np.diff(c.P[0]) >= 0).all()                  # cumulative in k
    # a constant input converges geometrically: always in the top-1
    c2 = oc.Controller([8], 1, 2, alpha, 0.0)
    for _ in range(30):
        c2.observe_hit(0, 0)
    assert c2.P[0, 0] == pytest.approx(1 - (1 - alpha) ** 30, abs=1e-15)


def test_iteration_time_running_mean():
    c = oc.Controller([16, 32], 1, 1, alpha=0.25, lam=0.0)
    c.observe_time(16, 4.0, now=0.0)
    assert c.t_perf[16] == 4.0 and c.t_perf[32] is None
    c.observe_time(16, 8.0, now=1.0)
    assert c.t_perf[16] == pytest.approx(0.75 * 4.0 + 0.25 * 8.0)
    # an outlier moves the mean by alpha of its distance only
    c.observe_time(16, 105.0, now=2.0)
    assert c.t_perf[16] == pytest.approx(5.0 + 0.25 * 100.0)


def test_weighted_fit_equals_polyfit_and_recovers_a_line():
    rng = np.random.default_rng(5)
    x = np.array([8, 16, 32, 48, 64, 96, 128], np.float64)
    y = 3.0 + 0.07 * x + rng.normal(scale=0.3, size=x.size)
    w = np.exp(-0.3 * rng.integers(0, 12, size=x.size))
    b0, b1 = oc.weighted_line_fit(x, y, w)
    q1, q0 = np.polyfit(x, y, 1, w=np.sqrt(w))           # polyfit weights multiply the residual
    assert b0 == pytest.approx(q0, rel=1e-9) and b1 == pytest.approx(q1, rel=1e-9)
    # points on a line give that line whatever the weights
    b0, b1 = oc.weighted_line_fit(x, 2.5 + 0.125 * x, w)
    assert b0 == pytest.approx(2.5, abs=1e-9) and b1 == pytest.approx(0.125, abs=1e-11)
    # a stale outlier loses its influence as its weight goes to zero
    y2 = 1.0 + 0.5 * x
    y2[3] += 50.0
    w2 = np.ones_like(x)
    w2[3] = 1e-12
    b0, b1 = oc.weighted_line_fit(x, y2, w2)
    assert b0 == pytest.approx(1.0, abs=1e-6) and b1 == pytest.approx(0.5, abs=1e-8)
    # one size only: slope undetermined -> 0
    assert oc.weighted_line_fit([32.0], [7.0], [0.4]) == (7.0, 0.0)


def test_controller_fit_uses_age_weights():
    lam = 0.5
    c = oc.Controller([8, 16, 32, 64], 1, 1, alpha=1.0, lam=lam)   # alpha = 1: mean = last sample
    for s, t, now in ((8, 1.0, 0.0), (16, 2.5, 3.0), (32, 4.0, 4.0)):
        c.observe_time(s, t, now)
    b0, b1 = c.fit(now=6.0)
    w = np.exp(-lam * np.array([6.0, 3.0, 2.0]))
    q1, q0 = np.polyfit([8, 16, 32], [1.0, 2.5, 4.0], 1, w=np.sqrt(w))
    assert b0 == pytest.approx(q0, rel=1e-9) and b1 == pytest.approx(q1, rel=1e-9)


def closed_subsets(nodes, size):
    """Every prefix-closed set of `size` candidate sequences (brute force)."""
    for sub in itertools.combinations(nodes, size):
        s = set(sub)
        if all(len(ks) == 1 or ks[:-1] in s for ks in sub):
            yield sub


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_best_tree_against_every_tree_of_its_size(seed):
    rng = np.random.default_rng(seed)
    n_heads, k_max = 3, 2
    P = np.sort(rng.random((n_heads, k_max)), axis=1)    # cumulative rates, rising in k
    p = P.copy()
    p[:, 1:] -= P[:, :-1]
    nodes = [ks for _, ks in oc.all_nodes(p)]            # 2 + 4 + 8 sequences
    for size in range(1, 7):
        best = max((oc.tree_value(p, sub) for sub in closed_subsets(nodes, size - 1)), default=1.0)
        assert oc.expected_length(p, size) == pytest.approx(best, abs=1e-12)
        chosen = set(oc.best_tree(p, size))
        assert all(len(ks) == 1 or ks[:-1] in chosen for ks in chosen)


def test_best_size_scans_speed():
    # time = 1 + 0.1 i exactly; accuracies as in the worked example
    p, _, _ = load_example()
    P = np.cumsum(p, axis=1)
    c = oc.Controller([1, 2, 3, 4, 5, 6, 7], n_heads=2, k_max=2, alpha=0.5, lam=0.1, hit_rate_init=P)
    for s in (1, 4, 7):
        c.observe_time(s, 1.0 + 0.1 * s, now=float(s))
    best, speeds, (b0, b1) = c.best_size(now=8.0)
    assert b0 == pytest.approx(1.0) and b1 == pytest.approx(0.1)
    want = [oc.expected_length(p, s) / (1.0 + 0.1 * s) for s in c.sizes]
    np.testing.assert_allclose(speeds, want, rtol=1e-12)
    assert best == c.sizes[int(np.argmax(want))]
    # l(i) = 1, 1.6, 1.78, 1.88, ... over 1.1, 1.2, 1.3, 1.4, ...: 0.909, 1.333, 1.369, 1.343, ...
    assert best == 3
