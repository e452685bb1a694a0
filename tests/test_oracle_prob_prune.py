"""Pins of the oracle's probability-based pruning criterion (Section 4.1, "Pruning Criterion"),
CPU only: the head's probabilities against a library log-softmax, the marginal as a product
along the path (normalisation over every token choice of a chain), and the decisions'
invariants (threshold 0 / above 1, monotone in the threshold, rank mode sizes, closure)."""
import itertools

import numpy as np
import torch

from paper_2402_13485_amd import synth


def small_case(rng, B=3, T_max=12, Hd=16, V=11):
    shapes = [synth.random_tree(rng, int(rng.integers(2, T_max + 1))) for _ in range(B)]
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = rng.integers(0, V, size=(B, T_max)).astype(np.int32)
    hid = rng.normal(size=(B, T_max, Hd)).astype(np.float32)
    W = rng.normal(size=(V, Hd)).astype(np.float32) * 0.7
    return n_nodes, parent, token, hid, W


def test_log_probabilities_against_library_log_softmax(oracle):
    rng = np.random.default_rng(11)
    n_nodes, parent, token, hid, W = small_case(rng)
    logq, logm = oracle.early_head_logprob(n_nodes, parent, token, hid, W)
    z = torch.from_numpy(hid.astype(np.float64)) @ torch.from_numpy(W.astype(np.float64)).T
    ref = torch.log_softmax(z, dim=-1).numpy()                     # [B, T_max, V]
    for b in range(len(n_nodes)):
        assert logq[b, 0] == 0.0 and logm[b, 0] == 0.0
        for c in range(1, int(n_nodes[b])):
            p = int(parent[b, c])
            assert abs(logq[b, c] - ref[b, p, token[b, c]]) < 1e-12
            path, j = [], c
            while j > 0:
                path.append(j)
                j = int(parent[b, j])
            want = sum(ref[b, int(parent[b, j]), token[b, j]] for j in path)
            assert abs(logm[b, c] - want) < 1e-11


def test_marginals_of_a_chain_sum_to_one_over_all_token_choices(oracle):
    # the tree is a chain root -> 1 -> 2; the head rows are fixed, so summing the leaf's marginal
    # over every (token_1, token_2) pair must give 1
    rng = np.random.default_rng(12)
    V, Hd = 5, 8
    n_nodes, parent, _ = synth.pad_trees([synth.chain_tree(3)], 3)
    hid = rng.normal(size=(1, 3, Hd)).astype(np.float32)
    W = rng.normal(size=(V, Hd)).astype(np.float32)
    total = 0.0
    for t1, t2 in itertools.product(range(V), repeat=2):
        token = np.array([[0, t1, t2]], np.int32)
        _, logm = oracle.early_head_logprob(n_nodes, parent, token, hid, W)
        total += np.exp(logm[0, 2])
    assert abs(total - 1.0) < 1e-12


def test_a_dominant_score_gives_probability_one(oracle):
    # one-hot hidden state times a weight matrix with one huge entry: that token's q -> 1
    n_nodes, parent, _ = synth.pad_trees([synth.star_tree(4)], 4)
    hid = np.zeros((1, 4, 4), np.float32)
    hid[0, 0, 2] = 1.0
    W = np.zeros((6, 4), np.float32)
    W[3, 2] = 60.0
    token = np.array([[0, 3, 1, 3]], np.int32)
    logq, logm = oracle.early_head_logprob(n_nodes, parent, token, hid, W)
    assert abs(logq[0, 1]) < 1e-12 and abs(logq[0, 3]) < 1e-12
    assert abs(logq[0, 2] - (-60.0)) < 1e-9                        # exp(0) / exp(60), five ids tie at 0


def test_decisions(oracle):
    rng = np.random.default_rng(13)
    n_nodes, parent, token, hid, W = small_case(rng, B=6, T_max=14, V=7)
    _, logm = oracle.early_head_logprob(n_nodes, parent, token, hid, W)
    B, T_max = logm.shape
    valid = np.arange(T_max)[None, :] < n_nodes[:, None]
    # marginals never grow along a path
    for b in range(B):
        for c in range(1, int(n_nodes[b])):
            assert logm[b, c] <= logm[b, parent[b, c]]
    assert (oracle.prob_fail_flags(n_nodes, logm, threshold=0.0) == 0).all()
    above_one = oracle.prob_fail_flags(n_nodes, logm, threshold=1.5)
    assert (above_one[:, 0] == 0).all() and above_one[valid].sum() == valid.sum() - B   # root only
    prev = np.zeros((B, T_max), np.int32)
    for thr in (1e-6, 1e-4, 1e-2, 0.1, 0.5):                       # monotone in the threshold
        f = oracle.prob_fail_flags(n_nodes, logm, threshold=thr)
        assert (f >= prev).all()
        prev = f
        # the kept set is closed under taking parents, so compaction removes nothing further
        c = oracle.prune_compact(n_nodes, parent, token, f, 1)
        assert (c["n_kept"] == (valid & (f == 0)).sum(axis=1)).all()
    for R in (1, 2, 5, 14, 50):
        f = oracle.prob_fail_flags(n_nodes, logm, keep_count=R)
        kept = (valid & (f == 0)).sum(axis=1)
        assert (kept == np.minimum(R, n_nodes)).all()
        c = oracle.prune_compact(n_nodes, parent, token, f, 1)
        assert (c["n_kept"] == kept).all()                          # closed: ties go to the lower index
        for b in range(B):                                          # nothing kept is less probable than something dropped
            T = int(n_nodes[b])
            k = [logm[b, i] for i in range(T) if f[b, i] == 0]
            d = [logm[b, i] for i in range(T) if f[b, i] == 1]
            assert not d or min(k) >= max(d)
