"""Pins for the oracle's tree mask and tree attention (CPU only).

The oracle is checked against things other than itself: closed forms, a
transitive closure computed with matrix products, the independently derived
shape figures under tests/golden/, and PyTorch's scaled-dot-product attention
(a library routine) for the causal special case, the explicit-mask general case
and per-path linear sequences (Section 2, "Verification").
"""
import os

import numpy as np
import pytest
import torch

from paper_2402_13485_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tree_shapes.txt")


def closure_mask(parent_row, T):
    """Ancestor-or-self relation as a boolean matrix via repeated squaring of (I + A)."""
    A = np.eye(T, dtype=np.int64)
    for i in range(1, T):
        A[i, parent_row[i]] = 1
    R = A.copy()
    for _ in range(8):
        R = ((R @ R) > 0).astype(np.int64)
    return R.astype(bool)


def bits_to_matrix(anc_b, T):
    M = np.zeros((T, T), dtype=bool)
    for i in range(T):
        for j in range(T):
            M[i, j] = (int(anc_b[i, j >> 6]) >> (j & 63)) & 1
    return M


def read_golden():
    rows, parents16 = [], None
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            if parts[0] == "parents16":
                parents16 = [int(x) for x in parts[1].split(",")]
            else:
                rows.append((int(parts[0]), int(parts[1]), [int(x) for x in parts[2].split(",")],
                             int(parts[3]), int(parts[4]), int(parts[5]), float(parts[6])))
    return rows, parents16


# ------------------------------------------------------------------ tree builder + mask


def test_tree_builder_matches_independent_shape_figures(oracle):
    rows, parents16 = read_golden()
    assert synth.rank_product_tree(16, 3).parent.tolist() == parents16
    for T, D, per_depth, internal, max_children, mask_bits, sum_score in rows:
        t = synth.rank_product_tree(T, D)
        assert np.bincount(t.depth, minlength=D + 1).tolist() == per_depth
        assert len(set(t.parent[1:].tolist())) == internal
        assert int(np.bincount(t.parent[1:]).max()) == max_children
        assert abs(float(sum(t.score)) - sum_score) < 5e-5
        n_nodes, parent, _ = synth.pad_trees([t], 128)
        depth, anc = oracle.tree_mask(n_nodes, parent)
        total = sum(bin(int(w)).count("1") for w in anc.reshape(-1))
        assert total == mask_bits
        assert (depth[0, :T] == t.depth).all() and (depth[0, T:] == -1).all()
        assert (anc[0, T:] == 0).all()


def test_mask_closed_forms_chain_and_star(oracle):
    for T in (1, 2, 63, 64, 65, 128):
        n_nodes, parent, _ = synth.pad_trees([synth.chain_tree(T), synth.star_tree(T)], 128)
        depth, anc = oracle.tree_mask(n_nodes, parent)
        for i in range(T):
            want = (1 << (i + 1)) - 1
            got = int(anc[0, i, 0]) | (int(anc[0, i, 1]) << 64)
            assert got == want
            got_star = int(anc[1, i, 0]) | (int(anc[1, i, 1]) << 64)
            assert got_star == (1 | (1 << i))
        assert depth[0, :T].tolist() == list(range(T))
        assert depth[1, :T].tolist() == [0] + [1] * (T - 1)


def test_mask_equals_transitive_closure_on_random_trees(oracle):
    rng = np.random.default_rng(7)
    shapes = [synth.random_tree(rng, int(T)) for T in rng.integers(1, 129, size=24)]
    n_nodes, parent, _ = synth.pad_trees(shapes, 128)
    depth, anc = oracle.tree_mask(n_nodes, parent)
    for b, s in enumerate(shapes):
        M = bits_to_matrix(anc[b], s.T)
        assert (M == closure_mask(parent[b], s.T)).all()
        assert (M.sum(axis=1) == depth[b, : s.T] + 1).all()
        assert (np.triu(M, 1) == 0).all()  # topological order => lower triangular


def test_mask_rejects_malformed_trees(oracle):
    with pytest.raises(ValueError):
        oracle.tree_mask(np.array([3]), np.array([[-1, 0, 2, -1]]))  # parent[2] = 2
    with pytest.raises(ValueError):
        oracle.tree_mask(np.array([2]), np.array([[0, 0]]))  # root must have parent -1


# ------------------------------------------------------------------ attention


def _inputs(rng, B, H, T_max, d, L_max, shapes, seq_lens, bf16=False):
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    mk = (lambda s: synth.normal_bf16(rng, s)) if bf16 else (lambda s: synth.normal_f32(rng, s))
    return dict(n_nodes=n_nodes, parent=parent, seq_lens=np.asarray(seq_lens, np.int32),
                q=mk((B, H, T_max, d)), k_cache=mk((B, H, L_max, d)), v_cache=mk((B, H, L_max, d)),
                k_tree=mk((B, H, T_max, d)), v_tree=mk((B, H, T_max, d)))


def _run(oracle, x, scale):
    return oracle.tree_attention(x["n_nodes"], x["parent"], x["seq_lens"], x["q"], x["k_cache"],
                                 x["v_cache"], x["k_tree"], x["v_tree"], scale)


def _t64(a):
    return torch.from_numpy(synth.as_float(a).astype(np.float64))


def sdpa_reference(x, b, scale, mask_tree):
    """Library attention over [cache ; tree] with an explicit boolean mask."""
    T = int(x["n_nodes"][b])
    L = int(x["seq_lens"][b])
    q = _t64(x["q"][b, :, :T])
    k = torch.cat([_t64(x["k_cache"][b, :, :L]), _t64(x["k_tree"][b, :, :T])], dim=1)
    v = torch.cat([_t64(x["v_cache"][b, :, :L]), _t64(x["v_tree"][b, :, :T])], dim=1)
    mask = torch.cat([torch.ones(T, L, dtype=torch.bool), torch.from_numpy(mask_tree)], dim=1)
    return torch.nn.functional.scaled_dot_product_attention(
        q, k, v, attn_mask=mask, scale=scale).numpy()


def test_chain_tree_is_causal_attention(oracle):
    """A chain-shaped tree is a linear sequence: the result must be the last T rows of
    ordinary causal attention over the L + T concatenation."""
    rng = np.random.default_rng(1)
    B, H, T, d, L = 2, 3, 9, 16, 21
    x = _inputs(rng, B, H, T, d, L, [synth.chain_tree(T)] * B, [L, L])
    scale = 0.3
    got = _run(oracle, x, scale)
    for b in range(B):
        q_full = torch.cat([_t64(x["k_cache"][b]) * 0, _t64(x["q"][b])], dim=1)  # prefix rows unused
        k = torch.cat([_t64(x["k_cache"][b]), _t64(x["k_tree"][b])], dim=1)
        v = torch.cat([_t64(x["v_cache"][b]), _t64(x["v_tree"][b])], dim=1)
        ref = torch.nn.functional.scaled_dot_product_attention(
            q_full, k, v, is_causal=True, scale=scale)[:, L:].numpy()
        np.testing.assert_allclose(got[b], ref, rtol=1e-12, atol=1e-13)


def test_single_node_is_plain_decode_attention(oracle):
    rng = np.random.default_rng(2)
    x = _inputs(rng, 1, 2, 1, 8, 33, [synth.chain_tree(1)], [33])
    got = _run(oracle, x, 0.5)
    k = torch.cat([_t64(x["k_cache"][0]), _t64(x["k_tree"][0])], dim=1)
    v = torch.cat([_t64(x["v_cache"][0]), _t64(x["v_tree"][0])], dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(_t64(x["q"][0]), k, v, scale=0.5)
    np.testing.assert_allclose(got[0], ref.numpy(), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("bf16", [False, True])
def test_general_trees_match_library_attention_with_explicit_mask(oracle, bf16):
    rng = np.random.default_rng(3)
    shapes = [synth.rank_product_tree(16, 3), synth.random_tree(rng, 11), synth.star_tree(7),
              synth.random_tree(rng, 16)]
    seq_lens = [20, 0, 5, 13]  # includes an empty cache
    x = _inputs(rng, 4, 2, 16, 32, 20, shapes, seq_lens, bf16=bf16)
    synth.poison_padding(x["k_cache"], x["seq_lens"])
    synth.poison_padding(x["v_cache"], x["seq_lens"])
    for name in ("q", "k_tree", "v_tree"):
        synth.poison_padding(x[name], x["n_nodes"])
    scale = 1.0 / np.sqrt(32)
    got = _run(oracle, x, scale)
    for b, s in enumerate(shapes):
        ref = sdpa_reference(x, b, scale, closure_mask(x["parent"][b], s.T))
        np.testing.assert_allclose(got[b, :, : s.T], ref, rtol=1e-11, atol=1e-12)
        assert np.isnan(got[b, :, s.T:]).all()  # rows beyond the tree are not written


def test_each_node_equals_causal_attention_on_its_own_sequence(oracle):
    """Verifying the tree must give every node the result of verifying its candidate
    sequence alone: cache followed by the node's root path, last position."""
    rng = np.random.default_rng(4)
    t = synth.rank_product_tree(32, 4)
    x = _inputs(rng, 1, 2, 32, 16, 17, [t], [17])
    got = _run(oracle, x, 0.25)
    for i in range(t.T):
        path = []
        n = i
        while n >= 0:
            path.append(n)
            n = int(t.parent[n])
        path.reverse()
        k = torch.cat([_t64(x["k_cache"][0]), _t64(x["k_tree"][0][:, path])], dim=1)
        v = torch.cat([_t64(x["v_cache"][0]), _t64(x["v_tree"][0][:, path])], dim=1)
        qq = torch.cat([torch.zeros(2, 17, 16, dtype=torch.float64), _t64(x["q"][0][:, path])], 1)
        ref = torch.nn.functional.scaled_dot_product_attention(qq, k, v, is_causal=True, scale=0.25)
        np.testing.assert_allclose(got[0, :, i], ref[:, -1].numpy(), rtol=1e-12, atol=1e-13)


def test_closed_forms_zero_query_and_constant_value(oracle):
    rng = np.random.default_rng(5)
    t = synth.rank_product_tree(16, 3)
    x = _inputs(rng, 1, 1, 16, 8, 10, [t], [10])
    x0 = dict(x, q=np.zeros_like(x["q"]))
    got = _run(oracle, x0, 1.0)
    for i in range(16):
        path = [i]
        while t.parent[path[-1]] >= 0:
            path.append(int(t.parent[path[-1]]))
        rows = np.concatenate([x["v_cache"][0, 0].astype(np.float64),
                               x["v_tree"][0, 0, path].astype(np.float64)])
        np.testing.assert_allclose(got[0, 0, i], rows.mean(axis=0), rtol=1e-13, atol=1e-14)
    x1 = dict(x, v_cache=np.full_like(x["v_cache"], 1.5), v_tree=np.full_like(x["v_tree"], 1.5))
    np.testing.assert_allclose(_run(oracle, x1, 0.7), 1.5, rtol=1e-14)


def test_sibling_permutation_equivariance(oracle):
    """Swapping two sibling leaves swaps their outputs and changes nothing else."""
    rng = np.random.default_rng(6)
    t = synth.star_tree(6)
    x = _inputs(rng, 1, 1, 6, 8, 7, [t], [7])
    got = _run(oracle, x, 0.4)
    perm = [0, 1, 4, 3, 2, 5]
    y = dict(x)
    for name in ("q", "k_tree", "v_tree"):
        y[name] = np.ascontiguousarray(x[name][:, :, perm])
    got_p = _run(oracle, y, 0.4)
    np.testing.assert_array_equal(got_p[0, 0], got[0, 0, perm])


def test_bf16_inputs_are_widened_exactly(oracle):
    rng = np.random.default_rng(8)
    t = synth.rank_product_tree(16, 3)
    xb = _inputs(rng, 1, 2, 16, 16, 12, [t], [12], bf16=True)
    xf = {k: (synth.bf16_bits_to_f32(v) if v.dtype == np.uint16 else v) for k, v in xb.items()}
    np.testing.assert_array_equal(_run(oracle, xb, 0.25), _run(oracle, xf, 0.25))


def test_rows_entry_matches_full_entry(oracle):
    rng = np.random.default_rng(9)
    shapes = [synth.rank_product_tree(16, 3), synth.random_tree(rng, 9)]
    x = _inputs(rng, 2, 3, 16, 8, 14, shapes, [14, 6])
    full = _run(oracle, x, 0.5)
    rows = np.array([[0, 0, 0], [1, 2, 8], [0, 1, 15], [1, 0, 3]], dtype=np.int32)
    got = oracle.tree_attention_rows(x["n_nodes"], x["parent"], x["seq_lens"], x["q"], x["k_cache"],
                                     x["v_cache"], x["k_tree"], x["v_tree"], 0.5, rows)
    for r, (b, h, i) in enumerate(rows):
        np.testing.assert_array_equal(got[r], full[b, h, i])
    with pytest.raises(ValueError):
        oracle.tree_attention_rows(x["n_nodes"], x["parent"], x["seq_lens"], x["q"], x["k_cache"],
                                   x["v_cache"], x["k_tree"], x["v_tree"], 0.5, [[1, 0, 9]])


def test_validate_tree_flags(oracle):
    """The debug check agrees with tree_mask on sound trees and names each kind of damage."""
    rng = np.random.default_rng(77)
    shapes = [synth.random_tree(rng, int(T)) for T in (1, 2, 17, 70, 128)]
    n_nodes, parent, _ = synth.pad_trees(shapes, 128)
    depth, anc = oracle.tree_mask(n_nodes, parent)
    assert (oracle.validate_tree(n_nodes, parent, depth, anc) == 0).all()
    assert (oracle.validate_tree(n_nodes, parent) == 0).all()
    bad_n = n_nodes.copy(); bad_n[0] = 0; bad_n[1] = 129
    f = oracle.validate_tree(bad_n, parent)
    assert f[0] == 1 and f[1] & 1 and (f[2:] == 0).all()   # 129 nodes: padding is then read as nodes too
    bad_p = parent.copy(); bad_p[2, 0] = 0; bad_p[3, 5] = 5; bad_p[4, 9] = 40
    f = oracle.validate_tree(n_nodes, bad_p, depth, anc)
    assert (f[2:] & 2).all() and (f[:2] == 0).all()
    bad_d = depth.copy(); bad_d[3, 69] += 1
    assert oracle.validate_tree(n_nodes, parent, bad_d, anc).tolist() == [0, 0, 0, 4, 0]
    bad_a = anc.copy(); bad_a[4, 100, 1] ^= np.uint64(1 << 5)
    assert oracle.validate_tree(n_nodes, parent, depth, bad_a).tolist() == [0, 0, 0, 0, 8]
