"""Pins of the oracle's commit step (the decoding-loop step after acceptance), CPU only.

  * the committed cache is exactly what the last accepted node attended to: its tree-attention
    output equals library attention of its query over the committed rows (Section 2: a node
    attends to the prefix and its own root path);
  * many steps of tree verification + commit reproduce plain greedy autoregressive decoding
    with a deterministic toy model, tokens and cache rows alike (Section 5.1: greedy decoding
    guarantees the large model's own output);
  * rows outside the appended range are untouched; a full cache drops what does not fit.
"""
import numpy as np
import torch

from paper_2402_13485_amd import synth
import decode_loop_util as dl


def test_committed_cache_is_the_context_of_the_last_accepted_node(oracle):
    w = synth.Workload(61, "case", "f32", 3, 2, 64, 16, 0, 0, 0, 1e-5)
    rng = np.random.default_rng(61)
    shapes = [synth.rank_product_tree(16, 3), synth.random_tree(rng, 11), synth.chain_tree(5)]
    seq = np.array([37, 0, 9], np.int32)
    x = synth.make_attention_inputs(w, seq_lens=seq, L_max=48, trees=shapes, poison=False)
    ref = oracle.tree_attention(x["n_nodes"], x["parent"], seq, x["q"], x["k_cache"], x["v_cache"],
                                x["k_tree"], x["v_tree"], x["scale"])
    ends = [int(rng.integers(0, int(n))) for n in x["n_nodes"]]
    paths = [dl.root_path(x["parent"][b], ends[b]) for b in range(3)]
    stride = 8
    path = np.full((3, stride), -1, np.int32)
    for b, p in enumerate(paths):
        path[b, : len(p)] = p
    alen = np.array([len(p) for p in paths], np.int32)
    token = np.zeros_like(x["parent"])
    kc, vc, new_len, _ = oracle.commit_path(x["n_nodes"], token, alen, path, np.zeros(3, np.int32),
                                            x["k_tree"], x["v_tree"], x["k_cache"], x["v_cache"], seq)
    assert (new_len == seq + alen).all()
    for b in range(3):
        n = int(new_len[b])
        q = torch.from_numpy(x["q"][b, :, ends[b]].astype(np.float64))[:, None, :]      # [H,1,d]
        k = torch.from_numpy(kc[b, :, :n].astype(np.float64))
        v = torch.from_numpy(vc[b, :, :n].astype(np.float64))
        lib = torch.nn.functional.scaled_dot_product_attention(q, k, v, scale=float(x["scale"]))
        np.testing.assert_allclose(lib[:, 0].numpy(), ref[b, :, ends[b]], rtol=1e-12, atol=1e-12)


def test_many_steps_equal_plain_greedy_decoding(oracle):
    rng = np.random.default_rng(62)
    B, H, d, T_max, L_max, steps = 4, 2, 16, 14, 96, 9
    start = [[int(t) for t in rng.integers(0, dl.VOCAB, size=n)] for n in (3, 0, 7, 1)]
    prefixes = [list(s) for s in start]
    roots = [dl.model_next(p) for p in prefixes]
    k_cache = np.full((B, H, L_max, d), -777.0, np.float32)
    v_cache = np.full((B, H, L_max, d), -777.0, np.float32)
    for b in range(B):
        k_cache[b, :, : len(prefixes[b])] = dl.expected_cache_rows(prefixes[b], H, d, 0, "f32")
        v_cache[b, :, : len(prefixes[b])] = dl.expected_cache_rows(prefixes[b], H, d, 1, "f32")
    seq = np.array([len(p) for p in prefixes], np.int32)
    emitted = [[r] for r in roots]
    lens_seen = []
    for _ in range(steps):
        n_nodes, parent, token, logits, kt, vt = dl.build_step(rng, prefixes, roots, H, d, T_max, "f32")
        alen, path, nxt = oracle.accept_path(n_nodes, parent, token, logits, path_stride=T_max)
        k_cache, v_cache, seq, out = oracle.commit_path(n_nodes, token, alen, path, nxt, kt, vt,
                                                        k_cache, v_cache, seq)
        for b in range(B):
            a = int(alen[b])
            step_tokens = [int(t) for t in out[b, :a]]
            assert (out[b, a:] == -1).all()
            prefixes[b] += [roots[b]] + step_tokens[:-1]   # rows now in the cache
            roots[b] = step_tokens[-1]
            emitted[b] += step_tokens
            lens_seen.append(a)
    assert max(lens_seen) >= 3 and min(lens_seen) == 1     # the loop saw short and long paths
    for b in range(B):
        # plain autoregressive greedy decoding with the same model
        seq_tokens = list(start[b])
        for _ in range(len(emitted[b])):
            seq_tokens.append(dl.model_next(seq_tokens))
        assert emitted[b] == seq_tokens[len(start[b]):]
        n = int(seq[b])
        assert n == len(prefixes[b]) and prefixes[b] == seq_tokens[:n]
        assert (k_cache[b, :, :n] == dl.expected_cache_rows(seq_tokens[:n], H, d, 0, "f32")).all()
        assert (v_cache[b, :, :n] == dl.expected_cache_rows(seq_tokens[:n], H, d, 1, "f32")).all()
        assert (k_cache[b, :, n:] == -777.0).all() and (v_cache[b, :, n:] == -777.0).all()


def test_full_cache_drops_rows_and_other_rows_stay(oracle):
    B, H, d, T_max, L_max = 2, 1, 8, 6, 10
    parent = np.array([[-1, 0, 1, 2, 3, 4]] * B, np.int32)        # chains
    n_nodes = np.array([6, 6], np.int32)
    token = np.arange(B * T_max, dtype=np.int32).reshape(B, T_max) + 100
    kt = np.arange(B * H * T_max * d, dtype=np.float32).reshape(B, H, T_max, d)
    vt = -kt
    kc = np.full((B, H, L_max, d), 5.5, np.float32)
    vc = np.full((B, H, L_max, d), 6.5, np.float32)
    seq = np.array([8, 2], np.int32)
    alen = np.array([4, 3], np.int32)
    path = np.array([[0, 1, 2, 3, -1, -1], [0, 1, 2, -1, -1, -1]], np.int32)
    nxt = np.array([41, 42], np.int32)
    kc2, vc2, seq2, out = oracle.commit_path(n_nodes, token, alen, path, nxt, kt, vt, kc, vc, seq,
                                             out_stride=5)
    assert seq2.tolist() == [10, 5]                                 # sequence 0 hit the end
    assert (kc2[0, 0, 8:10] == kt[0, 0, 0:2]).all() and (vc2[0, 0, 8:10] == vt[0, 0, 0:2]).all()
    assert (kc2[0, 0, :8] == 5.5).all()
    assert (kc2[1, 0, 2:5] == kt[1, 0, 0:3]).all() and (kc2[1, 0, 5:] == 5.5).all()
    assert (kc2[1, 0, :2] == 5.5).all() and (vc2[1, 0, 5:] == 6.5).all()
    assert out.tolist() == [[101, 102, 103, 41, -1], [107, 108, 42, -1, -1]]
    assert (kc == 5.5).all()                                         # inputs are not modified
