"""GPU parity: every C-ABI entry point against the CPU oracle, element by element.

Integer results (masks, ranks' pass/fail, compaction indices, compacted trees,
accepted paths) must match bit for bit.  Attention must match within
  fp32:  |gpu - ref| <= 1e-5 * max(|ref|, max|ref_row|)
  bf16:  |gpu - ref| <= 2e-2 absolute   (bf16 inputs, fp32 accumulation)
against the oracle's unrounded double-precision result.
"""
import numpy as np
import pytest
import torch

from paper_2402_13485_amd import synth
from gpu_util import host_f64, sentinel_like, to_dev, to_host, u64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pb():
    from paper_2402_13485_amd import binding
    binding.load_library()  # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available()
    return binding


def dev_tree(pb, n_nodes, parent, token=None):
    nn, par = to_dev(n_nodes.astype(np.int32)), to_dev(parent.astype(np.int32))
    depth, anc = pb.propd_tree_mask(nn, par)
    return pb.Tree(n_nodes=nn, parent=par, token=None if token is None else to_dev(token),
                   depth=depth, anc=anc)


# ------------------------------------------------------------------ mask


def test_tree_mask_matches_oracle(pb, oracle):
    rng = np.random.default_rng(101)
    shapes = [synth.random_tree(rng, int(T)) for T in rng.integers(1, 129, size=37)]
    shapes += [synth.chain_tree(128), synth.star_tree(128), synth.rank_product_tree(128, 5),
               synth.chain_tree(1)]
    for T_max in (128,):
        n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
        depth_ref, anc_ref = oracle.tree_mask(n_nodes, parent)
        depth, anc = pb.propd_tree_mask(to_dev(n_nodes), to_dev(parent))
        torch.cuda.synchronize()
        assert (to_host(depth) == depth_ref).all()
        assert (u64(anc) == anc_ref).all()
    small = [synth.random_tree(rng, int(T)) for T in rng.integers(1, 18, size=9)]
    n_nodes, parent, _ = synth.pad_trees(small, 17)
    depth_ref, anc_ref = oracle.tree_mask(n_nodes, parent)
    depth, anc = pb.propd_tree_mask(to_dev(n_nodes), to_dev(parent))
    assert (to_host(depth) == depth_ref).all() and (u64(anc) == anc_ref).all()


# ------------------------------------------------------------------ attention


def run_attention(pb, x):
    tree = dev_tree(pb, x["n_nodes"], x["parent"])
    sent = sentinel_like(x["q"])
    out = to_dev(sent)
    pb.propd_tree_attention(tree, to_dev(x["q"]), to_dev(x["k_cache"]), to_dev(x["v_cache"]),
                            to_dev(x["k_tree"]), to_dev(x["v_tree"]), to_dev(x["seq_lens"]),
                            x["scale"], out=out)
    torch.cuda.synchronize()
    return out, sent


def check_attention(oracle, x, out, sent):
    ref = oracle.tree_attention(x["n_nodes"], x["parent"], x["seq_lens"], x["q"], x["k_cache"],
                                x["v_cache"], x["k_tree"], x["v_tree"], x["scale"])
    got = host_f64(out)
    raw = to_host(out)
    worst = 0.0
    for b in range(x["B"]):
        T = int(x["n_nodes"][b])
        g, r = got[b, :, :T], ref[b, :, :T]
        assert np.isfinite(g).all()
        if x["dtype"] == "f32":
            bound = 1e-5 * np.maximum(np.abs(r), np.abs(r).max(axis=-1, keepdims=True))
            assert (np.abs(g - r) <= bound).all(), float(np.abs(g - r).max())
        else:
            err = float(np.abs(g - r).max())
            worst = max(worst, err)
            assert err <= 2e-2, err
        assert (raw[b, :, T:] == sent[b, :, T:]).all()  # rows beyond the tree stay untouched
    return worst


def small_bf16_case(seed, B, H, T_max, shapes, seq_lens, L_max=None):
    w = synth.Workload(90 + seed, "case", "bf16", B, H, 128, T_max, 0, 0, 0, 1e-3)
    return synth.make_attention_inputs(w, seq_lens=np.asarray(seq_lens, np.int32), L_max=L_max,
                                       trees=shapes)


def test_attention_c1_fp32(pb, oracle):
    w = synth.WORKLOADS[1]
    x = synth.make_attention_inputs(w)
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)


def test_attention_fp32_ragged_d128(pb, oracle):
    rng = np.random.default_rng(5)
    shapes = [synth.rank_product_tree(32, 4), synth.random_tree(rng, 7), synth.chain_tree(20)]
    w = synth.Workload(81, "case", "f32", 3, 2, 128, 32, 0, 0, 0, 1e-5)
    x = synth.make_attention_inputs(w, seq_lens=np.array([70, 0, 129], np.int32), trees=shapes)
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)


@pytest.mark.parametrize("T_max", [16, 128])
def test_attention_bf16_head_size_64(pb, oracle, T_max):
    """bf16 tensors with the smaller head size (the plain kernel, no workspace): ragged
    lengths, an empty cache, a one-node tree, trees smaller than the slot."""
    rng = np.random.default_rng(64 + T_max)
    shapes = [synth.rank_product_tree(T_max, 3 if T_max == 16 else 5),
              synth.random_tree(rng, max(1, T_max // 3)), synth.chain_tree(1)]
    w = synth.Workload(82, "case", "bf16", 3, 2, 64, T_max, 0, 0, 0, 1e-3)
    x = synth.make_attention_inputs(w, seq_lens=np.array([131, 0, 64], np.int32), trees=shapes)
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)


@pytest.mark.parametrize("T_max,kind", [(16, "rank"), (32, "random"), (64, "rank"), (128, "rank"),
                                        (128, "chain"), (96, "random")])
def test_attention_bf16_tree_sizes(pb, oracle, T_max, kind):
    """All three query-group layouts (T_max <= 32, <= 64, <= 128), ragged lengths that
    leave partial tiles, an empty cache, and trees smaller than the slot."""
    rng = np.random.default_rng(T_max)
    depth = {16: 3, 32: 4, 64: 4, 96: 5, 128: 5}[T_max]
    full = {"rank": lambda: synth.rank_product_tree(T_max, depth),
            "random": lambda: synth.random_tree(rng, T_max),
            "chain": lambda: synth.chain_tree(T_max)}[kind]()
    shapes = [full, synth.random_tree(rng, max(1, T_max // 3)), synth.chain_tree(1), full]
    x = small_bf16_case(T_max + len(kind), 4, 2, T_max, shapes, [300, 77, 0, 129])
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)


def test_attention_bf16_many_splits(pb, oracle):
    """Few (sequence, head) units and a long cache: the KV range is split across
    workgroups and merged by the second kernel; lengths leave some splits empty."""
    rng = np.random.default_rng(9)
    shapes = [synth.rank_product_tree(64, 4), synth.random_tree(rng, 40)]
    x = small_bf16_case(9, 2, 1, 64, shapes, [1500, 130], L_max=1536)
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)


@pytest.mark.parametrize("direction", ["rising", "falling", "late_spike"])
def test_attention_bf16_moving_maximum(pb, oracle, direction):
    """Scores whose running maximum keeps moving by many powers of two (keys scaled along the
    cache), so the kernel's reference-maximum updates, with an earlier stage's weights still
    to be added, are exercised in every position; and scores that only ever shrink, where the
    first reference must last."""
    rng = np.random.default_rng(31)
    shapes = [synth.rank_product_tree(128, 5), synth.random_tree(rng, 50)]
    x = small_bf16_case(31, 2, 2, 128, shapes, [700, 333], L_max=704)
    k = synth.as_float(x["k_cache"]).astype(np.float32)
    q = synth.as_float(x["q"]).astype(np.float32)
    L = k.shape[2]
    pos = np.arange(L, dtype=np.float32)
    if direction == "rising":
        gain = 0.2 + 6.0 * pos / L
    elif direction == "falling":
        gain = 6.0 - 5.8 * pos / L
    else:
        gain = np.where((pos > 500) & (pos < 520), 8.0, 0.3).astype(np.float32)
    # keys aligned with query 0 of each head so that the gain really moves the scores
    k = 0.3 * k + gain[None, None, :, None] * q[:, :, :1, :] / 4.0
    x["k_cache"] = synth.f32_to_bf16_bits(k.astype(np.float32))
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)


def test_attention_sizes_rewritten_in_place(pb, oracle):
    """A decoding loop rewrites seq_lens / n_nodes in place between calls and reuses the
    workspace: every call must see the current sizes (they are read on the scalar path).
    The second round is so short that some workgroups of the grid get no stage at all."""
    rng = np.random.default_rng(77)
    shapes = [synth.rank_product_tree(64, 4), synth.random_tree(rng, 40), synth.chain_tree(9)]
    x = small_bf16_case(77, 3, 2, 64, shapes, [400, 250, 90], L_max=448)
    tree = dev_tree(pb, x["n_nodes"], x["parent"])
    q, kc, vc = to_dev(x["q"]), to_dev(x["k_cache"]), to_dev(x["v_cache"])
    kt, vt, seq = to_dev(x["k_tree"]), to_dev(x["v_tree"]), to_dev(x["seq_lens"])
    ws = torch.empty(pb.workspace_bytes(pb.WS_TREE_ATTENTION, 3, 64, 2, 128, 448),
                     dtype=torch.uint8, device="cuda")
    for lens, nodes in ([400, 250, 90], [64, 40, 9]), ([33, 250, 0], [17, 40, 1]), ([399, 97, 64], [64, 33, 9]):
        y = dict(x, seq_lens=np.asarray(lens, np.int32), n_nodes=np.asarray(nodes, np.int32))
        seq.copy_(to_dev(y["seq_lens"]))          # same device buffers, new contents
        tree.n_nodes.copy_(to_dev(y["n_nodes"]))
        sent = sentinel_like(x["q"])
        out = to_dev(sent)
        pb.propd_tree_attention(tree, q, kc, vc, kt, vt, seq, x["scale"], out=out, workspace=ws)
        torch.cuda.synchronize()
        check_attention(oracle, y, out, sent)


def test_attention_survivors_unchanged_by_compaction(pb, oracle):
    """Section 4.1: pruning does not change what a surviving node computes."""
    rng = np.random.default_rng(12)
    shapes = [synth.rank_product_tree(128, 5)] * 2
    x = small_bf16_case(12, 2, 2, 128, shapes, [200, 333])
    out_full, _ = run_attention(pb, x)
    rank = rng.integers(0, 8, size=x["parent"].shape).astype(np.int32)
    rank[:, 0] = 0
    token = rng.integers(0, 100, size=x["parent"].shape).astype(np.int32)
    pr = oracle.prune_compact(x["n_nodes"], x["parent"], token, rank, 5)
    y = dict(x, n_nodes=pr["n_kept"], parent=pr["parent"])
    for name in ("q", "k_tree", "v_tree"):
        y[name] = oracle.gather_rows(x[name], pr["orig_index"], pr["n_kept"], fill_from=x[name])
    out_small, sent = run_attention(pb, y)
    check_attention(oracle, y, out_small, sent)
    a, b_ = host_f64(out_full), host_f64(out_small)
    for b in range(2):
        n = int(pr["n_kept"][b])
        assert 1 < n < 128
        np.testing.assert_allclose(b_[b, :, :n], a[b][:, pr["orig_index"][b, :n]], atol=2e-2)


# ------------------------------------------------------------------ early prune


def run_prune(pb, x, payload_arrays=(), want_rank=True):
    tree = dev_tree(pb, x["n_nodes"], x["parent"], x["token"])
    payloads = [to_dev(a) for a in payload_arrays]
    sentinels = [sentinel_like(a) for a in payload_arrays]
    outs = [to_dev(s) for s in sentinels]
    res = pb.propd_early_prune(tree, to_dev(x["hidden_states"]), to_dev(x["head_weight"]),
                               x["top_k"], payloads=payloads, payload_out=outs,
                               want_rank=want_rank)
    torch.cuda.synchronize()
    return res, sentinels


def check_prune(oracle, x, res, payload_arrays=(), sentinels=()):
    rank_ref, margin = oracle.early_head_rank(x["n_nodes"], x["parent"], x["token"],
                                              x["hidden_states"], x["head_weight"], x["top_k"])
    # the generator promises a margin around the k boundary; bit-exact masks are only
    # meaningful on such inputs, so assert it on the oracle's own scores first
    w = synth.WORKLOADS.get(x.get("config", 0))
    tau = x.get("tau", 1e-3)
    finite = margin[np.isfinite(margin)]                 # none when no node has a child
    assert finite.size == 0 or finite.min() >= 0.999 * tau
    ref = oracle.prune_compact(x["n_nodes"], x["parent"], x["token"], rank_ref, x["top_k"])
    rank = to_host(res.rank)
    k = x["top_k"]
    valid = rank_ref >= 0
    assert ((rank >= k) == (rank_ref >= k))[valid].all()
    assert (rank[~valid] == -1).all()
    assert (u64(res.keep_bits) == ref["keep_bits"]).all()
    for name in ("new_index", "orig_index", "n_kept", "cu_nodes"):
        assert (to_host(getattr(res, name)) == ref[name]).all(), name
    assert (to_host(res.tree.n_nodes) == ref["n_kept"]).all()
    for name in ("parent", "token", "depth"):
        assert (to_host(getattr(res.tree, name)) == ref[name]).all(), name
    assert (u64(res.tree.anc) == ref["anc"]).all()
    for arr, sent, got in zip(payload_arrays, sentinels, res.payloads):
        want = oracle.gather_rows(arr, ref["orig_index"], ref["n_kept"], fill_from=sent)
        assert (to_host(got) == want).all()
    return ref, rank_ref


def test_prune_c1_fp32(pb, oracle):
    w = synth.WORKLOADS[1]
    x = synth.make_prune_inputs(w)
    x["tau"] = w.tau
    res, sents = run_prune(pb, x, [x["hidden_states"]])
    ref, _ = check_prune(oracle, x, res, [x["hidden_states"]], sents)
    assert 1 <= ref["n_kept"][0] < 16


@pytest.mark.parametrize("B,T_max,Hd,V,k", [(3, 64, 256, 1003, 10), (2, 128, 512, 4096, 8),
                                            (5, 16, 64, 130, 3)])
def test_prune_bf16_small(pb, oracle, B, T_max, Hd, V, k):
    """MFMA early head with ragged vocabulary tiles, several sequences, payload gathers
    of hidden rows [B,T,Hd] and tree K rows [B,H,T,128]."""
    depth = {16: 3, 64: 4, 128: 5}[T_max]
    rng = np.random.default_rng(B * 1000 + V)
    shapes = [synth.rank_product_tree(T_max, depth)] * (B - 1) + \
        [synth.random_tree(rng, max(2, T_max // 2), max_depth=6)]
    w = synth.Workload(70 + B, "case", "bf16", B, 2, 128, T_max, Hd, V, k, 1e-3)
    x = synth.make_prune_inputs(w, trees=shapes)
    kt = synth.normal_bf16(rng, (B, 2, T_max, 128))
    res, sents = run_prune(pb, x, [x["hidden_states"], kt])
    ref, _ = check_prune(oracle, x, res, [x["hidden_states"], kt], sents)
    assert ref["n_kept"].min() >= 1 and ref["n_kept"].sum() < B * T_max


def test_prune_top_k_at_least_vocab_keeps_everything(pb, oracle):
    w = synth.Workload(75, "case", "bf16", 2, 1, 128, 32, 128, 200, 7, 1e-3)
    x = synth.make_prune_inputs(w, trees=[synth.rank_product_tree(32, 4)] * 2)
    for k in (200, 5000):
        x["top_k"] = k
        res, _ = run_prune(pb, x)
        assert to_host(res.n_kept).tolist() == [32, 32]
        assert (to_host(res.new_index) == np.arange(32)).all()
        ref = oracle.prune_compact(x["n_nodes"], x["parent"], x["token"],
                                   np.zeros_like(x["parent"]), k)
        assert (u64(res.tree.anc) == ref["anc"]).all()


def test_prune_out_of_range_token_fails(pb):
    w = synth.Workload(76, "case", "bf16", 1, 1, 128, 16, 64, 100, 50, 1e-3)
    x = synth.make_prune_inputs(w, trees=[synth.star_tree(16)])
    x["token"][0, 3] = 100   # == vocab
    x["token"][0, 5] = -4
    res, _ = run_prune(pb, x)
    keep = int(u64(res.keep_bits)[0, 0])
    assert not (keep >> 3) & 1 and not (keep >> 5) & 1 and keep & 1


def test_prune_tokens_that_nobody_placed(pb, oracle):
    """Token ids drawn at random, not placed at a distance from the k boundary: the decisions must
    agree with the oracle's wherever the oracle's own margin is at least tau, the counted ranks
    may differ only where scores are nearly equal, and everything after the decision must be the
    oracle's compaction of the GPU's own pass/fail flags."""
    rng = np.random.default_rng(4242)
    B, T_max, Hd, V, k, tau = 4, 64, 512, 4096, 2000, 1e-3
    shapes = [synth.rank_product_tree(64, 4), synth.random_tree(rng, 64, max_depth=7),
              synth.random_tree(rng, 33), synth.star_tree(40)]
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = synth.draw_tokens(rng, n_nodes, parent, V)
    hidden = synth.normal_bf16(rng, (B, T_max, Hd))
    weight = synth.normal_bf16(rng, (V, Hd), sigma=0.02)
    x = dict(n_nodes=n_nodes, parent=parent, token=token, hidden_states=hidden, head_weight=weight, top_k=k)
    res, sents = run_prune(pb, x, [hidden])
    rank_ref, margin = oracle.early_head_rank(n_nodes, parent, token, hidden, weight, k)
    rank = to_host(res.rank)
    valid = rank_ref >= 0
    sure = valid & (np.isfinite(margin)) & (margin >= tau)
    assert sure.sum() > 0.8 * (valid.sum() - B)            # most decisions are far from the boundary
    assert ((rank >= k) == (rank_ref >= k))[sure].all()
    assert (rank[~valid] == -1).all() and (rank[:, 0] == 0).all()
    diff = np.abs(rank - rank_ref)[valid]
    assert diff.max() <= 3 and (diff > 0).mean() < 0.05     # fp32 against fp64 order of near-equal scores
    assert 0.1 < (rank[valid] < k).mean() < 0.9
    ref = oracle.prune_compact(n_nodes, parent, token, rank, k)   # the GPU's own flags
    assert (u64(res.keep_bits) == ref["keep_bits"]).all()
    for name in ("new_index", "orig_index", "n_kept", "cu_nodes"):
        assert (to_host(getattr(res, name)) == ref[name]).all(), name
    for name in ("parent", "token", "depth"):
        assert (to_host(getattr(res.tree, name)) == ref[name]).all(), name
    assert (u64(res.tree.anc) == ref["anc"]).all()
    want = oracle.gather_rows(hidden, ref["orig_index"], ref["n_kept"], fill_from=sents[0])
    assert (to_host(res.payloads[0]) == want).all()


def test_prune_without_rank_output_gives_the_same_decisions(pb, oracle):
    """The call as a decoding loop makes it (no rank output asked for) on a batch whose score rows
    fill more than one row tile of either tile shape."""
    w = synth.Workload(77, "case", "bf16", 7, 1, 128, 128, 256, 2048, 6, 1e-3)
    x = synth.make_prune_inputs(w, trees=[synth.rank_product_tree(128, 5)] * 4 +
                                [synth.chain_tree(128), synth.star_tree(100), synth.chain_tree(128)])
    res, _ = run_prune(pb, x, want_rank=False)
    rank_ref, margin = oracle.early_head_rank(x["n_nodes"], x["parent"], x["token"], x["hidden_states"],
                                              x["head_weight"], x["top_k"])
    assert margin[np.isfinite(margin)].min() >= 0.999e-3
    ref = oracle.prune_compact(x["n_nodes"], x["parent"], x["token"], rank_ref, x["top_k"])
    assert res.rank is None and (u64(res.keep_bits) == ref["keep_bits"]).all()
    assert (to_host(res.orig_index) == ref["orig_index"]).all()
    assert (u64(res.tree.anc) == ref["anc"]).all()


@pytest.mark.parametrize("Hd", [32, 96])
def test_prune_many_rows_wide_vocabulary_short_rows(pb, oracle, Hd):
    """616 score rows against a 32000-entry vocabulary: on a 256-unit chip this is the case the
    352-row tile shape is picked for.  One and three K steps (hidden 32 and 96): the ring's
    prologue, its drain, and the accumulators read right after a single matrix instruction."""
    B = 14
    w = synth.Workload(78, "case", "bf16", B, 1, 128, 128, Hd, 32000, 8, 1e-3)
    x = synth.make_prune_inputs(w, trees=[synth.rank_product_tree(128, 5)] * B)
    res, sents = run_prune(pb, x, [x["hidden_states"]])
    ref, _ = check_prune(oracle, x, res, [x["hidden_states"]], sents)
    assert 0.1 < ref["n_kept"].sum() / (B * 128) < 0.5


@pytest.mark.parametrize("dtype,B,T_max,Hd,V", [("bf16", 3, 64, 256, 4096), ("bf16", 14, 128, 96, 32000),
                                                ("f32", 2, 32, 64, 700)])
def test_prune_equal_scores_rank_by_token_id(pb, oracle, dtype, B, T_max, Hd, V):
    """Vocabulary entries with identical weight rows score identically under every parent, in
    any arithmetic.  Two siblings that carry such a pair must be ranked next to each other, the
    lower id first: the score a child is compared against and the score the kernel computes
    for the same entry in another place have to be the same bits for that.  Both tile shapes of
    the bf16 kernel (few rows; 616 rows against a wide vocabulary) and the fp32 kernel; the
    twin entry lies in the same column tile or in a distant one."""
    rng = np.random.default_rng(B * 1000 + Hd)
    depth = {32: 4, 64: 4, 128: 5}[T_max]
    shapes = [synth.rank_product_tree(T_max, depth)] * B
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = synth.draw_tokens(rng, n_nodes, parent, V)
    if dtype == "bf16":
        hidden = synth.normal_bf16(rng, (B, T_max, Hd))
        weight = synth.normal_bf16(rng, (V, Hd), sigma=0.05)
    else:
        hidden = synth.normal_f32(rng, (B, T_max, Hd))
        weight = synth.normal_f32(rng, (V, Hd), 0.05)
    used = set(int(t) for t in token[token >= 0])
    pairs = []
    for b in range(B):
        kids = synth.children_lists(parent[b], int(n_nodes[b]))
        for p_, ks in enumerate(kids):
            if len(ks) < 2:
                continue
            c1, c2 = ks[0], ks[1]
            t1 = int(token[b, c1])
            t2 = (t1 + (1 if len(pairs) % 2 else 300)) % V
            if t2 in used or t2 == t1:
                continue
            used.add(t2)
            weight[t2] = weight[t1]
            token[b, c2] = t2
            pairs.append((b, c1, c2, t1, t2))
    assert len(pairs) >= 4 * B
    k = 8
    x = dict(n_nodes=n_nodes, parent=parent, token=token, hidden_states=hidden, head_weight=weight, top_k=k)
    res, _ = run_prune(pb, x)
    rank = to_host(res.rank)
    rank_ref, _ = oracle.early_head_rank(n_nodes, parent, token, hidden, weight, k)
    for b, c1, c2, t1, t2 in pairs:
        lo, hi = (c1, c2) if t1 < t2 else (c2, c1)
        assert rank_ref[b, hi] == rank_ref[b, lo] + 1
        assert rank[b, hi] == rank[b, lo] + 1, (b, c1, c2, t1, t2, rank[b, c1], rank[b, c2])
    valid = rank_ref >= 0
    assert np.abs(rank - rank_ref)[valid].max() <= 3


def test_prune_many_sequences_of_mixed_shapes(pb, oracle):
    """70 sequences: a sequence's score rows follow those of all sequences before it, counted
    by the table workgroups four sequences at a time, more than one round of counting for the
    last ones; chains, one-node trees and bushy trees in turn, so the counts differ."""
    B, T_max = 70, 16
    rng = np.random.default_rng(70)
    kinds = [lambda: synth.rank_product_tree(16, 3), lambda: synth.chain_tree(1),
             lambda: synth.random_tree(rng, int(rng.integers(2, 17))), lambda: synth.chain_tree(9)]
    shapes = [kinds[i % 4]() for i in range(B)]
    w = synth.Workload(77, "case", "bf16", B, 1, 128, T_max, 64, 700, 5, 1e-3)
    x = synth.make_prune_inputs(w, trees=shapes)
    res, sents = run_prune(pb, x, [x["hidden_states"]])
    check_prune(oracle, x, res, [x["hidden_states"]], sents)


# ------------------------------------------------------------------ accept


def run_accept(pb, n_nodes, parent, token, logits, path_stride=None):
    tree = dev_tree(pb, n_nodes, parent, token)
    alen, path, nxt = pb.propd_accept_path(tree, to_dev(logits), path_stride=path_stride)
    torch.cuda.synchronize()
    return to_host(alen), to_host(path), to_host(nxt)


@pytest.mark.parametrize("dtype,V", [("f32", 256), ("bf16", 32000), ("bf16", 1001), ("f32", 7)])
def test_accept_matches_oracle(pb, oracle, dtype, V):
    rng = np.random.default_rng(V)
    shapes = [synth.rank_product_tree(64, 4)] * 3 + [synth.random_tree(rng, 19, max_depth=6),
                                                      synth.chain_tree(1), synth.chain_tree(64)]
    n_nodes, parent, _ = synth.pad_trees(shapes, 64)
    token = synth.draw_tokens(rng, n_nodes, parent, V) if V >= 64 else \
        rng.integers(0, V, size=parent.shape).astype(np.int32)
    w = synth.Workload(60, "case", dtype, len(shapes), 1, 128, 64, 0, V, 0, 0.0)
    acc = synth.make_accept_inputs(w, n_nodes, parent, token)
    ref = oracle.accept_path(n_nodes, parent, token, acc["logits"], path_stride=9)
    got = run_accept(pb, n_nodes, parent, token, acc["logits"], path_stride=9)
    for g, r in zip(got, ref):
        assert (g == r).all()
    if V >= 64:
        assert got[0].tolist()[:5] == [len(c) for c in acc["chains"]][:5]


def test_accept_ties_pick_lowest_index(pb, oracle):
    rng = np.random.default_rng(33)
    V = 40
    shapes = [synth.random_tree(rng, 30, max_depth=5) for _ in range(16)]
    n_nodes, parent, _ = synth.pad_trees(shapes, 32)
    token = rng.integers(0, 4, size=parent.shape).astype(np.int32)
    vals = rng.integers(0, 3, size=(16, 32, V)).astype(np.float32)  # many equal maxima
    for logits in (vals, synth.f32_to_bf16_bits(vals)):
        ref = oracle.accept_path(n_nodes, parent, token, logits)
        got = run_accept(pb, n_nodes, parent, token, logits)
        for g, r in zip(got, ref):
            assert (g == r).all()


def test_accept_short_path_buffer_keeps_a_prefix(pb, oracle):
    """A path buffer shorter than the accepted path: the first path_stride nodes of the oracle's
    path, and the token that follows them on that path as the next token (the same greedy
    output, fewer tokens per step)."""
    rng = np.random.default_rng(35)
    V, T_max = 2000, 40
    shapes = [synth.chain_tree(int(T)) for T in (40, 7, 1, 23)] + [synth.random_tree(rng, 40, max_depth=12)]
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = synth.draw_tokens(rng, n_nodes, parent, V)
    logits = rng.standard_normal((len(shapes), T_max, V)).astype(np.float32)
    for b in range(len(shapes)):                      # every child carries its parent's greedy choice
        for i in range(1, int(n_nodes[b])):
            logits[b, parent[b, i], token[b, i]] = 9.0 + 0.01 * (i == 1 or parent[b, i] != parent[b, i - 1])
    full = oracle.accept_path(n_nodes, parent, token, logits, path_stride=T_max)
    assert full[0].max() >= 12
    for stride in (1, 4, 11):
        alen, path, nxt = run_accept(pb, n_nodes, parent, token, logits, path_stride=stride)
        for b in range(len(shapes)):
            a = int(full[0][b])
            if a <= stride:
                assert alen[b] == a and nxt[b] == full[2][b]
                assert (path[b] == full[1][b, :stride]).all()
            else:
                assert alen[b] == stride and (path[b] == full[1][b, :stride]).all()
                assert nxt[b] == token[b, full[1][b, stride]]


# ------------------------------------------------------------------ whole step, reduced size


def test_whole_step_reduced_c3(pb, oracle):
    """prune -> compact -> attention on survivors -> accept, all through the C ABI, on a
    reduced 7B-shaped case (B=3, H=4, ragged L, T=64, hidden 512, vocabulary 4096)."""
    w = synth.Workload(3, "c3_reduced", "bf16", 3, 4, 128, 64, 512, 4096, 10, 1e-3)
    trees = [synth.rank_product_tree(64, 4)] * 3
    seq = np.array([700, 512, 1031], np.int32)
    xa = synth.make_attention_inputs(w, seq_lens=seq, trees=trees)
    xp = synth.make_prune_inputs(w, trees=trees)
    acc = synth.make_accept_inputs(w, xp["n_nodes"], xp["parent"], xp["token"])
    payloads = [xa["q"], xa["k_tree"], xa["v_tree"], acc["logits"]]
    res, sents = run_prune(pb, xp, payloads)
    ref, _ = check_prune(oracle, xp, res, payloads, sents)
    # attention on the compacted tree, using the device outputs of the prune call directly
    q2, kt2, vt2, lg2 = res.payloads
    out = to_dev(sentinel_like(xa["q"]))
    pb.propd_tree_attention(res.tree, q2, to_dev(xa["k_cache"]), to_dev(xa["v_cache"]), kt2, vt2,
                            to_dev(seq), xa["scale"], out=out)
    alen, path, nxt = pb.propd_accept_path(res.tree, lg2)
    torch.cuda.synchronize()
    g = lambda a: oracle.gather_rows(a, ref["orig_index"], ref["n_kept"], fill_from=a)
    y = dict(xa, n_nodes=ref["n_kept"], parent=ref["parent"], q=g(xa["q"]),
             k_tree=g(xa["k_tree"]), v_tree=g(xa["v_tree"]))
    check_attention(oracle, y, out, sentinel_like(xa["q"]))
    r_len, r_path, r_next = oracle.accept_path(ref["n_kept"], ref["parent"], ref["token"],
                                               g(acc["logits"]))
    assert (to_host(alen) == r_len).all() and (to_host(path) == r_path).all()
    assert (to_host(nxt) == r_next).all()


def test_whole_step_replayed_from_a_captured_graph(pb):
    """The four calls of a step enqueue kernels only (no allocation of their own when the
    caller passes workspaces, no memset, no host round trip), so a step can be captured into a
    HIP graph.  Replayed three times, with eager steps and synchronisations in between, every
    replay must give the eager step's results bit for bit."""
    w = synth.Workload(3, "c3_reduced", "bf16", 3, 4, 128, 64, 512, 4096, 10, 1e-3)
    trees = [synth.rank_product_tree(64, 4)] * 3
    seq = np.array([700, 512, 1031], np.int32)
    xa = synth.make_attention_inputs(w, seq_lens=seq, trees=trees)
    xp = synth.make_prune_inputs(w, trees=trees)
    acc = synth.make_accept_inputs(w, xp["n_nodes"], xp["parent"], xp["token"])
    tree = dev_tree(pb, xp["n_nodes"], xp["parent"], xp["token"])
    d = {k: to_dev(xa[k]) for k in ("q", "k_cache", "v_cache", "k_tree", "v_tree")}
    seq_d, hid, hw, logits = to_dev(seq), to_dev(xp["hidden_states"]), to_dev(xp["head_weight"]), to_dev(acc["logits"])
    B, H, T, dd = xa["q"].shape
    ws_att = torch.empty(pb.workspace_bytes(pb.WS_TREE_ATTENTION, B, T, H, dd, xa["L_max"]), dtype=torch.uint8, device="cuda")
    ws_pr = torch.empty(pb.workspace_bytes(pb.WS_EARLY_PRUNE, B, T, hidden=512, vocab=4096), dtype=torch.uint8, device="cuda")
    ws_acc = torch.empty(pb.workspace_bytes(pb.WS_ACCEPT_PATH, B, T, vocab=4096), dtype=torch.uint8, device="cuda")
    payloads = [d["q"], d["k_tree"], d["v_tree"], logits]

    def step():
        out_full = pb.propd_tree_attention(tree, d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"],
                                           seq_d, xa["scale"], workspace=ws_att)
        res = pb.propd_early_prune(tree, hid, hw, 10, payloads=payloads, workspace=ws_pr)
        q2, kt2, vt2, lg2 = res.payloads
        out_small = torch.zeros_like(d["q"])
        pb.propd_tree_attention(res.tree, q2, d["k_cache"], d["v_cache"], kt2, vt2, seq_d, xa["scale"],
                                out=out_small, workspace=ws_att)
        alen, path, nxt = pb.propd_accept_path(res.tree, lg2, workspace=ws_acc)
        return [out_full, res.keep_bits, res.new_index, res.orig_index, res.n_kept, res.cu_nodes, res.tree.parent,
                res.tree.anc, out_small, alen, path, nxt]

    eager = [t.clone() for t in step()]
    torch.cuda.synchronize()
    kept = to_host(eager[4])
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        outs = step()
    for _ in range(3):
        again = step()                      # eager work between the replays
        torch.cuda.synchronize()
        for t in outs:
            t.fill_(0) if t.dtype != torch.bfloat16 else t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name_i, (got, want, eag) in enumerate(zip(outs, eager, again)):
            g, e = to_host(got), to_host(want)
            if name_i == 0:               # full-tree attention: rows of the tree only
                for b in range(B):
                    Tb = int(xp["n_nodes"][b])
                    assert (g[b, :, :Tb] == e[b, :, :Tb]).all()
            elif name_i == 8:             # compacted-tree attention: survivors' rows only
                for b in range(B):
                    assert (g[b, :, :kept[b]] == e[b, :, :kept[b]]).all()
            else:
                assert (g == e).all(), name_i
            assert (to_host(eag) == e).all() or name_i in (0, 8)


def test_layers_before_and_after_the_pruning_point(pb, oracle):
    """Figure 5 at reduced size: two layers of tree attention on the full tree, the pruning pass,
    two layers on the compacted tree, acceptance; every layer has its own K/V cache and its own
    tree q/k/v, the later layers' tensors reach the compacted tree as payloads of the pruning call.
    Every layer's output against the oracle, and (Section 4.1: pruning does not change what a
    surviving node computes) the later layers' survivors against the same layers run unpruned."""
    w = synth.Workload(31, "layers", "bf16", 3, 3, 128, 64, 256, 2048, 8, 1e-3)
    trees = [synth.rank_product_tree(64, 4), synth.rank_product_tree(64, 4), synth.chain_tree(20)]
    seq = np.array([333, 64, 700], np.int32)
    n_layers, n_full = 4, 2
    layers = []
    for l in range(n_layers):
        wl = synth.Workload(310 + l, "layers", "bf16", 3, 3, 128, 64, 256, 2048, 8, 1e-3)
        layers.append(synth.make_attention_inputs(wl, seq_lens=seq, trees=trees))
    xp = synth.make_prune_inputs(w, trees=trees)
    acc = synth.make_accept_inputs(w, xp["n_nodes"], xp["parent"], xp["token"])
    tree = dev_tree(pb, xp["n_nodes"], xp["parent"], xp["token"])
    seq_d = to_dev(seq)
    dev = [{k: to_dev(x[k]) for k in ("q", "k_cache", "v_cache", "k_tree", "v_tree")} for x in layers]
    outs_full = []
    for l in range(n_layers):            # every layer on the full tree (the later ones for reference)
        sent = sentinel_like(layers[l]["q"])
        out = to_dev(sent)
        d = dev[l]
        pb.propd_tree_attention(tree, d["q"], d["k_cache"], d["v_cache"], d["k_tree"], d["v_tree"], seq_d,
                                layers[l]["scale"], out=out)
        torch.cuda.synchronize()
        if l < n_full:
            check_attention(oracle, layers[l], out, sent)
        outs_full.append(host_f64(out))
    payload_names = [(l, name) for l in range(n_full, n_layers) for name in ("q", "k_tree", "v_tree")]
    payload_host = [layers[l][name] for l, name in payload_names] + [acc["logits"]]
    res, sents = run_prune(pb, xp, payload_host)
    ref, _ = check_prune(oracle, xp, res, payload_host, sents)
    g = lambda a: oracle.gather_rows(a, ref["orig_index"], ref["n_kept"], fill_from=a)
    for n, l in enumerate(range(n_full, n_layers)):
        q2, kt2, vt2 = res.payloads[3 * n: 3 * n + 3]
        sent = sentinel_like(layers[l]["q"])
        out = to_dev(sent)
        pb.propd_tree_attention(res.tree, q2, dev[l]["k_cache"], dev[l]["v_cache"], kt2, vt2, seq_d,
                                layers[l]["scale"], out=out)
        torch.cuda.synchronize()
        y = dict(layers[l], n_nodes=ref["n_kept"], parent=ref["parent"], q=g(layers[l]["q"]),
                 k_tree=g(layers[l]["k_tree"]), v_tree=g(layers[l]["v_tree"]))
        check_attention(oracle, y, out, sent)
        got = host_f64(out)
        for b in range(3):
            n_b = int(ref["n_kept"][b])
            assert np.abs(got[b, :, :n_b] - outs_full[l][b][:, ref["orig_index"][b, :n_b]]).max() <= 2e-2
    alen, path, nxt = pb.propd_accept_path(res.tree, res.payloads[-1])
    torch.cuda.synchronize()
    r_len, r_path, r_next = oracle.accept_path(ref["n_kept"], ref["parent"], ref["token"], g(acc["logits"]))
    assert (to_host(alen) == r_len).all() and (to_host(path) == r_path).all() and (to_host(nxt) == r_next).all()


# ------------------------------------------------------------------ scratch bounds


def test_workspace_bounds_respected(pb, oracle):
    """Every entry point stays inside the scratch size it asks for: the bytes after
    propd_workspace_bytes() of a larger buffer keep their fill pattern."""
    guard = 1 << 16

    def guarded(nbytes):
        return torch.full((nbytes + guard,), 0xA5, dtype=torch.uint8, device="cuda"), nbytes

    def intact(ws, nbytes):
        torch.cuda.synchronize()
        return bool((ws[nbytes:] == 0xA5).all().item())

    rng = np.random.default_rng(5)
    # attention: a full tree on all four query groups, many splits, and a whole-units case
    for B, H, T_max, lens, L_max in ((2, 1, 128, [1500, 130], 1536), (3, 2, 64, [300, 77, 0], 320),
                                     (4, 160, 128, [96, 96, 96, 96], 96)):
        shapes = [synth.rank_product_tree(T_max, 5 if T_max == 128 else 4)] * B
        x = small_bf16_case(200 + B, B, H, T_max, shapes, lens, L_max=L_max)
        tree = dev_tree(pb, x["n_nodes"], x["parent"])
        ws, n = guarded(pb.workspace_bytes(pb.WS_TREE_ATTENTION, B, T_max, H, 128, L_max))
        sent = sentinel_like(x["q"])
        out = to_dev(sent)
        pb.propd_tree_attention(tree, to_dev(x["q"]), to_dev(x["k_cache"]), to_dev(x["v_cache"]),
                                to_dev(x["k_tree"]), to_dev(x["v_tree"]), to_dev(x["seq_lens"]),
                                x["scale"], out=out, workspace=ws)
        assert intact(ws, n), (B, H, T_max)
        check_attention(oracle, x, out, sent)
    # early prune and acceptance
    w = synth.Workload(95, "case", "bf16", 3, 1, 128, 64, 256, 1000, 5, 1e-3)
    trees = [synth.rank_product_tree(64, 4), synth.random_tree(rng, 30), synth.chain_tree(7)]
    xp = synth.make_prune_inputs(w, trees=trees)
    tree = dev_tree(pb, xp["n_nodes"], xp["parent"], xp["token"])
    ws, n = guarded(pb.workspace_bytes(pb.WS_EARLY_PRUNE, 3, 64, hidden=256, vocab=1000))
    pb.propd_early_prune(tree, to_dev(xp["hidden_states"]), to_dev(xp["head_weight"]), 5,
                         workspace=ws)
    assert intact(ws, n)
    ws, n = guarded(pb.workspace_bytes(pb.WS_EARLY_PRUNE, 3, 64, hidden=256, vocab=1000))
    pb.propd_early_prune_prob(tree, to_dev(xp["hidden_states"]), to_dev(xp["head_weight"]),
                              keep_count=9, want_log_marginal=True, workspace=ws)
    assert intact(ws, n)
    acc = synth.make_accept_inputs(w, xp["n_nodes"], xp["parent"], xp["token"])
    ws, n = guarded(pb.workspace_bytes(pb.WS_ACCEPT_PATH, 3, 64, vocab=1000))
    pb.propd_accept_path(tree, to_dev(acc["logits"]), workspace=ws)
    assert intact(ws, n)


# ------------------------------------------------------------------ commit of the accepted path


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 24)])
def test_commit_path_decoding_loop(pb, oracle, dtype, d):
    """Several steps of acceptance + commit on the GPU, every step against the oracle's, bit for
    bit: caches (all rows, so untouched ones too), lengths, the step's tokens.  The last steps
    run into the end of the cache."""
    import decode_loop_util as dl
    rng = np.random.default_rng(401)
    B, H, T_max, L_max, steps = 5, 3, 19, 40, 8
    prefixes = [[int(t) for t in rng.integers(0, dl.VOCAB, size=n)] for n in (0, 5, 17, 30, 2)]
    roots = [dl.model_next(p) for p in prefixes]
    np_dt = np.uint16 if dtype == "bf16" else np.float32
    kc = sentinel_like(np.zeros((B, H, L_max, d), np_dt))
    vc = sentinel_like(np.zeros((B, H, L_max, d), np_dt))
    for b in range(B):
        kc[b, :, : len(prefixes[b])] = dl.expected_cache_rows(prefixes[b], H, d, 0, dtype)
        vc[b, :, : len(prefixes[b])] = dl.expected_cache_rows(prefixes[b], H, d, 1, dtype)
    seq = np.array([len(p) for p in prefixes], np.int32)
    kc_d, vc_d, seq_d = to_dev(kc), to_dev(vc), to_dev(seq)
    clipped = False
    for step in range(steps):
        n_nodes, parent, token, logits, kt, vt = dl.build_step(rng, prefixes, roots, H, d, T_max, dtype)
        alen_r, path_r, nxt_r = oracle.accept_path(n_nodes, parent, token, logits, path_stride=T_max)
        kc, vc, seq_new, out_r = oracle.commit_path(n_nodes, token, alen_r, path_r, nxt_r, kt, vt,
                                                    kc, vc, seq, out_stride=T_max)
        tree = dev_tree(pb, n_nodes, parent, token)
        alen, path, nxt = pb.propd_accept_path(tree, to_dev(logits), path_stride=T_max)
        out = pb.propd_commit_path(tree, alen, path, nxt, to_dev(kt), to_dev(vt), kc_d, vc_d, seq_d,
                                   out_stride=T_max)
        torch.cuda.synchronize()
        assert (to_host(alen) == alen_r).all() and (to_host(nxt) == nxt_r).all()
        assert (to_host(out) == out_r).all(), step
        assert (to_host(seq_d) == seq_new).all(), step
        assert (to_host(kc_d) == kc).all() and (to_host(vc_d) == vc).all(), step
        clipped |= bool((seq_new - seq < alen_r).any())
        for b in range(B):
            a = int(alen_r[b])
            toks = [int(t) for t in out_r[b, :a]]
            prefixes[b] = (prefixes[b] + [roots[b]] + toks[:-1])[: int(seq_new[b])]
            roots[b] = toks[-1]
        seq = seq_new
    assert clipped and (seq == L_max).any()


def test_commit_path_bad_indices_write_nothing(pb):
    """Path entries outside the tree and lengths outside [0, path_stride] come from device memory;
    they must not turn into accesses outside the tensors."""
    B, H, T_max, L_max, d = 3, 2, 8, 12, 64
    shapes = [synth.chain_tree(8), synth.chain_tree(4), synth.chain_tree(8)]
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = np.arange(B * T_max, dtype=np.int32).reshape(B, T_max)
    tree = dev_tree(pb, n_nodes, parent, token)
    kt = np.arange(B * H * T_max * d, dtype=np.float32).reshape(B, H, T_max, d)
    kc = sentinel_like(np.zeros((B, H, L_max, d), np.float32))
    kc_d, vc_d = to_dev(kc), to_dev(kc)
    seq_d = to_dev(np.array([3, 50, -4], np.int32))
    alen = to_dev(np.array([3, 2, 99], np.int32))
    path = to_dev(np.array([[0, 77, 2, -1], [0, 5, -1, -1], [0, -3, 2, 3]], np.int32))
    out = pb.propd_commit_path(tree, alen, path, to_dev(np.array([9, 9, 9], np.int32)), to_dev(kt),
                               to_dev(-kt), kc_d, vc_d, seq_d, out_stride=4)
    torch.cuda.synchronize()
    got = to_host(kc_d)
    assert to_host(seq_d).tolist() == [6, 12, 4]
    assert (got[0, :, 3] == kt[0, :, 0]).all() and (got[0, :, 5] == kt[0, :, 2]).all()
    assert (got[0, :, 4] == kc[0, :, 4]).all() and (got[0, :, 6:] == kc[0, :, 6:]).all()
    assert (got[1] == kc[1]).all()                       # length past the end: nothing fits
    assert (got[2, :, 0] == kt[2, :, 0]).all() and (got[2, :, 1] == kc[2, :, 1]).all()
    assert (got[2, :, 2] == kt[2, :, 2]).all() and (got[2, :, 3] == kt[2, :, 3]).all()
    assert (got[2, :, 4:] == kc[2, :, 4:]).all()
    assert to_host(out).tolist() == [[-1, 2, 9, -1], [-1, 9, -1, -1], [-1, 18, 19, 9]]


# ------------------------------------------------------------------ probability-based pruning


def prob_reference(oracle, x, threshold=None, keep_count=None):
    """Oracle decisions + compaction, and the distance of every decision from its boundary."""
    _, logm = oracle.early_head_logprob(x["n_nodes"], x["parent"], x["token"], x["hidden_states"],
                                        x["head_weight"])
    fail = oracle.prob_fail_flags(x["n_nodes"], logm, threshold=threshold, keep_count=keep_count)
    ref = oracle.prune_compact(x["n_nodes"], x["parent"], x["token"], fail, 1)
    return logm, fail, ref


def threshold_in_a_gap(logm, n_nodes, tau, quantile=0.5):
    """A probability threshold whose logarithm sits in the middle of a gap of at least 2*tau
    between the marginals of the batch, near the given quantile."""
    vals = np.sort(np.concatenate([logm[b, 1:int(n)] for b, n in enumerate(n_nodes)]))
    gaps = np.diff(vals)
    order = np.argsort(np.abs(np.arange(len(gaps)) - quantile * len(gaps)))
    j = next(int(j) for j in order if gaps[j] >= 2 * tau)
    return float(np.exp(0.5 * (vals[j] + vals[j + 1])))


def check_prob(pb, oracle, x, res, ref, logm, payload_arrays=(), sentinels=()):
    lm = to_host(res.log_marginal).astype(np.float64)
    for b, n in enumerate(x["n_nodes"]):
        assert np.abs(lm[b, :int(n)] - logm[b, :int(n)]).max() < 2e-4 * max(1.0, np.abs(logm[b, :int(n)]).max())
        assert (lm[b, int(n):] == 0).all()
    assert (u64(res.keep_bits) == ref["keep_bits"]).all()
    for name in ("new_index", "orig_index", "n_kept", "cu_nodes"):
        assert (to_host(getattr(res, name)) == ref[name]).all(), name
    assert (to_host(res.tree.n_nodes) == ref["n_kept"]).all()
    for name in ("parent", "token", "depth"):
        assert (to_host(getattr(res.tree, name)) == ref[name]).all(), name
    assert (u64(res.tree.anc) == ref["anc"]).all()
    for arr, sent, got in zip(payload_arrays, sentinels, res.payloads):
        want = oracle.gather_rows(arr, ref["orig_index"], ref["n_kept"], fill_from=sent)
        assert (to_host(got) == want).all()


def run_prob(pb, x, payload_arrays=(), **crit):
    tree = dev_tree(pb, x["n_nodes"], x["parent"], x["token"])
    payloads = [to_dev(a) for a in payload_arrays]
    sentinels = [sentinel_like(a) for a in payload_arrays]
    res = pb.propd_early_prune_prob(tree, to_dev(x["hidden_states"]), to_dev(x["head_weight"]),
                                    payloads=payloads, payload_out=[to_dev(s) for s in sentinels],
                                    want_log_marginal=True, **crit)
    torch.cuda.synchronize()
    return res, sentinels


@pytest.mark.parametrize("dtype,B,T_max,Hd,V", [("bf16", 3, 64, 256, 1003), ("bf16", 2, 128, 512, 4096),
                                                ("f32", 2, 16, 64, 256)])
def test_prob_prune_threshold(pb, oracle, dtype, B, T_max, Hd, V):
    tau = 1e-3
    depth = {16: 3, 64: 4, 128: 5}[T_max]
    rng = np.random.default_rng(500 + V)
    shapes = [synth.rank_product_tree(T_max, depth)] * (B - 1) + \
        [synth.random_tree(rng, max(2, T_max // 2), max_depth=6)]
    w = synth.Workload(80 + B, "case", dtype, B, 2, 128, T_max, Hd, V, 8 if V > 300 else 4, tau)
    x = synth.make_prune_inputs(w, trees=shapes)
    kt = synth.normal_bf16(rng, (B, 2, T_max, 128))
    logm, _, _ = prob_reference(oracle, x, threshold=0.5)
    for quantile in (0.3, 0.7):
        thr = threshold_in_a_gap(logm, x["n_nodes"], tau, quantile)
        thr = float(np.float32(thr))                                   # what the call receives
        _, fail, ref = prob_reference(oracle, x, threshold=thr)
        valid = np.arange(T_max)[None, :] < x["n_nodes"][:, None]
        valid[:, 0] = False
        assert np.abs(logm[valid] - np.log(thr)).min() >= 0.999 * tau     # decisions are well separated
        res, sents = run_prob(pb, x, [x["hidden_states"], kt], threshold=thr)
        check_prob(pb, oracle, x, res, ref, logm, [x["hidden_states"], kt], sents)
        assert 1 < ref["n_kept"].sum() < x["n_nodes"].sum()
    # the ends of the range: 0 keeps every sequence, 1 only the roots
    res, _ = run_prob(pb, x, threshold=0.0)
    assert (to_host(res.n_kept) == x["n_nodes"]).all()
    res, _ = run_prob(pb, x, threshold=1.0)
    assert (to_host(res.n_kept) == 1).all()


@pytest.mark.parametrize("B,T_max,Hd,V", [(3, 64, 256, 1003), (2, 128, 512, 4096)])
def test_prob_prune_rank(pb, oracle, B, T_max, Hd, V):
    tau = 1e-3
    depth = {64: 4, 128: 5}[T_max]
    w = synth.Workload(90 + B, "case", "bf16", B, 2, 128, T_max, Hd, V, 8, tau)
    x = synth.make_prune_inputs(w, trees=[synth.rank_product_tree(T_max, depth)] * B)
    logm, _, _ = prob_reference(oracle, x, keep_count=1)
    srt = -np.sort(-logm[:, :T_max], axis=1)                          # per tree, descending
    gap = srt[:, :-1] - srt[:, 1:]                                    # gap[b, R-1]: between the R-th and the next
    candidates = [R for R in range(2, T_max) if gap[:, R - 1].min() >= 2 * tau]
    assert len(candidates) >= 3
    for R in (candidates[0], candidates[len(candidates) // 2], candidates[-1]):
        _, fail, ref = prob_reference(oracle, x, keep_count=R)
        assert (ref["n_kept"] == R).all()
        res, _ = run_prob(pb, x, keep_count=R)
        check_prob(pb, oracle, x, res, ref, logm)
    res, _ = run_prob(pb, x, keep_count=1)
    assert (to_host(res.n_kept) == 1).all()
    res, _ = run_prob(pb, x, keep_count=T_max + 5)
    assert (to_host(res.n_kept) == T_max).all()


def test_prob_prune_token_outside_vocabulary_goes(pb):
    w = synth.Workload(95, "case", "bf16", 2, 1, 128, 16, 64, 130, 3, 1e-3)
    x = synth.make_prune_inputs(w, trees=[synth.chain_tree(6), synth.star_tree(5)])
    x["token"][0, 3] = 130            # one past the vocabulary: node 3 and the chain below it go
    x["token"][1, 2] = -7
    res, _ = run_prob(pb, x, threshold=0.0)
    assert to_host(res.n_kept).tolist() == [3, 4]
    assert to_host(res.orig_index)[1, :4].tolist() == [0, 1, 3, 4]
    lm = to_host(res.log_marginal)
    assert np.isneginf(lm[0, 3:6]).all() and np.isneginf(lm[1, 2]) and np.isfinite(lm[1, [1, 3, 4]]).all()


# ------------------------------------------------------------------ pruning: degenerate shapes


def test_prune_root_only_trees_and_odd_step_count(pb, oracle):
    """No parent rows at all (every tree is its root), then a batch that mixes root-only trees with
    ordinary ones at a hidden size that gives an odd number of K steps (96 = 3 x 32)."""
    w = synth.Workload(96, "case", "bf16", 3, 1, 128, 16, 96, 130, 3, 1e-3)
    x = synth.make_prune_inputs(w, trees=[synth.chain_tree(1)] * 3)
    res, _ = run_prune(pb, x)
    assert to_host(res.n_kept).tolist() == [1, 1, 1] and to_host(res.cu_nodes).tolist() == [0, 1, 2, 3]
    assert (to_host(res.new_index)[:, 0] == 0).all() and (to_host(res.new_index)[:, 1:] == -1).all()
    res, _ = run_prob(pb, x, threshold=0.5)
    assert to_host(res.n_kept).tolist() == [1, 1, 1]
    rng = np.random.default_rng(96)
    x = synth.make_prune_inputs(w, trees=[synth.chain_tree(1), synth.rank_product_tree(16, 3),
                                         synth.random_tree(rng, 9)])
    res, sents = run_prune(pb, x, [x["hidden_states"]])
    ref, _ = check_prune(oracle, x, res, [x["hidden_states"]], sents)
    assert ref["n_kept"][0] == 1 and ref["n_kept"][1] > 1


# ------------------------------------------------------------------ debug check of a tree


def test_validate_tree_matches_oracle(pb, oracle):
    rng = np.random.default_rng(78)
    shapes = [synth.random_tree(rng, int(T)) for T in (1, 2, 17, 70, 128, 33)]
    n_nodes, parent, _ = synth.pad_trees(shapes, 128)
    depth, anc = oracle.tree_mask(n_nodes, parent)

    def gpu_flags(n, p, d, a):
        tree = pb.Tree(n_nodes=to_dev(n), parent=to_dev(p), depth=None if d is None else to_dev(d),
                       anc=None if a is None else to_dev(a))
        f = pb.propd_validate_tree(tree)
        torch.cuda.synchronize()
        return to_host(f)

    assert (gpu_flags(n_nodes, parent, depth, anc) == 0).all()
    assert (gpu_flags(n_nodes, parent, None, None) == 0).all()
    cases = []
    n2 = n_nodes.copy(); n2[0] = 0; n2[1] = 129; n2[5] = -3
    cases.append((n2, parent, depth, anc))
    p2 = parent.copy(); p2[2, 0] = 0; p2[3, 5] = 5; p2[4, 9] = 40; p2[5, 7] = -1
    cases.append((n_nodes, p2, depth, anc))
    d2 = depth.copy(); d2[3, 69] += 1; d2[1, 1] = 0
    cases.append((n_nodes, parent, d2, anc))
    a2 = anc.copy(); a2[4, 100, 1] ^= np.uint64(1 << 5); a2[2, 3, 0] = np.uint64(0)
    cases.append((n_nodes, parent, depth, a2))
    for n, p, d, a in cases:
        want = oracle.validate_tree(n, p, d, a)
        assert want.any()
        assert (gpu_flags(n, p, d, a) == want).all()


# ------------------------------------------------------------------ random shapes


@pytest.mark.parametrize("seed", list(range(10)))
def test_random_shapes_attention_prune_accept(pb, oracle, seed):
    """Seeded random batch shapes through the three main calls: odd tree slot sizes, few or many
    heads, lengths from empty to several stages, trees of every kind and size in one batch."""
    rng = np.random.default_rng(9000 + seed)
    B = int(rng.integers(1, 7))
    H = int(rng.choice([1, 2, 3, 5, 8]))
    T_max = int(rng.choice([1, 3, 17, 32, 33, 64, 100, 128]))
    L_max = int(rng.choice([1, 31, 32, 65, 200, 513]))
    kinds = ["random", "chain", "star", "one"]
    shapes = []
    for _ in range(B):
        kind = kinds[int(rng.integers(0, len(kinds)))]
        T = int(rng.integers(1, T_max + 1))
        shapes.append({"random": lambda: synth.random_tree(rng, T), "chain": lambda: synth.chain_tree(T),
                       "star": lambda: synth.star_tree(min(T, 40)), "one": lambda: synth.chain_tree(1)}[kind]())
    lens = rng.integers(0, L_max + 1, size=B)
    x = small_bf16_case(300 + seed, B, H, T_max, shapes, lens, L_max=L_max)
    out, sent = run_attention(pb, x)
    check_attention(oracle, x, out, sent)
    # pruning and acceptance on the same trees
    V = int(rng.choice([1003, 4096]))     # wide enough to place a star's tokens with a margin
    Hd = int(rng.choice([32, 64, 96, 256]))
    k = int(rng.integers(1, 12))
    w = synth.Workload(400 + seed, "case", "bf16", B, 1, 128, T_max, Hd, V, k, 1e-3)
    xp = synth.make_prune_inputs(w, trees=shapes)
    res, sents = run_prune(pb, xp, [xp["hidden_states"]])
    check_prune(oracle, xp, res, [xp["hidden_states"]], sents)
    acc = synth.make_accept_inputs(w, xp["n_nodes"], xp["parent"], xp["token"])
    ref = oracle.accept_path(xp["n_nodes"], xp["parent"], xp["token"], acc["logits"], path_stride=T_max)
    got = run_accept(pb, xp["n_nodes"], xp["parent"], xp["token"], acc["logits"], path_stride=T_max)
    for g, r in zip(got, ref):
        assert (g == r).all()
