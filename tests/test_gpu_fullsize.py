"""GPU parity at the full benchmark sizes (workloads C2..C5 of the benchmark spec), through the
C ABI in the launch configuration bench.py times.

Integer outputs (prune masks, compaction indices, compacted trees and masks, accepted
paths) are compared in full and bit for bit.  Attention outputs are compared in full too:
every (sequence, head, node) row of the full tree and of the compacted tree against the
oracle (bf16: |gpu - ref| <= 2e-2 against the unrounded fp64 result), and padding rows for
being untouched.
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
    binding.load_library()
    assert torch.cuda.is_available()
    return binding


def check_attention_everywhere(oracle, x, n_nodes, parent, q, kt, vt, out_dev, sent):
    """Every row of every (sequence, head) unit against the oracle; rows beyond a tree untouched."""
    ref = oracle.tree_attention(n_nodes, parent, x["seq_lens"], q, x["k_cache"], x["v_cache"], kt, vt,
                                x["scale"])
    raw = to_host(out_dev)
    got = synth.as_float(raw).astype(np.float64)
    worst = 0.0
    for b, T in enumerate(n_nodes):
        T = int(T)
        assert np.isfinite(got[b, :, :T]).all()
        worst = max(worst, float(np.abs(got[b, :, :T] - ref[b, :, :T]).max()))
        assert (raw[b, :, T:] == sent[b, :, T:]).all()
    assert worst <= 2e-2, worst
    return worst


def run_workload(pb, oracle, index):
    w = synth.WORKLOADS[index]
    seq_lens = synth.workload_seq_lens(w)
    trees = synth.workload_trees(w)
    xa = synth.make_attention_inputs(w, seq_lens=seq_lens, trees=trees)
    prune = w.top_k > 0
    if prune:
        xp = synth.make_prune_inputs(w, trees=trees)
        token = xp["token"]
    else:
        token = synth.draw_tokens(synth.rng_for(w.index, 3), xa["n_nodes"], xa["parent"], w.vocab)
    acc = synth.make_accept_inputs(w, xa["n_nodes"], xa["parent"], token)

    nn, par = to_dev(xa["n_nodes"]), to_dev(xa["parent"])
    depth, anc = pb.propd_tree_mask(nn, par)
    d_ref, a_ref = oracle.tree_mask(xa["n_nodes"], xa["parent"])
    assert (to_host(depth) == d_ref).all() and (u64(anc) == a_ref).all()
    tree = pb.Tree(n_nodes=nn, parent=par, token=to_dev(token), depth=depth, anc=anc)
    q, kt, vt = to_dev(xa["q"]), to_dev(xa["k_tree"]), to_dev(xa["v_tree"])
    kc, vc, seq = to_dev(xa["k_cache"]), to_dev(xa["v_cache"]), to_dev(xa["seq_lens"])
    sent = sentinel_like(xa["q"])

    # 1. attention on the full tree
    out = to_dev(sent)
    pb.propd_tree_attention(tree, q, kc, vc, kt, vt, seq, xa["scale"], out=out)
    torch.cuda.synchronize()
    check_attention_everywhere(oracle, xa, xa["n_nodes"], xa["parent"], xa["q"], xa["k_tree"],
                               xa["v_tree"], out, sent)
    if not prune:
        ref_acc = oracle.accept_path(xa["n_nodes"], xa["parent"], token, acc["logits"])
        got = pb.propd_accept_path(tree, to_dev(acc["logits"]))
        torch.cuda.synchronize()
        for g, r in zip(got, ref_acc):
            assert (to_host(g) == r).all()
        assert to_host(got[0]).tolist() == [len(c) for c in acc["chains"]]
        return

    # 2. early prune with the payloads the next layer needs, plus the final logits
    lg = to_dev(acc["logits"])
    res = pb.propd_early_prune(tree, to_dev(xp["hidden_states"]), to_dev(xp["head_weight"]),
                               w.top_k, payloads=[q, kt, vt, lg], want_rank=True)
    torch.cuda.synchronize()
    rank_ref, margin = oracle.early_head_rank(xp["n_nodes"], xp["parent"], token,
                                              xp["hidden_states"], xp["head_weight"], w.top_k)
    assert margin[np.isfinite(margin)].min() >= 0.999 * w.tau
    ref = oracle.prune_compact(xp["n_nodes"], xp["parent"], token, rank_ref, w.top_k)
    rank = to_host(res.rank)
    valid = rank_ref >= 0
    assert ((rank >= w.top_k) == (rank_ref >= w.top_k))[valid].all()
    assert (u64(res.keep_bits) == ref["keep_bits"]).all()
    for name in ("new_index", "orig_index", "n_kept", "cu_nodes"):
        assert (to_host(getattr(res, name)) == ref[name]).all(), name
    for name in ("parent", "token", "depth"):
        assert (to_host(getattr(res.tree, name)) == ref[name]).all(), name
    assert (u64(res.tree.anc) == ref["anc"]).all()
    g = lambda a: oracle.gather_rows(a, ref["orig_index"], ref["n_kept"])
    q2, kt2, vt2, lg2 = res.payloads
    for b in range(w.B):  # survivor rows of every payload, bit for bit
        n = int(ref["n_kept"][b])
        assert (to_host(q2)[b, :, :n] == xa["q"][b][:, ref["orig_index"][b, :n]]).all()
        assert (to_host(lg2)[b, :n] == acc["logits"][b, ref["orig_index"][b, :n]]).all()
    frac = ref["n_kept"].sum() / xa["n_nodes"].sum()
    assert 0.1 < frac < 0.45  # the paper's pruning rates are 57.6 .. 79 percent (Table 2)

    # 3. attention on the compacted tree, fed with the device outputs of the prune call
    out2 = to_dev(sent)
    pb.propd_tree_attention(res.tree, q2, kc, vc, kt2, vt2, seq, xa["scale"], out=out2)
    alen, path, nxt = pb.propd_accept_path(res.tree, lg2, path_stride=8)
    torch.cuda.synchronize()
    check_attention_everywhere(oracle, xa, ref["n_kept"], ref["parent"], g(xa["q"]), g(xa["k_tree"]),
                               g(xa["v_tree"]), out2, sent)
    # a surviving node computes the same thing before and after pruning (Section 4.1)
    a, b2 = host_f64(out), host_f64(out2)
    for b in range(w.B):
        n = int(ref["n_kept"][b])
        assert np.abs(b2[b, :, :n] - a[b][:, ref["orig_index"][b, :n]]).max() <= 2e-2

    # 4. acceptance on the compacted tree
    r_len, r_path, r_next = oracle.accept_path(ref["n_kept"], ref["parent"], ref["token"],
                                               g(acc["logits"]), path_stride=8)
    assert (to_host(alen) == r_len).all() and (to_host(path) == r_path).all()
    assert (to_host(nxt) == r_next).all()
    # and it is the unpruned accepted chain cut at its first pruned node
    f_len, f_path, _ = oracle.accept_path(xa["n_nodes"], xa["parent"], token, acc["logits"],
                                          path_stride=8)
    for b in range(w.B):
        kept = []
        for node in f_path[b, : f_len[b]]:
            if ref["new_index"][b, node] < 0:
                break
            kept.append(int(node))
        assert [int(ref["orig_index"][b, j]) for j in r_path[b, : r_len[b]]] == kept


@pytest.mark.parametrize("index", [2, 3, 4, 5])
def test_full_size_workload(pb, oracle, index):
    print(f"workload C{index}", flush=True)
    run_workload(pb, oracle, index)
