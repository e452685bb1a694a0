"""The allocation-free entry point, propd_accept_path_static, against propd_accept_path.

Two calls in a row through the C ABI on the library's own fixed device array, the second
with a smaller batch, smaller trees and a smaller vocabulary: every output must equal, bit
for bit, what the workspace form of the call gives on the same inputs.
"""
import numpy as np
import pytest
import torch

from paper_2402_13485_amd import synth
from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu


def accept_case(pb, seed, B, T_max, V, dtype, path_stride):
    rng = np.random.default_rng(seed)
    shapes = [synth.random_tree(rng, int(rng.integers(1, T_max + 1)), max_depth=6) for _ in range(B - 1)]
    shapes.append(synth.rank_product_tree(T_max, 4) if T_max in (32, 64) else synth.chain_tree(min(T_max, 5)))
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = synth.draw_tokens(rng, n_nodes, parent, V)
    w = synth.Workload(61, "case", dtype, B, 1, 128, T_max, 0, V, 0, 0.0)
    logits = synth.make_accept_inputs(w, n_nodes, parent, token)["logits"]
    nn, par = to_dev(n_nodes), to_dev(parent)
    depth, anc = pb.propd_tree_mask(nn, par)
    tree = pb.Tree(n_nodes=nn, parent=par, token=to_dev(token), depth=depth, anc=anc)
    return tree, to_dev(logits), path_stride


def test_static_accept_matches_workspace_form_on_two_calls_in_a_row():
    from paper_2402_13485_amd import binding as pb
    pb.load_library()
    assert torch.cuda.is_available()
    cases = [accept_case(pb, 1, 6, 64, 32000, "bf16", 9),
             accept_case(pb, 2, 3, 32, 1001, "bf16", 3),      # smaller; paths longer than the buffer
             accept_case(pb, 3, 2, 16, 300, "f32", 16)]
    # outputs are allocated before the calls: the entry point itself allocates nothing
    outs = [(torch.full((t.B,), -5, dtype=torch.int32, device="cuda"),
             torch.full((t.B, stride), -5, dtype=torch.int32, device="cuda"),
             torch.full((t.B,), -5, dtype=torch.int32, device="cuda")) for t, _, stride in cases]
    torch.cuda.synchronize()
    for (tree, logits, stride), (alen, path, nxt) in zip(cases, outs):
        pb.propd_accept_path_static(tree, logits, alen, path, nxt)
    torch.cuda.synchronize()
    for (tree, logits, stride), (alen, path, nxt) in zip(cases, outs):
        r_len, r_path, r_next = pb.propd_accept_path(tree, logits, path_stride=stride)
        torch.cuda.synchronize()
        assert (to_host(alen) == to_host(r_len)).all()
        assert (to_host(path) == to_host(r_path)).all()
        assert (to_host(nxt) == to_host(r_next)).all()
        assert (to_host(alen) >= 1).all()


def test_static_accept_rejects_what_does_not_fit():
    from paper_2402_13485_amd import binding as pb
    pb.load_library()
    B, T_max, V = 65, 128, 64          # 8320 nodes: one sequence more than the fixed array holds
    assert B * T_max > pb.STATIC_ACCEPT_MAX_NODES
    n_nodes = torch.ones(B, dtype=torch.int32, device="cuda")
    parent = torch.full((B, T_max), -1, dtype=torch.int32, device="cuda")
    depth, anc = pb.propd_tree_mask(n_nodes, parent)
    tree = pb.Tree(n_nodes=n_nodes, parent=parent, token=torch.zeros_like(parent), depth=depth, anc=anc)
    logits = torch.zeros((B, T_max, V), dtype=torch.bfloat16, device="cuda")
    alen = torch.empty(B, dtype=torch.int32, device="cuda")
    path = torch.empty((B, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(pb.PropdError) as e:
        pb.propd_accept_path_static(tree, logits, alen, path, torch.empty_like(alen))
    assert e.value.code == 2
