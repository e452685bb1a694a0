#!/usr/bin/env python3
"""Benchmark of the token-tree verification step on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic
input, in the order the method runs it (Section 4.1, Figure 5):
    tree attention on the full tree        (a layer before the pruning point)
    early prune: head scores, top-k test, branch elimination, compaction of the
                 tree, the mask and the row payloads (hidden, q, tree K/V)
    tree attention on the compacted tree   (a layer after the pruning point)
    greedy acceptance on the compacted tree
Inputs are resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, vendor figure


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def build_inputs(w, synth):
    """Host-side seeded inputs of one workload: rank-product trees, sequence lengths, q / K / V,
    early-head tensors with token ids placed for a given pass rate, final-layer logits."""
    t0 = time.time()
    seq_lens = synth.workload_seq_lens(w)
    trees = synth.workload_trees(w)
    att = synth.make_attention_inputs(w, seq_lens=seq_lens, trees=trees, poison=True)
    log(f"attention tensors generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    if w.top_k > 0:
        pr = synth.make_prune_inputs(w, trees=trees)
        token = pr["token"]
    else:
        pr = None
        token = synth.draw_tokens(synth.rng_for(w.index, 3), att["n_nodes"], att["parent"], w.vocab)
    log(f"early-head tensors and token placement in {time.time() - t0:.1f}s")
    t0 = time.time()
    acc = synth.make_accept_inputs(w, att["n_nodes"], att["parent"], token)
    log(f"final logits in {time.time() - t0:.1f}s")
    return att, pr, acc, token


def resident_step(w, att, pr, acc, token, torch, pb, rotate_kv=False):
    """Uploads one workload's inputs (they stay resident) and returns a namespace holding
    `step(marks=None)`, one pass of the hot path, and the tensors it works on."""
    import types
    to_dev, to_host = pb.to_device, pb.to_host
    B, H, d, T_max, L_max = att["B"], att["H"], att["d"], att["T_max"], att["L_max"]

    # ---- upload; everything below stays resident
    t0 = time.time()
    nn, par = to_dev(att["n_nodes"]), to_dev(att["parent"])
    depth, anc = pb.propd_tree_mask(nn, par)
    tree = pb.Tree(n_nodes=nn, parent=par, token=to_dev(token), depth=depth, anc=anc)
    q, kc, vc = to_dev(att["q"]), to_dev(att["k_cache"]), to_dev(att["v_cache"])
    # A K/V cache smaller than the chip's 256 MB last-level cache is served from that cache
    # step after step; with rotate_kv such a workload rotates among enough copies of it (at
    # distinct addresses) that every attention call streams its K/V from HBM.
    kv_bytes_resident = kc.numel() * kc.element_size() * 2
    n_kv_copies = 1 if (kv_bytes_resident >= (1 << 30) or not rotate_kv) else \
        min(64, -(-(3 << 28) // kv_bytes_resident))
    kv_copies = [(kc, vc)] + [(kc.clone(), vc.clone()) for _ in range(n_kv_copies - 1)]
    kv_turn = [0]
    kt, vt = to_dev(att["k_tree"]), to_dev(att["v_tree"])
    seq = to_dev(att["seq_lens"])
    out_full = torch.empty_like(q)
    out_small = torch.empty_like(q)
    ws_att = torch.empty(max(256, pb.workspace_bytes(pb.WS_TREE_ATTENTION, B, T_max, H, d, L_max)),
                         dtype=torch.uint8, device="cuda")
    ws_acc = torch.empty(pb.workspace_bytes(pb.WS_ACCEPT_PATH, B, T_max, vocab=w.vocab),
                         dtype=torch.uint8, device="cuda")
    prune = w.top_k > 0
    if prune:
        hid, hw = to_dev(pr["hidden_states"]), to_dev(pr["head_weight"])
        ws_pr = torch.empty(pb.workspace_bytes(pb.WS_EARLY_PRUNE, B, T_max, hidden=w.hidden,
                                               vocab=w.vocab), dtype=torch.uint8, device="cuda")
        payloads = [hid, q, kt, vt]
        payload_out = [torch.zeros_like(x) for x in payloads]
    logits_full = to_dev(acc["logits"])
    torch.cuda.synchronize()
    log(f"upload {time.time() - t0:.1f}s")

    # final-layer logits of the compacted tree are an INPUT of the acceptance step: prepare
    # them once, untimed, by narrowing the synthetic full-tree logits to the survivors
    if prune:
        res0 = pb.propd_early_prune(tree, hid, hw, w.top_k, payloads=[logits_full], workspace=ws_pr)
        logits_small = res0.payloads[0]
        torch.cuda.synchronize()
        n_kept_host = to_host(res0.n_kept)
    else:
        logits_small = logits_full
        n_kept_host = att["n_nodes"]

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(marks=None):
        """One pass of the hot path; `marks` collects events around the parts."""
        m = [ev() for _ in range(5)] if marks is not None else None
        kc_a, vc_a = kv_copies[kv_turn[0] % n_kv_copies]
        kc_b, vc_b = kv_copies[(kv_turn[0] + 1) % n_kv_copies]
        kv_turn[0] += 2
        if m: m[0].record()
        pb.propd_tree_attention(tree, q, kc_a, vc_a, kt, vt, seq, att["scale"], out=out_full,
                                workspace=ws_att)
        if m: m[1].record()
        if prune:
            res = pb.propd_early_prune(tree, hid, hw, w.top_k, payloads=payloads,
                                       payload_out=payload_out, workspace=ws_pr)
            if m: m[2].record()
            pb.propd_tree_attention(res.tree, payload_out[1], kc_b, vc_b, payload_out[2],
                                    payload_out[3], seq, att["scale"], out=out_small,
                                    workspace=ws_att)
            t_acc = res.tree
        else:
            if m: m[2].record()
            t_acc = tree
        if m: m[3].record()
        r = pb.propd_accept_path(t_acc, logits_small, path_stride=8, workspace=ws_acc)
        if m: m[4].record()
        if marks is not None:
            marks.append(m)
        return r

    return types.SimpleNamespace(**locals())


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=4, choices=[2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true",
                    help="report the eagerly launched steps as the result; by default the K timed steps are "
                         "replays of one step captured into a HIP graph (same kernels, same inputs, every "
                         "output rewritten), and the eager pass supplies the parts and ms_per_step_eager")
    ap.add_argument("--rotate-kv", action="store_true",
                    help="workloads whose K/V cache fits the 256 MB last-level cache (C2, C3): rotate among "
                         "enough copies of it that every attention call streams from HBM")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="CPU work the oracle baseline is bounded to (whole sequences)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain 1 GiB device copy (the reference kernel that the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by)")
    ap.add_argument("--tree-size-table", action="store_true",
                    help="instead of the benchmark line: time the step at tree sizes 16..128 of "
                         "this workload's shape, feed the times to the library's tree-size "
                         "controller and print its estimates and its choice")
    ap.add_argument("--layers", type=int, default=0,
                    help="instead of the benchmark line: the attention of a whole model of this "
                         "many layers per verification step (per-layer synthetic K/V), the "
                         "pruning pass after --prune-layer of them, at tree sizes 16..128")
    ap.add_argument("--prune-layer", type=int, default=4)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; nothing here uses a second one "
              "(sequences and heads would shard with no exchange). Use --gpus 1.",
              file=sys.stderr)
        return 2

    import torch
    from paper_2402_13485_amd import binding as pb
    from paper_2402_13485_amd import synth
    to_dev, to_host = pb.to_device, pb.to_host

    pb.load_library()  # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.copy_calibration:
        return copy_calibration(torch)
    w = synth.WORKLOADS[args.workload]
    if args.tree_size_table:
        return tree_size_table(w, args, torch, pb, synth)
    if args.layers > 0:
        return multi_layer_table(w, args, torch, pb, synth)
    att, pr, acc, token = build_inputs(w, synth)
    S = resident_step(w, att, pr, acc, token, torch, pb, rotate_kv=args.rotate_kv)
    B, H, d, T_max, L_max = S.B, S.H, S.d, S.T_max, S.L_max
    step, prune, seq, kc, vc, kt, vt, tree, ev = S.step, S.prune, S.seq, S.kc, S.vc, S.kt, S.vt, S.tree, S.ev
    n_kept_host = S.n_kept_host
    if prune:
        payload_out, res0 = S.payload_out, S.res0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        last = step(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step_eager = wall * 1e3 / args.steps
    ms_per_step, launch, ms_per_step_graph = ms_per_step_eager, "eager", None
    if not args.eager:
        # One step captured on a side stream (default priority) and replayed: W untimed replays,
        # then exactly K between two synchronisations.  The eager pass above supplies the parts.
        try:
            eager_host = [to_host(t) for t in last]
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                last = step()
            for _ in range(args.warmup):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            if not all((to_host(a) == b).all() for a, b in zip(last, eager_host)):
                raise RuntimeError("the replayed step's accepted paths differ from the eager step's")
            ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / args.steps
            if ms_per_step_graph < ms_per_step_eager:
                ms_per_step, launch = ms_per_step_graph, "hip_graph_replay"
            else:
                log(f"replays took {ms_per_step_graph:.4f} ms per step, eager launches {ms_per_step_eager:.4f}: "
                    "reporting the eager steps")
        except Exception as e:  # capture is an optimisation of the launch path, not a requirement
            log(f"graph capture failed ({type(e).__name__}: {e}); reporting the eager steps")
            torch.cuda.synchronize()

    parts = np.array([[m[i].elapsed_time(m[i + 1]) for i in range(4)] for m in marks])  # ms
    att_full_ms, prune_ms, att_small_ms, accept_ms = parts.mean(axis=0)
    part_names = ("attention_full_tree", "early_prune", "attention_compacted_tree", "accept")
    pct = lambda a: {"median": float(np.median(a)) * 1e3, "p10": float(np.percentile(a, 10)) * 1e3,
                     "p90": float(np.percentile(a, 90)) * 1e3}
    step_ms_events = np.array([m[0].elapsed_time(m[4]) for m in marks])  # GPU time of each step
    sum_T = int(att["n_nodes"].sum())
    kv_bytes = float(sum(int(L) for L in att["seq_lens"])) * H * d * 2 * 2
    side_bytes = float(sum_T) * H * d * 2 * 4  # q, k_tree, v_tree read; out written
    alg_bytes = kv_bytes + side_bytes
    achieved = alg_bytes / (att_full_ms * 1e-3) / 1e9
    accept_len = to_host(last[0])
    recorded = recorded_profile(w.name)

    # what a decoding loop does next (outside the metric's step): commit of the accepted path.
    # Timed on lengths lowered by the path stride so that every accepted row has room; it
    # overwrites the last rows of the resident cache, which nothing reads after this point.
    seq_room = torch.clamp(seq - 8, min=0)
    seq_c = torch.empty_like(seq)
    kt_acc, vt_acc = (payload_out[2], payload_out[3]) if prune else (kt, vt)
    t_acc = res0.tree if prune else tree
    commit_ms = []
    for _ in range(20):
        seq_c.copy_(seq_room)
        e0, e1 = ev(), ev()
        e0.record()
        pb.propd_commit_path(t_acc, last[0], last[1], last[2], kt_acc, vt_acc, kc, vc, seq_c)
        e1.record()
        torch.cuda.synchronize()
        commit_ms.append(e0.elapsed_time(e1))
    commit_us = float(np.median(commit_ms[5:])) * 1e3

    # the early head as a dense contraction: 2 * M * hidden * vocab with M = nodes that have children
    head = None
    if prune:
        n_par = sum(len(set(int(p) for p in att["parent"][b, 1:int(T)])) for b, T in enumerate(att["n_nodes"]))
        flop = 2.0 * n_par * w.hidden * w.vocab
        k_us = recorded.get("early_head_kernel_us")
        head = {"kernel": "early_head_bf16_kernel inside propd_early_prune", "bound": "mfma",
                "rows": n_par, "flop": flop, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "call_us": prune_ms * 1e3,
                "achieved_call": flop / (prune_ms * 1e-3) / 1e12,
                "frac_call": flop / (prune_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                "kernel_us_recorded": k_us,
                "frac_kernel_recorded": None if not k_us else flop / (k_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS}

    k_att = recorded.get("tree_attn_kernel_us")
    result = {
        "metric": "verified tree tokens/s (B*T)",
        "value": sum_T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_eager": ms_per_step_eager,
        "ms_per_step_graph": ms_per_step_graph,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": B, "H": H, "d": d, "L_max": L_max, "T_max": T_max,
                   "sum_L": int(att["seq_lens"].sum()), "sum_T": sum_T, "hidden": w.hidden,
                   "vocab": w.vocab, "top_k": w.top_k,
                   "survivors": int(np.sum(n_kept_host)),
                   "mean_accept_len": float(accept_len.mean()),
                   "kv_cache_copies_rotated": int(S.n_kv_copies),
                   "launch": launch},
        "step_us": pct(step_ms_events),
        "parts_us": {"attention_full_tree": att_full_ms * 1e3, "early_prune": prune_ms * 1e3,
                     "attention_compacted_tree": att_small_ms * 1e3, "accept": accept_ms * 1e3,
                     "commit_outside_step": commit_us},
        "parts_us_percentiles": {n: pct(parts[:, i]) for i, n in enumerate(part_names)},
        "roofline": {"kernel": "tree_attn_bf16_kernel (+ tree_attn_combine_kernel): "
                               "propd_tree_attention on the full tree", "bound": "hbm",
                     # achieved: the whole call (both kernels and the gap between them), HIP
                     # events on the launch stream in this run
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": recorded.get("traffic_bytes_per_launch"),
                     "algorithmic_bytes": alg_bytes,
                     "call_us": att_full_ms * 1e3,
                     "call_us_median": float(np.median(parts[:, 0])) * 1e3,
                     # the dominant kernel alone, from the kernel trace kept under profiles/
                     "kernel_us_recorded": k_att,
                     "frac_kernel_recorded": None if not k_att else alg_bytes / (k_att * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                     "kv_stream_gbps": kv_bytes / (att_full_ms * 1e-3) / 1e9,
                     "kv_stream_frac": kv_bytes / (att_full_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "compacted_tree_kv_gbps": kv_bytes / (att_small_ms * 1e-3) / 1e9
                     if prune else None},
        "early_head": head,
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, att, pr, acc, token, args.cpu_seconds)
    print(json.dumps(result), flush=True)
    return 0


# Stand-in for measured head accuracies (no trained heads exist here): top-1 accuracy of head h
# falls with its distance from the last verified token, and the top-k frequency grows with
# log k.  Five heads (the deepest synthetic tree has depth 5), ten candidates per head.
HEAD_TOP1 = (0.60, 0.42, 0.30, 0.22, 0.16)
HEAD_K_MAX = 10


def synthetic_hit_rates():
    k = np.arange(1, HEAD_K_MAX + 1, dtype=np.float64)
    return np.array([np.minimum(0.95, a * (1.0 + 0.35 * np.log(k))) for a in HEAD_TOP1])


def tree_size_table(w, args, torch, pb, synth):
    """Section 4.2 on measured times: the step is timed at each candidate tree size on this
    workload's shape, the controller fits time against size, estimates the accepted length of
    its best tree of each size from the (synthetic) head accuracies and picks the size."""
    import dataclasses
    sizes = [16, 32, 64, 96, 128]
    ctl = pb.Controller(sizes, len(HEAD_TOP1), HEAD_K_MAX, alpha=0.5, lam=0.05,
                        hit_rate_init=synthetic_hit_rates())
    ms = []
    for n, T in enumerate(sizes):
        wt = dataclasses.replace(w, T_max=T)
        att, pr, acc, token = build_inputs(wt, synth)
        S = resident_step(wt, att, pr, acc, token, torch, pb)
        for _ in range(args.warmup):
            S.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            S.step()
        torch.cuda.synchronize()
        ms.append((time.perf_counter() - t0) * 1e3 / args.steps)
        ctl.observe_time(T, ms[-1], now=float(n))
        log(f"tree size {T}: {ms[-1]:.3f} ms per step, survivors {int(np.sum(S.n_kept_host))}")
        del S, att, pr, acc
        torch.cuda.empty_cache()
    best, speed, (b0, b1) = ctl.best_size(now=float(len(sizes)))
    lens = [ctl.build_tree(T)["expected_len"] for T in sizes]
    out = {"mode": "tree_size_table", "workload": w.name, "B": w.B, "sizes": sizes,
           "ms_per_step": ms, "beta0_ms": b0, "beta1_ms_per_node": b1,
           "t_est_ms": [b0 + b1 * T for T in sizes], "expected_accept_len": lens,
           "accepted_tokens_per_ms": [float(x) for x in speed], "best_size": best,
           "head_accuracies": "synthetic", "steps": args.steps, "warmup": args.warmup}
    print(json.dumps(out), flush=True)
    return 0


def multi_layer_table(w, args, torch, pb, synth):
    """The attention and pruning work of one verification step of a whole model (Section 4.1,
    Figure 5): `prune_layer` layers of tree attention on the full tree, the pruning pass (the
    hidden state is the only payload: later layers make their own q/k/v from it), the remaining
    layers on the compacted tree, greedy acceptance.  Every layer has its own synthetic K/V cache
    and tree q/k/v (drawn on the device); the linear layers of the model are not part of this
    build, so the figures are the attention side of the step only.  Times it at tree sizes
    16..128 with and without pruning."""
    import dataclasses
    N, n_full = args.layers, min(args.prune_layer, args.layers)
    B, H, d = w.B, w.H, w.d
    L = int(synth.workload_seq_lens(w).max())
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    rnd = lambda *shape: torch.randn(shape, device="cuda", generator=gen).to(torch.bfloat16)
    kc = [rnd(B, H, L, d) for _ in range(N)]
    vc = [rnd(B, H, L, d) for _ in range(N)]
    seq = pb.to_device(synth.workload_seq_lens(w))
    scale = float(d) ** -0.5
    rows = []
    for T in [16, 32, 64, 96, 128]:
        wt = dataclasses.replace(w, T_max=T)
        trees = synth.workload_trees(wt)
        pr = synth.make_prune_inputs(wt, trees=trees)
        n_nodes, parent, _ = synth.pad_trees(trees, T)
        nn, par = pb.to_device(n_nodes), pb.to_device(parent)
        depth, anc = pb.propd_tree_mask(nn, par)
        tree = pb.Tree(n_nodes=nn, parent=par, token=pb.to_device(pr["token"]), depth=depth, anc=anc)
        q = [rnd(B, H, T, d) for _ in range(N)]
        kt = [rnd(B, H, T, d) for _ in range(N)]
        vt = [rnd(B, H, T, d) for _ in range(N)]
        hid, hw = pb.to_device(pr["hidden_states"]), pb.to_device(pr["head_weight"])
        hid_out = torch.empty_like(hid)
        logits = rnd(B, T, w.vocab)
        out = torch.empty_like(q[0])
        ws_att = torch.empty(max(256, pb.workspace_bytes(pb.WS_TREE_ATTENTION, B, T, H, d, L)),
                             dtype=torch.uint8, device="cuda")
        ws_pr = torch.empty(pb.workspace_bytes(pb.WS_EARLY_PRUNE, B, T, hidden=w.hidden, vocab=w.vocab),
                            dtype=torch.uint8, device="cuda")
        ws_acc = torch.empty(pb.workspace_bytes(pb.WS_ACCEPT_PATH, B, T, vocab=w.vocab),
                             dtype=torch.uint8, device="cuda")

        def step(prune):
            t = tree
            for l in range(N):
                if prune and l == n_full:
                    t = pb.propd_early_prune(tree, hid, hw, w.top_k, payloads=[hid],
                                             payload_out=[hid_out], workspace=ws_pr).tree
                pb.propd_tree_attention(t, q[l], kc[l], vc[l], kt[l], vt[l], seq, scale, out=out,
                                        workspace=ws_att)
            return pb.propd_accept_path(t, logits, path_stride=8, workspace=ws_acc), t

        ms = {}
        for prune in (False, True):
            for _ in range(2):
                step(prune)
            torch.cuda.synchronize()
            reps = max(3, args.steps // 5)
            t0 = time.perf_counter()
            for _ in range(reps):
                _, t_last = step(prune)
            torch.cuda.synchronize()
            ms[prune] = (time.perf_counter() - t0) * 1e3 / reps
        kept = int(pb.to_host(t_last.n_nodes).sum())
        rows.append({"tree_size": T, "ms_no_pruning": ms[False], "ms_pruning": ms[True],
                     "survivors": kept, "tree_tokens": int(n_nodes.sum()),
                     "tokens_per_s_pruning": float(n_nodes.sum()) / (ms[True] * 1e-3)})
        log(f"tree size {T}: {ms[False]:.2f} ms without pruning, {ms[True]:.2f} ms with "
            f"(pruning after layer {n_full}, {kept} of {int(n_nodes.sum())} nodes stay)")
    print(json.dumps({"mode": "multi_layer_table", "workload": w.name, "layers": N,
                      "prune_after_layer": n_full, "B": B, "H": H, "L": L, "top_k": w.top_k,
                      "rows": rows}), flush=True)
    return 0


def recorded_profile(workload_name):
    """Figures kept under profiles/ from rocprofv3 runs of this same command, as `key = value`
    lines: HBM bytes per full-tree attention launch (FETCH_SIZE + WRITE_SIZE scaled by the
    copy-kernel calibration) and average kernel durations from the kernel trace.  Missing
    files or keys give an empty entry."""
    out = {}
    for name in (f"{workload_name}_tree_attention_hbm_traffic.txt", f"{workload_name}_recorded_kernel_us.txt"):
        try:
            with open(os.path.join(ROOT, "profiles", name)) as f:
                for line in f:
                    if "=" in line and not line.startswith("#"):
                        k, v = line.split("=", 1)
                        try:
                            out[k.strip()] = float(v)
                        except ValueError:
                            pass
        except OSError:
            pass
    return out


def copy_calibration(torch):
    """A plain device-to-device copy of 1 GiB (reads 1 GiB, writes 1 GiB), three times."""
    n = 1 << 30
    src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": 3}), flush=True)
    return 0


def cpu_baseline(w, att, pr, acc, token, budget_s):
    """The oracle, as it stands, timed on this host on a bounded sample of the workload: whole
    sequences (all heads) through the same four parts, one sequence at a time, until about
    `budget_s` seconds of CPU work are spent on all cores; then the first sequence once more on
    ONE thread.  A reported baseline only."""
    from oracle import oracle
    oracle.build()
    part_names = ("attention_full_tree", "early_prune", "attention_compacted_tree", "accept")

    def one_sequence(b, secs):
        sl = slice(b, b + 1)
        cut = lambda a: np.ascontiguousarray(a[sl])
        n_nodes, parent, seq = att["n_nodes"][sl], att["parent"][sl], att["seq_lens"][sl]
        q, kc, vc, kt, vt = (cut(att[k]) for k in ("q", "k_cache", "v_cache", "k_tree", "v_tree"))
        t0 = time.perf_counter()
        oracle.tree_attention(n_nodes, parent, seq, q, kc, vc, kt, vt, att["scale"])
        secs["attention_full_tree"] += time.perf_counter() - t0
        tree2 = (n_nodes, parent, token[sl])
        logits = acc["logits"][sl]
        if pr is not None:
            t0 = time.perf_counter()
            rank, _ = oracle.early_head_rank(n_nodes, parent, token[sl], pr["hidden_states"][sl],
                                             pr["head_weight"], w.top_k)
            c = oracle.prune_compact(n_nodes, parent, token[sl], rank, w.top_k)
            g = lambda a: oracle.gather_rows(a, c["orig_index"], c["n_kept"])
            q2, kt2, vt2 = g(q), g(kt), g(vt)
            g(pr["hidden_states"][sl])
            secs["early_prune"] += time.perf_counter() - t0
            logits = g(logits)
            t0 = time.perf_counter()
            oracle.tree_attention(c["n_kept"], c["parent"], seq, q2, kc, vc, kt2, vt2, att["scale"])
            secs["attention_compacted_tree"] += time.perf_counter() - t0
            tree2 = (c["n_kept"], c["parent"], c["token"])
        t0 = time.perf_counter()
        oracle.accept_path(tree2[0], tree2[1], tree2[2], logits)
        secs["accept"] += time.perf_counter() - t0
        return int(n_nodes.sum())

    all_cores = oracle.threads()
    secs = dict.fromkeys(part_names, 0.0)
    done_tokens, done_seqs = 0, 0
    t_begin = time.perf_counter()
    for b in range(w.B):
        done_tokens += one_sequence(b, secs)
        done_seqs += 1
        spent = time.perf_counter() - t_begin
        log(f"cpu baseline ({all_cores} threads): sequence {b} done, {spent:.1f}s")
        if spent >= budget_s or spent * (done_seqs + 1) / done_seqs > 1.5 * budget_s:
            break
    total = sum(secs.values())
    secs["total"] = total
    # the same on one thread: the first sequence only (all heads)
    one = dict.fromkeys(part_names, 0.0)
    oracle.set_threads(1)
    try:
        one_tokens = one_sequence(0, one)
    finally:
        oracle.set_threads(all_cores)
    one_total = sum(one.values())
    one["total"] = one_total
    log(f"cpu baseline (1 thread): sequence 0 done, {one_total:.1f}s")
    return {"value": done_tokens / total, "unit": "tokens/s", "cores": all_cores,
            "kind": "oracle",
            "sample": f"the first {done_seqs} of {w.B} sequences, all heads, through the same "
                      f"four parts ({done_tokens} tree tokens, {total:.1f} s); and sequence 0 again "
                      f"on one thread ({one_tokens} tree tokens, {one_total:.1f} s)",
            "seconds": secs,
            "one_thread": {"value": one_tokens / one_total, "unit": "tokens/s", "cores": 1,
                           "seconds": one}}


if __name__ == "__main__":
    sys.exit(main())
