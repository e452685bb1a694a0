"""A toy deterministic "model" and the per-step inputs of a greedy decoding loop, for the
tests of acceptance + commit.  Input construction only: neither the oracle nor the GPU
library is called here."""
import numpy as np

from paper_2402_13485_amd import synth

VOCAB = 53


def model_next(prefix):
    """The toy model's greedy choice after a token prefix."""
    acc = 7 * len(prefix) + 3
    for i, t in enumerate(prefix):
        acc = (acc * 31 + (i + 1) * (int(t) + 11)) % 1000003
    return acc % VOCAB


def kv_row(token, pos, h, d, which):
    """The K (which=0) or V (which=1) row the toy model would compute for a token at a position:
    small integers, exact in bf16 and fp32."""
    base = (int(token) * 7 + pos * 3 + h * 5 + which * 11) % 64
    return (base + (np.arange(d) % 8)).astype(np.float32)


def root_path(parent, i):
    path = []
    while i >= 0:
        path.append(i)
        i = int(parent[i])
    return path[::-1]


def build_step(rng, prefixes, roots, H, d, T_max, dtype, p_follow=0.65):
    """Trees, candidate tokens, final logits and tree K/V of one step.
    prefixes[b]: tokens whose rows are in the cache; roots[b]: the token fixed by the last step."""
    B = len(prefixes)
    shapes = [synth.random_tree(rng, int(rng.integers(1, T_max + 1))) for _ in range(B)]
    n_nodes, parent, _ = synth.pad_trees(shapes, T_max)
    token = np.full((B, T_max), -1, np.int32)
    logits = rng.normal(size=(B, T_max, VOCAB)).astype(np.float32)
    k_tree = np.zeros((B, H, T_max, d), np.float32)
    v_tree = np.zeros((B, H, T_max, d), np.float32)
    for b in range(B):
        T = int(n_nodes[b])
        used = {}
        for i in range(T):
            p = int(parent[b, i])
            if i == 0:
                token[b, i] = roots[b]
            else:
                path_tokens = [int(token[b, j]) for j in root_path(parent[b], p)]
                want = model_next(list(prefixes[b]) + path_tokens)
                taken = used.setdefault(p, set())
                if want not in taken and rng.random() < p_follow:
                    tok = want
                else:
                    tok = int(rng.integers(0, VOCAB))
                    while tok in taken or tok == want:
                        tok = int(rng.integers(0, VOCAB))
                taken.add(tok)
                token[b, i] = tok
            path = root_path(parent[b], i)
            seq = list(prefixes[b]) + [int(token[b, j]) for j in path]
            logits[b, i, model_next(seq)] = 9.0  # the model's choice after this node
            pos = len(prefixes[b]) + len(path) - 1
            for h in range(H):
                k_tree[b, h, i] = kv_row(token[b, i], pos, h, d, 0)
                v_tree[b, h, i] = kv_row(token[b, i], pos, h, d, 1)
    if dtype == "bf16":
        conv = synth.f32_to_bf16_bits
        return n_nodes, parent, token, conv(logits), conv(k_tree), conv(v_tree)
    return n_nodes, parent, token, logits, k_tree, v_tree


def expected_cache_rows(tokens, H, d, which, dtype):
    """Rows [H, len(tokens), d] the toy model computes for a token sequence from position 0."""
    rows = np.stack([np.stack([kv_row(t, pos, h, d, which) for pos, t in enumerate(tokens)])
                     for h in range(H)]) if len(tokens) else np.zeros((H, 0, d), np.float32)
    return synth.f32_to_bf16_bits(rows) if dtype == "bf16" else rows
