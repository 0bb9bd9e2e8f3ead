"""The five workload recipes.  Each returns a dict of NumPy arrays (float64 master copies of
the parameters; the bf16 workloads hold values that are exactly representable in bf16).

  1 fib      : arguments n = 0..20, one evaluation each
  2 treernn  : 256 trees, leaves U{2..50}, uniform split, vocab 10k, D=H=128, fp32
  3 treernn  : 1024 trees, leaves U{2..60}, D=H=300, bf16 values, 5-class head
  4 treelstm : 4096 trees, leaves U{2..128}, 20% left chains, H=D=256, vocab 20k Zipf(1.1)
  5 treernn  : 64 left chains + 64 complete trees of 4096 leaves, H=D=512, bf16 values

`scale` shrinks the number of trees (and, for 5, the leaves per tree) for quick tests while
keeping every distribution the same.
"""
import numpy as np
from .rng import SplitMix64
from .trees import random_split_tree, left_chain_tree, complete_tree, build_forest

BASE_SEED = 20225
CONFIG_NAMES = {1: "fib_0_20", 2: "treernn_fp32_256", 3: "treernn_bf16_1024_grad",
                4: "treelstm_bf16_4096_grad", 5: "treernn_bf16_deep_grad", 6: "gcd_loop_65536"}


def round_to_bf16(x):
    """Round float64/32 values to the nearest bf16 (ties to even); returns float64."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def _zipf_tokens(rng, n, vocab, s):
    p = (np.arange(vocab, dtype=np.float64) + 1.0) ** (-s)
    cdf = np.cumsum(p / p.sum())
    return np.minimum(np.searchsorted(cdf, rng.uniform(n), side="right"), vocab - 1)


def make_config(cfg, n_trees=None, max_leaves=None, seed=None, vocab=None, hidden=None):
    """Build workload `cfg` (1..5).  The optional arguments override the recipe's tree count,
    largest tree, seed, vocabulary and hidden size for reduced-size test cases."""
    rng = SplitMix64((BASE_SEED if seed is None else seed) + cfg)
    if cfg == 1:
        return {"cfg": 1, "kind": "fib", "args": np.arange(0, 21, dtype=np.int64)}
    if cfg == 6:
        # while-loops with data-dependent trip counts: pairs (a, b) uniform in 1..1024 for the
        # subtractive gcd loop; the caller provisions 64 tags (loop iterations) per instance
        B = 65536 if n_trees is None else int(n_trees)
        ab = np.stack([rng.fork(0).randint(1, 1024, B), rng.fork(1).randint(1, 1024, B)], 1).astype(np.int64)
        return {"cfg": 6, "kind": "gcd_loop", "args": ab, "max_tags": 64 * B}

    if cfg == 2:
        B, lo, hi, V, H, bf16, cell = 256, 2, 50, 10000, 128, False, "rnn"
    elif cfg == 3:
        B, lo, hi, V, H, bf16, cell = 1024, 2, 60, 10000, 300, True, "rnn"
    elif cfg == 4:
        B, lo, hi, V, H, bf16, cell = 4096, 2, 128, 20000, 256, True, "lstm"
    elif cfg == 5:
        B, lo, hi, V, H, bf16, cell = 128, 4096, 4096, 10000, 512, True, "rnn"
    else:
        raise ValueError("cfg must be 1..6")
    B = B if n_trees is None else int(n_trees)
    hi = hi if max_leaves is None else int(max_leaves)
    lo = min(lo, hi)
    V = V if vocab is None else int(vocab)
    H = H if hidden is None else int(hidden)

    r_shape, r_tok, r_par, r_lab = rng.fork(0), rng.fork(1), rng.fork(2), rng.fork(3)
    shapes = []
    if cfg == 5:
        for b in range(B):
            shapes.append(left_chain_tree(hi) if b < B // 2 else complete_tree(hi))
    else:
        leaves = r_shape.randint(lo, hi, B)
        chain = (r_shape.uniform(B) < 0.2) if cfg == 4 else np.zeros(B, bool)
        for b in range(B):
            if chain[b]:
                shapes.append(left_chain_tree(int(leaves[b])))
            else:
                shapes.append(random_split_tree(int(leaves[b]), r_shape.fork(b)))
    if cfg == 4:
        tok_fn = lambda n: _zipf_tokens(r_tok, n, V, 1.1)
    else:
        tok_fn = lambda n: r_tok.randint(0, V - 1, n)
    forest = build_forest(shapes, tok_fn)

    rows = 5 * H if cell == "lstm" else H
    E = r_par.normal(V * H).reshape(V, H)
    W = r_par.xavier_uniform(rows, 2 * H)
    b = np.zeros(rows)
    U = r_par.xavier_uniform(5, H)
    u0 = np.zeros(5)
    if bf16:
        E, W = round_to_bf16(E), round_to_bf16(W)
    else:
        E, W = E.astype(np.float32).astype(np.float64), W.astype(np.float32).astype(np.float64)
    U = U.astype(np.float32).astype(np.float64)
    labels = r_lab.randint(0, 4, B)
    node_labels = rng.fork(4).randint(0, 4, forest.n_nodes)   # fully labelled trees: one class per node
    return {"cfg": cfg, "kind": "tree" + cell, "cell": cell, "bf16": bf16, "H": H, "V": V,
            "forest": forest, "E": E, "W": W, "b": b, "U": U, "u0": u0, "labels": labels,
            "node_labels": node_labels,
            "grad": cfg >= 3}
