"""Binary trees as flat arrays.  A forest holds, for every tree node, the indices of its
left and right children (-1 at a leaf) and its token id (-1 at an internal node).  Node
indices are global over the forest; `roots[b]` is the root of tree b.
"""
from dataclasses import dataclass
import numpy as np


@dataclass
class Forest:
    left: np.ndarray      # int32[N]
    right: np.ndarray     # int32[N]
    token: np.ndarray     # int32[N]
    roots: np.ndarray     # int64[B]
    n_leaves: np.ndarray  # int64[B]

    @property
    def n_nodes(self):
        return int(self.left.shape[0])

    @property
    def n_trees(self):
        return int(self.roots.shape[0])

    def subset(self, ids):
        """A forest holding only the trees `ids`, nodes renumbered from 0."""
        lefts, rights, toks, roots, nl = [], [], [], [], []
        base = 0
        for b in ids:
            r = int(self.roots[b])
            n = 2 * int(self.n_leaves[b]) - 1          # a tree's nodes are contiguous from its root
            sl = slice(r, r + n)
            l = self.left[sl].astype(np.int64)
            rr = self.right[sl].astype(np.int64)
            lefts.append(np.where(l >= 0, l - r + base, -1))
            rights.append(np.where(rr >= 0, rr - r + base, -1))
            toks.append(self.token[sl])
            roots.append(base)
            nl.append(self.n_leaves[b])
            base += n
        return Forest(np.concatenate(lefts).astype(np.int32), np.concatenate(rights).astype(np.int32),
                      np.concatenate(toks).astype(np.int32), np.asarray(roots, np.int64),
                      np.asarray(nl, np.int64))


def permuted(forest, perm):
    """The same trees with node v renumbered perm[v]: trees no longer occupy contiguous index
    ranges and a child may have a smaller index than its parent."""
    perm = np.asarray(perm, np.int64)
    n = forest.n_nodes
    assert sorted(perm.tolist()) == list(range(n))
    left = np.full(n, -1, np.int32)
    right = np.full(n, -1, np.int32)
    token = np.full(n, -1, np.int32)
    inner = forest.left >= 0
    left[perm[inner]] = perm[forest.left[inner]]
    right[perm[inner]] = perm[forest.right[inner]]
    token[perm] = forest.token
    return Forest(left, right, token, perm[forest.roots], forest.n_leaves.copy())


def _shape_from_splits(n_leaves, split_fn):
    """Nodes in pre-order, root first.  split_fn(L) -> number of leaves of the left child."""
    n = 2 * n_leaves - 1
    left = np.full(n, -1, np.int64)
    right = np.full(n, -1, np.int64)
    nxt = 1
    stack = [(0, n_leaves)]
    while stack:
        v, L = stack.pop()
        if L == 1:
            continue
        k = split_fn(L)
        a, nxt = nxt, nxt + 1
        b, nxt = nxt, nxt + 1
        left[v], right[v] = a, b
        stack.append((b, L - k))
        stack.append((a, k))
    return left, right


def random_split_tree(n_leaves, rng):
    """Internal node over L>=2 leaves: left child gets k ~ U{1..L-1} leaves, right L-k."""
    draws = rng.uniform(max(n_leaves - 1, 1))
    it = iter(draws)
    return _shape_from_splits(n_leaves, lambda L: 1 + min(int(next(it) * (L - 1)), L - 2))


def left_chain_tree(n_leaves):
    """The right child of every internal node is a single leaf (depth n_leaves-1)."""
    return _shape_from_splits(n_leaves, lambda L: L - 1)


def right_chain_tree(n_leaves):
    """The left child of every internal node is a single leaf (depth n_leaves-1)."""
    return _shape_from_splits(n_leaves, lambda L: 1)


def complete_tree(n_leaves):
    """Halving split; n_leaves is a power of two."""
    assert n_leaves & (n_leaves - 1) == 0
    return _shape_from_splits(n_leaves, lambda L: L // 2)


def build_forest(shapes, tokens_fn):
    """shapes: list of (left,right) local arrays; tokens_fn(n) -> n token ids for the leaves
    of one tree, assigned in node order."""
    lefts, rights, toks, roots, nl = [], [], [], [], []
    base = 0
    for l, r in shapes:
        n = l.shape[0]
        leaf = l < 0
        t = np.full(n, -1, np.int64)
        t[leaf] = tokens_fn(int(leaf.sum()))
        lefts.append(np.where(l >= 0, l + base, -1))
        rights.append(np.where(r >= 0, r + base, -1))
        toks.append(t)
        roots.append(base)
        nl.append(int(leaf.sum()))
        base += n
    return Forest(np.concatenate(lefts).astype(np.int32), np.concatenate(rights).astype(np.int32),
                  np.concatenate(toks).astype(np.int32), np.asarray(roots, np.int64),
                  np.asarray(nl, np.int64))
