"""Pins of the oracle on recursive tree networks: counts that have closed forms, values by
direct recursion written out here, and special cases that reduce to textbook / library
routines (one affine+tanh; an Elman RNN over a left chain; LSTM algebra)."""
import numpy as np
import pytest
import torch

from oracle import transform, Interpreter, programs
from tdf_workloads import make_config, left_chain_tree, complete_tree, build_forest, SplitMix64


def _env(c):
    F = c["forest"]
    return dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"],
                U=c["U"], u0=c["u0"])


def _sig(x):
    return 1.0 / (1.0 + np.exp(-x))


def direct_rnn(c, v):
    F = c["forest"]
    if F.left[v] < 0:
        return c["E"][F.token[v]]
    x = np.concatenate([direct_rnn(c, F.left[v]), direct_rnn(c, F.right[v])])
    return np.tanh(c["W"] @ x + c["b"])


def direct_lstm(c, v):
    F, H = c["forest"], c["H"]
    if F.left[v] < 0:
        return c["E"][F.token[v]], np.zeros(H)
    (hl, cl), (hr, cr) = direct_lstm(c, F.left[v]), direct_lstm(c, F.right[v])
    z = c["W"] @ np.concatenate([hl, hr]) + c["b"]
    i, fl, fr, o = _sig(z[:H]), _sig(z[H:2 * H]), _sig(z[2 * H:3 * H]), _sig(z[3 * H:4 * H])
    u = np.tanh(z[4 * H:])
    cc = i * u + fl * cl + fr * cr
    return o * np.tanh(cc), cc


@pytest.mark.parametrize("cfg,cell", [(2, "rnn"), (4, "lstm")])
def test_values_equal_direct_recursion_and_counts(cfg, cell):
    c = make_config(cfg, n_trees=12, max_leaves=9, vocab=40, hidden=5)
    c["b"] = SplitMix64(5).normal(c["b"].shape[0]) * 0.1          # exercise the bias
    F = c["forest"]
    it = Interpreter(transform(programs.tree_program(cell)), _env(c))
    out = it.run({("in", 0): F.roots.tolist()}, F.n_trees)[("out", 0)]
    for b in range(F.n_trees):
        if cell == "rnn":
            want = direct_rnn(c, int(F.roots[b]))
        else:
            want = np.concatenate(direct_lstm(c, int(F.roots[b])))
        np.testing.assert_allclose(out[b], want, rtol=1e-13, atol=1e-15)
    L = int(F.n_leaves.sum())
    cnt = it.count_by_op()
    assert len(it.tags) == 2 * L - F.n_trees == F.n_nodes          # 2L-1 tags per tree
    assert cnt[cell + "_cell"] == L - F.n_trees                    # L-1 cell firings per tree
    assert cnt["embed" if cell == "rnn" else "embed_lstm"] == L    # L leaf firings per tree
    assert set(it.fwd_body.values()) == {1} and len(it.fwd_body) == F.n_nodes


def test_two_leaf_tree_is_one_affine_tanh():
    c = make_config(2, n_trees=1, max_leaves=2, vocab=7, hidden=6)
    F = c["forest"]
    assert F.n_nodes == 3
    it = Interpreter(transform(programs.tree_program("rnn")), _env(c))
    out = it.run({("in", 0): [0]}, 1)[("out", 0)][0]
    x = np.concatenate([c["E"][F.token[F.left[0]]], c["E"][F.token[F.right[0]]]])
    np.testing.assert_allclose(out, np.tanh(c["W"] @ x + c["b"]), rtol=1e-14)


def test_left_chain_is_an_elman_rnn():
    # right child always a leaf: h_k = tanh(W_hh h_{k-1} + W_xh x_k + b), W = [W_hh, W_xh]
    H, n = 6, 9
    rng = SplitMix64(77)
    forest = build_forest([left_chain_tree(n)], lambda k: rng.randint(0, 19, k))
    E, W, b = rng.normal(20 * H).reshape(20, H), rng.xavier_uniform(H, 2 * H), rng.normal(H) * 0.1
    env = dict(left=forest.left, right=forest.right, token=forest.token, E=E, W=W, b=b)
    it = Interpreter(transform(programs.tree_program("rnn")), env)
    out = it.run({("in", 0): [0]}, 1)[("out", 0)][0]
    assert it.max_tag_len == n                     # n-1 path labels + the first call
    # leaf sequence: deepest left leaf first, then the right leaves bottom-up
    v, rights = 0, []
    while forest.left[v] >= 0:
        rights.append(forest.token[forest.right[v]])
        v = forest.left[v]
    seq = [forest.token[v]] + rights[::-1]
    cell = torch.nn.RNNCell(H, H, bias=True, nonlinearity="tanh").double()
    with torch.no_grad():
        cell.weight_hh.copy_(torch.tensor(W[:, :H]))
        cell.weight_ih.copy_(torch.tensor(W[:, H:]))
        cell.bias_ih.copy_(torch.tensor(b))
        cell.bias_hh.zero_()
        h = torch.tensor(E[seq[0]])[None]
        for t in seq[1:]:
            h = cell(torch.tensor(E[t])[None], h)
    np.testing.assert_allclose(out, h[0].numpy(), rtol=1e-12)


def test_lstm_left_chain_with_closed_right_gate_is_a_textbook_lstm():
    # leaves carry c=0, so along a left chain the f_r path contributes nothing and the cell is
    # the standard LSTM c_k = i*u + f*c_{k-1}, h_k = o*tanh(c_k) with input x_k = E[right leaf]
    H, n = 4, 7
    rng = SplitMix64(78)
    forest = build_forest([left_chain_tree(n)], lambda k: rng.randint(0, 9, k))
    E, W, b = rng.normal(10 * H).reshape(10, H), rng.xavier_uniform(5 * H, 2 * H), rng.normal(5 * H) * 0.1
    env = dict(left=forest.left, right=forest.right, token=forest.token, E=E, W=W, b=b)
    it = Interpreter(transform(programs.tree_program("lstm")), env)
    out = it.run({("in", 0): [0]}, 1)[("out", 0)][0]
    v, rights = 0, []
    while forest.left[v] >= 0:
        rights.append(forest.token[forest.right[v]])
        v = forest.left[v]
    seq = [forest.token[v]] + rights[::-1]
    # torch.nn.LSTMCell orders gates (i, f, g, o); ours are (i, f_l, f_r, o, u): drop f_r
    cell = torch.nn.LSTMCell(H, H, bias=True).double()
    rows = np.r_[0:H, H:2 * H, 4 * H:5 * H, 3 * H:4 * H]
    with torch.no_grad():
        cell.weight_hh.copy_(torch.tensor(W[rows][:, :H]))
        cell.weight_ih.copy_(torch.tensor(W[rows][:, H:]))
        cell.bias_ih.copy_(torch.tensor(b[rows]))
        cell.bias_hh.zero_()
        h, cc = torch.tensor(E[seq[0]])[None], torch.zeros(1, H, dtype=torch.float64)
        for t in seq[1:]:
            h, cc = cell(torch.tensor(E[t])[None], (h, cc))
    np.testing.assert_allclose(out[:H], h[0].numpy(), rtol=1e-12)
    np.testing.assert_allclose(out[H:], cc[0].numpy(), rtol=1e-12)


def test_deep_and_complete_tree_counts():
    # complete tree with 2^k leaves: 2^(k+1)-1 tags, longest tag k+1 labels;
    # left chain with n leaves: 2n-1 tags, longest tag n labels
    H = 2
    rng = SplitMix64(3)
    for shape, n, depth in ((complete_tree(64), 64, 7), (left_chain_tree(300), 300, 300)):
        forest = build_forest([shape], lambda k: rng.randint(0, 4, k))
        env = dict(left=forest.left, right=forest.right, token=forest.token,
                   E=rng.normal(5 * H).reshape(5, H), W=rng.xavier_uniform(H, 2 * H), b=np.zeros(H))
        it = Interpreter(transform(programs.tree_program("rnn")), env)
        it.run({("in", 0): [0]}, 1)
        assert len(it.tags) == 2 * n - 1
        assert it.max_tag_len == depth
        assert set(it.fwd_body.values()) == {1}


def test_workload_generators_have_the_stated_shape():
    c = make_config(4, n_trees=400)
    F = c["forest"]
    assert F.n_nodes == int((2 * F.n_leaves - 1).sum())
    assert F.n_leaves.min() >= 2 and F.n_leaves.max() <= 128
    leaf_tok = F.token[F.token >= 0]
    assert 0.10 < np.mean(leaf_tok == 0) < 0.20            # Zipf(1.1): P(id 0) = 0.1456
    assert np.array_equal(make_config(4, n_trees=400)["forest"].left, F.left)   # seeded
    # 20 % of the trees are left chains: the right child of every internal node is a leaf
    chains = 0
    for b in range(F.n_trees):
        r, n = int(F.roots[b]), int(2 * F.n_leaves[b] - 1)
        inner = np.arange(r, r + n)[F.left[r:r + n] >= 0]
        chains += bool(np.all(F.left[F.right[inner]] < 0))
    assert 0.1 < chains / F.n_trees < 0.35
    c5 = make_config(5, n_trees=4, max_leaves=64)
    assert c5["forest"].n_nodes == 4 * 127
    # bf16 workloads hold bf16-representable parameters
    w = c["W"].astype(np.float32).view(np.uint32)
    assert not np.any(w & 0xFFFF)
