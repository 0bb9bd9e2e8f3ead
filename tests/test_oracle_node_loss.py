"""Pins of the oracle's per-node losses (fully labelled trees, Section 6; gradient operators of
Section 4): a closed form (zero classifier: every term is log of the class count), autograd of
the direct recursion with a weight on every node's term, central finite differences, the
special case "only the root is labelled" against the head program, and the state going through
the loss operator unchanged."""
import math

import numpy as np
import pytest
import torch

from oracle import transform, differentiate, Interpreter, programs
from tdf_workloads import make_config, SplitMix64


def _cfg(cfg, seed=3, **kw):
    c = make_config(cfg, **kw)
    c["b"] = SplitMix64(seed).normal(c["b"].shape[0]) * 0.2
    c["u0"] = SplitMix64(seed + 1).normal(5) * 0.3
    return c


def _env(c, node_labels, dnode=None):
    F = c["forest"]
    env = dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"], U=c["U"], u0=c["u0"],
               node_label=node_labels)
    if dnode is not None:
        env["dnode"] = dnode
    return env


def _run(c, cell, node_labels, dnode=None, dy=None):
    F, B = c["forest"], c["forest"].n_trees
    prog = programs.tree_program(cell, node_loss=True)
    if dnode is None:
        it = Interpreter(transform(prog), _env(c, node_labels))
        out = it.run({("in", 0): F.roots.tolist()}, B)
    else:
        it = Interpreter(transform(differentiate(prog)), _env(c, node_labels, dnode))
        D = c["H"] * (2 if cell == "lstm" else 1)
        out = it.run({("in", 0): F.roots.tolist(), ("gin", 0): list(np.zeros((B, D)) if dy is None else dy)}, B)
    return out, it


@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
def test_zero_classifier_gives_log_of_the_class_count_per_labelled_node(cell, cfg):
    c = _cfg(cfg, n_trees=5, max_leaves=7, vocab=12, hidden=4)
    c["U"] = np.zeros_like(c["U"])
    c["u0"] = np.zeros(5)
    lab = c["node_labels"].copy()
    lab[::3] = -1                                            # partly labelled: no term there
    out, it = _run(c, cell, lab)
    assert set(it.node_loss) == {v for v in range(c["forest"].n_nodes) if lab[v] >= 0}
    for v, l in it.node_loss.items():
        assert l == pytest.approx(math.log(5.0), rel=1e-14)
    # the state is not changed by the loss operator
    plain = Interpreter(transform(programs.tree_program(cell)), _env(c, lab))
    want = plain.run({("in", 0): c["forest"].roots.tolist()}, c["forest"].n_trees)[("out", 0)]
    for a, b in zip(out[("out", 0)], want):
        assert np.array_equal(a, b)
    assert it.count_by_op()["ce_node"] == c["forest"].n_nodes  # fires once per tag, labelled or not


def _direct(c, cell, node_labels, dnode, dy=None):
    """Direct recursion in torch: per-node losses and the gradients of sum_v dnode[v] loss_v (+ <dy, root state>)."""
    F, H = c["forest"], c["H"]
    E = torch.tensor(c["E"], requires_grad=True)
    W = torch.tensor(c["W"], requires_grad=True)
    b = torch.tensor(c["b"], requires_grad=True)
    U, u0 = torch.tensor(c["U"]), torch.tensor(c["u0"])
    losses = {}

    def f(v):
        if F.left[v] < 0:
            h, cc = E[F.token[v]], torch.zeros(H, dtype=torch.float64)
        else:
            (hl, cl), (hr, cr) = f(F.left[v]), f(F.right[v])
            z = W @ torch.cat([hl, hr]) + b
            if cell == "rnn":
                h, cc = torch.tanh(z), None
            else:
                i, fl, fr, o = (torch.sigmoid(z[k * H:(k + 1) * H]) for k in range(4))
                cc = i * torch.tanh(z[4 * H:]) + fl * cl + fr * cr
                h = o * torch.tanh(cc)
        if node_labels[v] >= 0:
            lg = U @ h + u0
            losses[v] = torch.logsumexp(lg, 0) - lg[int(node_labels[v])]
        return h, cc

    total = 0.0
    for bi in range(F.n_trees):
        h, cc = f(int(F.roots[bi]))
        if dy is not None:
            s = h if cell == "rnn" else torch.cat([h, cc])
            total = total + (torch.tensor(dy[bi]) * s).sum()
    for v, l in losses.items():
        total = total + float(dnode[v]) * l
    total.backward()
    return {v: float(l.detach()) for v, l in losses.items()}, W.grad.numpy(), b.grad.numpy(), E.grad.numpy()


@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
@pytest.mark.parametrize("with_dy", [False, True])
def test_losses_and_gradients_match_autograd_of_the_direct_recursion(cell, cfg, with_dy):
    c = _cfg(cfg, n_trees=6, max_leaves=9, vocab=14, hidden=5)
    F = c["forest"]
    lab = c["node_labels"].copy()
    lab[1::4] = -1
    dnode = SplitMix64(21).normal(F.n_nodes)                 # a different weight on every node's term
    D = c["H"] * (2 if cell == "lstm" else 1)
    dy = SplitMix64(22).normal(F.n_trees * D).reshape(F.n_trees, D) if with_dy else None
    out, it = _run(c, cell, lab, dnode, dy)
    losses, dW, db, dE = _direct(c, cell, lab, dnode, dy)
    assert set(it.node_loss) == set(losses)
    for v in losses:
        assert it.node_loss[v] == pytest.approx(losses[v], rel=1e-12)
    np.testing.assert_allclose(it.param_grad["dW"], dW, rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(it.param_grad["db"], db, rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(it.param_grad["dE"], dE, rtol=1e-9, atol=1e-13)
    assert set(it.fwd_body.values()) == {1} and set(it.bwd_body.values()) == {1}
    assert set(it.bwd_body) == set(it.fwd_body) and len(it.fwd_body) == F.n_nodes


@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
def test_gradients_match_central_finite_differences(cell, cfg):
    c = _cfg(cfg, n_trees=3, max_leaves=6, vocab=9, hidden=4)
    F = c["forest"]
    lab = c["node_labels"]
    dnode = SplitMix64(31).uniform(F.n_nodes) + 0.5

    def objective():
        _, it = _run(c, cell, lab)
        return sum(dnode[v] * l for v, l in it.node_loss.items())

    _, it = _run(c, cell, lab, dnode)
    eps = 1e-6
    rng = SplitMix64(5)
    for name, key in (("W", "dW"), ("b", "db"), ("E", "dE")):
        flat = c[name].reshape(-1)
        picks = [int(i) for i in rng.randint(0, flat.shape[0] - 1, 8)]
        if name == "E":
            toks = np.unique(F.token[F.token >= 0])
            picks = [int(toks[i % len(toks)]) * c["H"] + i % c["H"] for i in picks]
        for idx in picks:
            old = flat[idx]
            flat[idx] = old + eps
            lp = objective()
            flat[idx] = old - eps
            lm = objective()
            flat[idx] = old
            assert it.param_grad[key].reshape(-1)[idx] == pytest.approx((lp - lm) / (2 * eps), rel=2e-6, abs=1e-9), (name, idx)


@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
def test_only_the_root_labelled_is_the_head_program(cell, cfg):
    c = _cfg(cfg, n_trees=5, max_leaves=8, vocab=10, hidden=4)
    F, B = c["forest"], c["forest"].n_trees
    lab = np.full(F.n_nodes, -1)
    lab[F.roots] = c["labels"]
    dnode = np.zeros(F.n_nodes)
    dnode[F.roots] = 1.0 / B
    _, it = _run(c, cell, lab, dnode)
    head = Interpreter(transform(differentiate(programs.tree_program(cell, head=True))), _env(c, lab))
    out = head.run({("in", 0): F.roots.tolist(), ("in", 1): c["labels"].tolist(), ("gin", 0): [1.0 / B] * B}, B)
    for bi in range(B):
        assert it.node_loss[int(F.roots[bi])] == pytest.approx(out[("out", 0)][bi], rel=1e-13)
    for k in ("dW", "db", "dE"):
        np.testing.assert_allclose(it.param_grad[k], head.param_grad[k], rtol=1e-11, atol=1e-15)


def test_joint_graph_has_one_gradient_operator_per_loss_operator():
    g = transform(differentiate(programs.tree_program("rnn", node_loss=True)))
    ops_ = [nd.op for nd in g.nodes]
    assert ops_.count("ce_node") == 1 and ops_.count("ce_node_grad") == 1
    nd = [n for n in g.nodes if n.op == "ce_node_grad"][0]
    assert len(nd.ins) == 3                                  # the two forward inputs and the output gradient
    assert g.nodes[nd.ins[0][0]].op == "merge" and g.nodes[nd.ins[1][0]].op == "merge_entry"
