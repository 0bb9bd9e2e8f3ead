"""Pins of the oracle's reverse-mode graph (paper Section 4: op-level gradient operators, the
joint function with one label for f and f^grad): closed-form gradient of a scalar recursion,
central finite differences, torch.autograd on the direct-recursion definition, and the
fire-exactly-once invariant in the backward pass."""
import numpy as np
import pytest
import torch

from oracle import transform, differentiate, Interpreter, programs
from tdf_workloads import make_config, SplitMix64


def _env(c):
    F = c["forest"]
    return dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"],
                U=c["U"], u0=c["u0"])


def _small(cfg):
    c = make_config(cfg, n_trees=3, max_leaves=6, vocab=9, hidden=4)
    c["b"] = SplitMix64(11).normal(c["b"].shape[0]) * 0.2
    return c


def _loss_and_grads(c, cell, env=None):
    F = c["forest"]
    B = F.n_trees
    it = Interpreter(transform(differentiate(programs.tree_program(cell, head=True))), env or _env(c))
    out = it.run({("in", 0): F.roots.tolist(), ("in", 1): c["labels"].tolist(),
                  ("gin", 0): [1.0 / B] * B}, B)
    return sum(out[("out", 0)]) / B, it


def test_power_gradient_closed_form():
    # d/dx x^n = n x^(n-1); the gradient returns through Return_i^grad of parameter x and is
    # summed over the two consumers of x in the body
    g = transform(differentiate(programs.power_program()))
    xs, ns = [1.5, -2.0, 0.5, 3.0], [3, 5, 1, 0]
    it = Interpreter(g)
    out = it.run({("in", 0): xs, ("in", 1): ns, ("gin", 0): [1.0] * 4}, 4)
    for b, (x, n) in enumerate(zip(xs, ns)):
        assert out[("out", 0)][b] == pytest.approx(x ** n)
        got = out[("gout", 0)][b]
        assert (0.0 if got is None else got) == pytest.approx(n * x ** (n - 1) if n else 0.0)
    # f and f^grad share labels: the gradient pass visits exactly the forward tags, once each
    assert set(it.bwd_body) == set(it.fwd_body)
    assert set(it.bwd_body.values()) == {1}


def test_joint_graph_structure():
    # one label for Call_i/Return_i of f and of f^grad; the gradient entry is a Merge fed by the
    # gradient Call nodes
    g = transform(differentiate(programs.tree_program("rnn", head=True)))
    fwd = sorted(nd.attr["label"] for nd in g.nodes if nd.op == "call" and nd.attr["kind"] == "in")
    bwd = sorted(nd.attr["label"] for nd in g.nodes if nd.op == "call" and nd.attr["kind"] == "gin")
    assert fwd == bwd == [0, 1, 2]
    gm = [nd for nd in g.nodes if nd.op == "merge_entry" and nd.attr["kind"] == "gin"]
    assert len(gm) == 1 and len(gm[0].ins) == 3
    # op^grad takes the n forward inputs and the output gradient
    cg = [nd for nd in g.nodes if nd.op == "rnn_cell_grad"][0]
    assert len(cg.ins) == 3


@pytest.mark.parametrize("cfg,cell", [(3, "rnn"), (4, "lstm")])
def test_gradients_match_central_finite_differences(cfg, cell):
    c = _small(cfg)
    _, it = _loss_and_grads(c, cell)
    eps = 1e-6
    rng = SplitMix64(5)
    for name, key in (("W", "dW"), ("b", "db"), ("E", "dE")):
        P = c[name]
        flat = P.reshape(-1)
        picks = rng.randint(0, flat.shape[0] - 1, 12)
        if name == "E":                                    # only rows of tokens that occur
            F = c["forest"]
            toks = np.unique(F.token[F.token >= 0])
            picks = [int(toks[i % len(toks)]) * P.shape[1] + int(i % P.shape[1]) for i in picks]
        for idx in picks:
            old = flat[idx]
            flat[idx] = old + eps
            lp, _ = _loss_and_grads(c, cell)
            flat[idx] = old - eps
            lm, _ = _loss_and_grads(c, cell)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            got = it.param_grad[key].reshape(-1)[idx]
            assert got == pytest.approx(fd, rel=2e-6, abs=1e-9), (name, idx)


@pytest.mark.parametrize("cfg,cell", [(3, "rnn"), (4, "lstm")])
def test_gradients_match_autograd_of_direct_recursion(cfg, cell):
    c = make_config(cfg, n_trees=6, max_leaves=10, vocab=15, hidden=5)
    c["b"] = SplitMix64(12).normal(c["b"].shape[0]) * 0.2
    F, H, B = c["forest"], c["H"], c["forest"].n_trees
    loss, it = _loss_and_grads(c, cell)
    E = torch.tensor(c["E"], requires_grad=True)
    W = torch.tensor(c["W"], requires_grad=True)
    b = torch.tensor(c["b"], requires_grad=True)
    U = torch.tensor(c["U"])

    def f(v):
        if F.left[v] < 0:
            return (E[F.token[v]], torch.zeros(H, dtype=torch.float64))
        (hl, cl), (hr, cr) = f(F.left[v]), f(F.right[v])
        z = W @ torch.cat([hl, hr]) + b
        if cell == "rnn":
            return (torch.tanh(z), None)
        i, fl, fr, o = (torch.sigmoid(z[k * H:(k + 1) * H]) for k in range(4))
        cc = i * torch.tanh(z[4 * H:]) + fl * cl + fr * cr
        return (o * torch.tanh(cc), cc)

    total = 0.0
    for bi in range(B):
        lg = U @ f(int(F.roots[bi]))[0]
        total = total + (torch.logsumexp(lg, 0) - lg[int(c["labels"][bi])]) / B
    total.backward()
    assert loss == pytest.approx(float(total.detach()), rel=1e-12)
    np.testing.assert_allclose(it.param_grad["dW"], W.grad.numpy(), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(it.param_grad["db"], b.grad.numpy(), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(it.param_grad["dE"], E.grad.numpy(), rtol=1e-9, atol=1e-14)
    # exactly once per tag in each pass, over the same tags
    assert set(it.fwd_body.values()) == {1} and set(it.bwd_body.values()) == {1}
    assert set(it.bwd_body) == set(it.fwd_body) and len(it.fwd_body) == F.n_nodes


def test_vector_output_with_given_dy():
    # without the head the caller supplies dy per instance: check against autograd
    c = make_config(3, n_trees=4, max_leaves=7, vocab=11, hidden=5)
    F, B = c["forest"], c["forest"].n_trees
    dy = SplitMix64(9).normal(B * 5).reshape(B, 5)
    it = Interpreter(transform(differentiate(programs.tree_program("rnn"))), _env(c))
    it.run({("in", 0): F.roots.tolist(), ("gin", 0): list(dy)}, B)
    E = torch.tensor(c["E"], requires_grad=True)
    W = torch.tensor(c["W"], requires_grad=True)

    def f(v):
        if F.left[v] < 0:
            return E[F.token[v]]
        return torch.tanh(W @ torch.cat([f(F.left[v]), f(F.right[v])]))

    s = sum((f(int(F.roots[b])) * torch.tensor(dy[b])).sum() for b in range(B))
    s.backward()
    np.testing.assert_allclose(it.param_grad["dW"], W.grad.numpy(), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(it.param_grad["dE"], E.grad.numpy(), rtol=1e-9, atol=1e-14)
