"""Pins of the oracle's diagnostic 16-bit variant (oracle/ops_bf16.py): the rounding function against
values fixed by the format, the variant against the unrounded oracle (equal where nothing needs
rounding, within the rounding bound elsewhere)."""
import numpy as np

import oracle
from oracle import ops, ops_bf16, programs as oprog
from tdf_workloads import make_config


def test_bf16_rounding_is_nearest_even_on_eight_bits():
    r = ops_bf16.bf16
    assert r(1.0) == 1.0 and r(-0.5) == -0.5 and r(0.0) == 0.0
    assert r(1.0 + 2.0 ** -7) == 1.0 + 2.0 ** -7            # representable: 8 significant bits
    assert r(1.0 + 2.0 ** -8) == 1.0                        # a tie: to the even neighbour (down)
    assert r(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6        # a tie: to the even neighbour (up)
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7   # just above the tie: up
    x = np.linspace(-4, 4, 10001)
    y = r(x)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8 * (1 + 1e-6))      # half an ulp of 8 significant bits
    assert np.array_equal(r(y), y)                                        # idempotent
    assert np.all((y.astype(np.float32).view(np.uint32) & 0xFFFF) == 0)   # low 16 bits clear


def test_cells_without_anything_to_round_are_unchanged():
    # zero weights: every pre-activation is the bias; with b = 0, h = 0 and the gates are 1/2
    H = 4
    W, b = np.zeros((5 * H, 2 * H)), np.zeros(5 * H)
    sl = np.concatenate([np.ones(H) * 0.5, np.ones(H) * 0.25])
    sr = np.concatenate([np.ones(H) * -0.5, np.ones(H) * 0.75])
    a, r = ops.lstm_cell(W, b, sl, sr), ops_bf16.lstm_cell(W, b, sl, sr)
    assert np.array_equal(a[H:], r[H:])                     # c = (0.25 + 0.75) / 2, exact
    assert np.allclose(a[:H], r[:H], rtol=2.0 ** -8, atol=0)
    Wr = np.zeros((H, 2 * H))
    assert np.array_equal(ops.rnn_cell(Wr, np.zeros(H), sl[:H], sr[:H]), ops_bf16.rnn_cell(Wr, np.zeros(H), sl[:H], sr[:H]))


def _run(c, grad, rounded):
    F = c["forest"]
    B = F.n_trees
    prog = oprog.tree_program(c["cell"], head=True)
    if grad:
        prog = oracle.differentiate(prog)
    env = dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"], U=c["U"], u0=c["u0"], round_bf16=rounded)
    it = oracle.Interpreter(oracle.transform(prog), env)
    inputs = {("in", 0): F.roots.tolist(), ("in", 1): c["labels"].tolist()}
    if grad:
        inputs[("gin", 0)] = [1.0 / B] * B
    out = it.run(inputs, B)[("out", 0)]
    return np.array(out), it.param_grad


def test_rounded_variant_stays_within_the_rounding_bound_of_the_oracle():
    for cfg in (3, 4):
        c = make_config(cfg, n_trees=12, max_leaves=10, hidden=16, vocab=50)
        la, ga = _run(c, True, False)
        lb, gb = _run(c, True, True)
        assert not np.array_equal(la, lb)                     # it does round something
        rel = lambda x, y: np.linalg.norm(x - y) / np.linalg.norm(y)
        assert rel(lb, la) < 5e-3
        for k in ("dW", "db", "dE"):
            assert 0 < rel(gb[k], ga[k]) < 1e-2, k
        # same tags, same firings: rounding changes values only
    # and the head alone (no cell on the path: single-leaf trees) is untouched by the switch
    c = make_config(3, n_trees=6, max_leaves=1, hidden=8, vocab=20)
    la, _ = _run(c, False, False)
    lb, _ = _run(c, False, True)
    assert np.array_equal(la, lb)
