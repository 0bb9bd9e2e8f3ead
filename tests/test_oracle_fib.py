"""Pins of the oracle on integer recursion: Fibonacci values and invocation counts have
closed forms (workload 1: fib(n) for n = 0..20 in one batch)."""
import os

from oracle import transform, Interpreter, programs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _fib_table():
    rows = [l for l in open(os.path.join(GOLDEN, "fibonacci.txt")) if not l.startswith("#")]
    return [int(x) for x in " ".join(rows).split()]


def test_values_match_the_table():
    F = _fib_table()
    it = Interpreter(transform(programs.fib_program()))
    out = it.run({("in", 0): list(range(21))}, 21)
    assert out[("out", 0)] == F


def test_invocation_and_firing_counts_have_closed_forms():
    F = _fib_table() + [10946]
    g = transform(programs.fib_program())
    total = 0
    for n in (0, 1, 2, 5, 12, 20):
        it = Interpreter(g)
        it.run({("in", 0): [n]}, 1)
        c = it.count_by_op()
        assert len(it.tags) == 2 * F[n + 1] - 1          # one tag per invocation
        assert c["id"] == F[n + 1]                        # base cases
        assert c["add"] == F[n + 1] - 1                   # additions
        assert c["call_1"] == c["call_2"] == F[n + 1] - 1
        assert it.max_tag_len == max(n, 1)                # longest list of labels
        assert set(it.fwd_body.values()) == {1} and len(it.fwd_body) == len(it.tags)
    it = Interpreter(g)
    it.run({("in", 0): list(range(21))}, 21)
    assert len(it.tags) == sum(2 * F[n + 1] - 1 for n in range(21)) == 57291


def test_batch_equals_separate_evaluations():
    g = transform(programs.fib_program())
    it = Interpreter(g)
    both = it.run({("in", 0): [7, 9]}, 2)[("out", 0)]
    n_both = len(it.tags)
    singles, n_single = [], 0
    for n in (7, 9):
        it = Interpreter(g)
        singles += it.run({("in", 0): [n]}, 1)[("out", 0)]
        n_single += len(it.tags)
    assert both == singles and n_both == n_single
