"""Oracle pins for recursion with several parameters per call and calls nested as arguments
(Ackermann, Takeuchi: the microbenchmarks of Section 6.1): values and invocation counts
against direct recursive evaluation written here, the exactly-once invariant, tag depths."""
import sys

import pytest

import oracle
from oracle import programs as oprog


def _ack(m, n, c, d=1):
    c[0] += 1
    c[1] = max(c[1], d)
    if m == 0:
        return n + 1
    if n == 0:
        return _ack(m - 1, 1, c, d + 1)
    return _ack(m - 1, _ack(m, n - 1, c, d + 1), c, d + 1)


def _tak(x, y, z, c, d=1):
    c[0] += 1
    c[1] = max(c[1], d)
    if y < x:
        return _tak(_tak(x - 1, y, z, c, d + 1), _tak(y - 1, z, x, c, d + 1), _tak(z - 1, x, y, c, d + 1), c, d + 1)
    return z


@pytest.mark.parametrize("name,prog,direct,args", [
    ("ack", oprog.ack_program, _ack, [(0, 0), (0, 5), (1, 0), (1, 2), (2, 0), (2, 3), (3, 2)]),
    ("tak", oprog.tak_program, _tak, [(1, 2, 3), (2, 1, 0), (3, 2, 1), (7, 4, 2), (9, 5, 1)]),
])
def test_values_counts_and_depth_match_direct_recursion(name, prog, direct, args):
    sys.setrecursionlimit(20000)
    for a in args:
        it = oracle.Interpreter(oracle.transform(prog()))
        out = it.run({("in", k): [a[k]] for k in range(len(a))}, 1)[("out", 0)]
        c = [0, 0]
        assert out == [direct(*a, c)], a
        assert len(it.tags) == c[0], a            # one tag per invocation
        assert it.max_tag_len == c[1], a          # tag length = call depth
        assert set(it.fwd_body.values()) == {1}   # every tag fired exactly once


def test_known_values():
    # A(2,n) = 2n+3, A(3,n) = 2^(n+3)-3 (closed forms); tak(18,12,6) = 7 is the classic benchmark value
    it = oracle.Interpreter(oracle.transform(oprog.ack_program()))
    out = it.run({("in", 0): [2, 2, 3, 3], ("in", 1): [0, 4, 0, 3]}, 4)[("out", 0)]
    assert out == [3, 11, 5, 61]


def test_batch_equals_separate_runs():
    args = [(2, 1), (1, 3), (2, 2)]
    it = oracle.Interpreter(oracle.transform(oprog.ack_program()))
    out = it.run({("in", 0): [a[0] for a in args], ("in", 1): [a[1] for a in args]}, len(args))[("out", 0)]
    total = 0
    for a, o in zip(args, out):
        one = oracle.Interpreter(oracle.transform(oprog.ack_program()))
        assert one.run({("in", 0): [a[0]], ("in", 1): [a[1]]}, 1)[("out", 0)] == [o]
        total += len(one.tags)
    assert total == len(it.tags)
