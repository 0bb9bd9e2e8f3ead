"""Oracle pins for tagged iteration (Section 2.3: Enter <t,d> = <0:t,d>, Next <n:t,d> =
<(n+1):t,d>, Exit <n:t,d> = <t,d>; figure "Dataflow implementation of a while-loop") and for
loops and functions sharing one tag stack (Section 5.1).  Pinned against the three equations
applied by hand to a small loop, closed forms (triangular and tetrahedral numbers, Fibonacci
numbers and their partial sums), math.gcd, and the same loop written as a tail recursion."""
import math

import pytest

import oracle
from oracle import programs as oprog
from oracle.graph import Function, Program, INT

FIB = [0, 1, 1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377]


def _run(prog, *cols):
    n = len(cols[0])
    it = oracle.Interpreter(oracle.transform(prog))
    out = it.run({("in", k): list(c) for k, c in enumerate(cols)}, n)[("out", 0)]
    return out, it


def test_the_three_equations_on_one_loop():
    # n = 3 under root tag (0,): Enter pushes counter 0, Next counts 1, 2, 3, the fourth
    # iteration finds the condition false and Exit pops the counter: the value comes out
    # under the root tag again.
    out, it = _run(oprog.sum_loop_program(), [3])
    assert out == [6]
    assert it.iter_tags == {("S", (k, 0)) for k in range(4)}
    assert it.max_tag_len == 1
    assert not it.tags                                   # no call, no call-context tag
    c = it.count_by_op()
    assert c["enter_0"] == 2 and c["exit_0"] == 1        # one Enter per loop variable
    assert c["next"] == 2 * 3                          # three live Next firings per variable
    assert c["merge_entry"] == 2 * 4 and c["switch"] == 2 * 4 and c["lt"] == 4
    assert c["add"] == 3 and c["sub"] == 3               # the body is dead in the last iteration


def test_static_graph_of_a_loop_is_the_papers_figure():
    g = oracle.transform(oprog.sum_loop_program())
    kinds = [nd.op for nd in g.nodes]
    assert kinds.count("enter") == 2 and kinds.count("next") == 2 and kinds.count("exit") == 1
    for j, nd in enumerate(g.nodes):
        if nd.op == "merge_entry":                       # Merge <- (Enter, Next)
            assert sorted(g.nodes[s].op for s, _ in nd.ins) == ["enter", "next"]
        if nd.op == "exit":                              # Exit <- false side of the Switch
            (src, port), = nd.ins
            assert g.nodes[src].op == "switch" and port == 1
            assert sorted(g.nodes[s].op for s in nd.ctl) == ["enter", "enter"]
        if nd.op == "next":                              # Next <- body
            assert g.nodes[nd.ins[0][0]].op in ("add", "sub")


def test_sum_loop_is_the_triangular_number_and_equals_its_tail_recursion():
    ns = list(range(0, 40, 3))
    out, it = _run(oprog.sum_loop_program(), ns)
    assert out == [n * (n + 1) // 2 for n in ns]
    assert len(it.iter_tags) == sum(n + 1 for n in ns)
    rec, it2 = _run(oprog.sum_recursive_program(), ns)
    assert rec == out
    assert it.max_tag_len == 1 and it2.max_tag_len == max(ns) + 1   # counter replaced vs labels pushed
    assert len(it2.tags) == len(it.iter_tags)            # one tag per trip either way


def test_fib_loop_against_the_table_and_the_recursion():
    ns = list(range(15))
    out, it = _run(oprog.fib_loop_program(), ns)
    assert out == FIB
    rec, _ = _run(oprog.fib_program(), ns)
    assert rec == out
    assert len(it.iter_tags) == sum(n + 1 for n in ns)


def test_gcd_loop_against_math_gcd_and_its_trip_count():
    pairs = [(a, b) for a in (1, 2, 9, 12, 35, 64) for b in (1, 3, 12, 18, 49)]
    out, it = _run(oprog.gcd_loop_program(), [a for a, _ in pairs], [b for _, b in pairs])
    assert out == [math.gcd(a, b) for a, b in pairs]
    trips = 0
    for a, b in pairs:                                   # subtractive Euclid, counted by hand
        while a != b:
            a, b = (a, b - a) if a < b else (a - b, b)
            trips += 1
        trips += 1                                       # the iteration that leaves
    assert len(it.iter_tags) == trips


def test_loop_in_a_loop_has_tags_two_counters_long():
    ns = list(range(9))
    out, it = _run(oprog.nested_loop_program(), ns)
    assert out == [n * (n + 1) // 2 for n in ns]
    assert it.max_tag_len == 2
    outer = sum(n + 1 for n in ns)
    inner = sum(sum(i + 1 for i in range(1, n + 1)) for n in ns)
    assert len(it.iter_tags) == outer + inner
    assert {len(t) for f, t in it.iter_tags if f == "I"} == {3} and {len(t) for f, t in it.iter_tags if f == "O"} == {2}


def test_calls_from_a_loop_body():
    ns = list(range(11))
    out, it = _run(oprog.loop_of_calls_program(), ns)
    assert out == [FIB[n + 2] - 1 for n in ns]           # sum of the first n Fibonacci numbers
    assert len(it.tags) == sum(sum(2 * FIB[i + 1] - 1 for i in range(1, n + 1)) for n in ns)   # fib(i) makes 2 fib(i+1) - 1 calls
    assert it.max_tag_len == 1 + max(ns)                 # counter, then fib(n)'s n labels
    assert all(t[-2] in range(0, 11) for t in it.tags)   # every call tag sits on an iteration counter


def test_loop_in_a_recursive_function_and_a_loop_that_is_not_entered():
    ns = list(range(10))
    out, it = _run(oprog.loop_in_function_program(), ns)
    assert out == [n * (n + 1) * (n + 2) // 6 for n in ns]
    assert len(it.tags) == sum(n + 1 for n in ns)        # tet(n) .. tet(0)
    assert len(it.iter_tags) == sum(sum(k + 1 for k in range(1, n + 1)) for n in ns)   # no loop in tet(0)
    c = it.count_by_op()
    assert c["exit_1"] == sum(ns)                        # live Exits: one per tet(k), k >= 1
    assert c["enter_1"] == 2 * sum(ns)
    assert it.max_tag_len == max(ns) + 1                 # tet(0)'s ten labels; tet(1)'s loop: nine and a counter


def test_every_node_fires_at_most_once_per_tag():
    it = oracle.Interpreter(oracle.transform(oprog.nested_loop_program()))
    seen = set()
    fire = it._fire

    def spy(j, tag):
        assert (j, tag) not in seen
        seen.add((j, tag))
        fire(j, tag)
    it._fire = spy
    assert it.run({("in", 0): [4, 2]}, 2)[("out", 0)] == [10, 3]


def test_loop_graphs_are_checked():
    def sum_graph(name="S"):
        return oprog._counting_loop(name, 2, lambda g, i, acc: (g.op("sub", i, g.const(1)), g.op("add", acc, i)))
    r = Function("result", [INT], INT)
    r.output(r.call("S", r.param(0), r.const(0)))
    with pytest.raises(ValueError):
        Program([r, sum_graph()])                        # a loop graph cannot be called
    r = Function("result", [INT], INT)
    r.output(r.op("add", r.loop("S", r.param(0), r.const(0)), r.loop("S", r.param(0), r.const(1))))
    with pytest.raises(ValueError):
        Program([r, sum_graph()])                        # ... and belongs to one loop node
    r = Function("result", [INT], INT)
    r.output(r.loop("S", r.param(0)))
    with pytest.raises(ValueError):
        Program([r, sum_graph()])                        # one initial value per variable
    r = Function("result", [INT], INT)
    r.output(r.loop("fib", r.param(0)))
    with pytest.raises(ValueError):
        Program([r, oprog.fib_program().functions["fib"]])   # a function is not a loop graph
