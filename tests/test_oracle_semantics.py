"""Pins of the oracle's token semantics against the paper's equations (Sections 2.2 and 3)
and its worked factorial example (Section 2.4, figure "The transformed graph of fact")."""
import os
from collections import Counter

import pytest

from oracle import Function, Program, transform, Interpreter, DEAD, programs, INT

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _run(prog, inputs, n):
    it = Interpreter(transform(prog))
    return it.run(inputs, n), it


def test_addition_keeps_the_tag():
    # [[+]](<t,a>,<t,b>) = <t,a+b>: instance b only ever meets instance b
    r = Function("result", [INT, INT], INT)
    r.output(r.op("add", r.param(0), r.param(1)))
    out, _ = _run(Program([r]), {("in", 0): [1, 20, 300], ("in", 1): [4, 50, 600]}, 3)
    assert out[("out", 0)] == [5, 70, 900]


@pytest.mark.parametrize("pred,expect_true,expect_false", [(1, 7, DEAD), (0, DEAD, 7)])
def test_switch_equations(pred, expect_true, expect_false):
    # Switch(<t,true>,<t,d>) = (<t,d>,<t,*>) and mirrored for false
    r = Function("result", [INT, INT], INT)
    t, f = r.switch(r.param(0), r.param(1))
    m = r.merge(r.op("id", t), r.op("id", f))
    r.output(m)
    g = transform(Program([r]))
    it = Interpreter(g)
    out = it.run({("in", 0): [pred], ("in", 1): [7]}, 1)
    assert out[("out", 0)] == [7]
    merge = [j for j, nd in enumerate(g.nodes) if nd.op == "merge"][0]
    vals = it.slots[(merge, (0,))][0]
    # the Merge saw the live side; the dead side either arrived as * or had not arrived yet
    assert vals[0] in (expect_true, None) and vals[1] in (expect_false, None)
    assert (vals[0] is DEAD) != (vals[1] is DEAD) or None in vals


def test_merge_forwards_the_live_input_and_ops_propagate_hiatons():
    # neg(false side) is dead when pred is true: the Merge must output the live value
    r = Function("result", [INT, INT], INT)
    t, f = r.switch(r.param(0), r.param(1))
    r.output(r.merge(r.op("add", t, r.const(100)), r.op("neg", f)))
    out, it = _run(Program([r]), {("in", 0): [1, 0], ("in", 1): [7, 7]}, 2)
    assert out[("out", 0)] == [107, -7]
    counts = it.count_by_op()
    assert counts["add"] == 1 and counts["neg"] == 1      # live firings only


def test_factorial_example_value_and_tags():
    # result = fact(3)+5 = 11; invocations run under tags [0], [1,0], [1,1,0]
    out, it = _run(programs.fact_program(), {}, 1)
    assert out[("out", 0)] == [11]
    assert sorted(t[:-1] for t in it.tags) == [(0,), (1, 0), (1, 1, 0)]
    c = it.count_by_op()
    assert c["call_0"] == 1 and c["call_1"] == 2 and c["return_0"] == 1 and c["return_1"] == 2
    assert c["mul"] == 2 and c["id"] == 1


def test_call_pushes_and_return_pops_the_label():
    # Call_i <t,d> = <i:t,d>; Return_i <i:t,d> = <t,d>: g(x)=x+1 called twice from result
    gfn = Function("g", [INT], INT)
    gfn.output(gfn.op("add", gfn.param(0), gfn.const(1)))
    r = Function("result", [INT], INT)
    r.output(r.op("mul", r.call("g", r.param(0)), r.call("g", r.op("add", r.param(0), r.const(10)))))
    out, it = _run(Program([r, gfn]), {("in", 0): [2, 5]}, 2)
    assert out[("out", 0)] == [3 * 13, 6 * 16]
    assert it.tags == {(0, 0), (1, 0), (0, 1), (1, 1)}
    # g's output fans out to Return_0 and Return_1; the wrong label produces no output
    assert it.dropped == 4


def test_return_label_check_drops_exactly_the_other_returns():
    out, it = _run(programs.fib_program(), {("in", 0): [10]}, 1)
    n_tags = len(it.tags)
    assert it.dropped == 2 * n_tags          # three Returns hang on fib's output


def test_dead_call_creates_no_tag():
    # the untaken recursive branch must not enter the callee, else fib would not terminate
    out, it = _run(programs.fib_program(), {("in", 0): [1]}, 1)
    assert out[("out", 0)] == [1]
    assert it.tags == {(0, 0)}
    c = it.count_by_op()
    assert c["call_1"] == 0 and c["call_2"] == 0 and c["return_1"] == 0


def _label(nd):
    if nd.op == "call":
        return "Call_%d" % nd.attr["label"]
    if nd.op == "return":
        return "Return_%d" % nd.attr["label"]
    if nd.op == "const":
        return str(nd.attr["value"])
    return {"merge_entry": "Merge", "merge": "Merge", "eq": "=", "switch": "Switch", "sub": "-",
            "mul": "*", "add": "+"}.get(nd.op, nd.op)


def test_transformed_factorial_graph_matches_the_figure():
    want = Counter()
    for line in open(os.path.join(GOLDEN, "fact_transformed_graph.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            want[tuple(line.split())] += 1
    # reading: constants are immediates of their consumers, so the two Merge->constant
    # control edges of the figure have no counterpart
    assert want.pop(("Merge", "1", "control-to-constant")) == 2
    g = transform(programs.fact_program())
    got = Counter((_label(g.nodes[s]), _label(g.nodes[d]), kind) for s, d, kind in g.edge_list())
    assert got == want
    assert Counter(_label(n) for n in g.nodes) == Counter(
        ["Call_0", "Call_1", "Return_0", "Return_1", "Merge", "Merge", "=", "Switch", "id", "-",
         "*", "+", "1", "1", "3", "5", "out"])


def test_multi_parameter_call_gets_one_call_node_per_parameter():
    # Section 3: the i-th call of an m-parameter function becomes m Call_i nodes, each with a
    # control edge to Return_i
    g = transform(programs.power_program())
    calls = [nd for nd in g.nodes if nd.op == "call" and nd.attr["label"] == 1]
    assert sorted(nd.attr["k"] for nd in calls) == [0, 1]
    ret = [nd for nd in g.nodes if nd.op == "return" and nd.attr["label"] == 1][0]
    assert len(ret.ctl) == 2
    out, it = Interpreter(g).run({("in", 0): [2.0], ("in", 1): [10]}, 1), None
    assert out[("out", 0)] == [1024.0]


def test_undefined_callee_and_arity_are_rejected():
    r = Function("result", [INT], INT)
    r.output(r.call("nope", r.param(0)))
    with pytest.raises(ValueError):
        Program([r])
    g = Function("g", [INT, INT], INT)
    g.output(g.op("add", g.param(0), g.param(1)))
    r = Function("result", [INT], INT)
    r.output(r.call("g", r.param(0)))
    with pytest.raises(ValueError):
        Program([r, g])
