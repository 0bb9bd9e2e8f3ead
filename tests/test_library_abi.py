"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, builds and rejects programs, and its Section-3 transformation reproduces the
paper's transformed factorial graph."""
import os
import re
from collections import Counter

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

tdf = pytest.importorskip("paper_2410_20225_amd.tdf")
from paper_2410_20225_amd import programs  # noqa: E402


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "tdf.h")).read()
    names = set(re.findall(r"\b(tdf_[a-z_]+)\s*\(", header))
    assert {"tdf_graph_build", "tdf_eval", "tdf_eval_grad", "tdf_workspace_size", "tdf_graph_info",
            "tdf_graph_destroy", "tdf_last_error"} <= names
    for n in names:
        assert hasattr(tdf.lib, n), n


def test_the_product_library_has_no_test_hook():
    """The switches that make the host pretend its die-private kernels left their dies, or take the
    64-bit offsets of large workspaces on a small one, exist in the tests' build of the library only."""
    here = os.path.dirname(tdf.__file__)
    product = open(os.path.join(here, "libtdf.so"), "rb").read()
    hooks = open(os.path.join(here, "libtdf_hooks.so"), "rb").read()
    for name in (b"TDF_TEST_MIXED_DIES", b"TDF_TEST_WIDE_OFFSETS"):
        assert name not in product and name in hooks, name
    assert b"TDF_TEST_" not in product


_NAMES = {tdf.OP_EQ: "=", tdf.OP_SWITCH: "Switch", tdf.OP_SUB: "-", tdf.OP_MUL: "*", tdf.OP_ADD: "+",
          tdf.OP_ID: "id", tdf.OP_MERGE: "Merge", tdf.SNODE_MERGE_ENTRY: "Merge", tdf.OP_OUT: "out"}


def _label(n):
    if n["kind"] == tdf.SNODE_CALL:
        return "Call_%d" % n["label"]
    if n["kind"] == tdf.SNODE_RETURN:
        return "Return_%d" % n["label"]
    if n["kind"] == tdf.OP_CONST:
        return str(n["imm"])
    return _NAMES[n["kind"]]


def test_transformed_factorial_graph_matches_the_figure():
    want = Counter()
    for line in open(os.path.join(ROOT, "tests", "golden", "fact_transformed_graph.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            want[tuple(line.split())] += 1
    # constants are immediates of their consumers: the figure's Merge->constant control edges
    # have no counterpart
    assert want.pop(("Merge", "1", "control-to-constant")) == 2
    fns, r = programs.fact()
    info = tdf.graph_info(tdf.graph_build(fns, r))
    nodes = info["nodes"]
    got = Counter((_label(nodes[e["src"]]), _label(nodes[e["dst"]]), "control" if e["is_control"] else "data")
                  for e in info["edges"])
    assert got == want
    assert info["n_labels"] == 2


def test_joint_gradient_graph_shares_labels():
    fns, r = programs.tree("rnn", head=True)
    info = tdf.graph_info(tdf.graph_build(fns, r, want_grad=True))
    fwd = sorted(n["label"] for n in info["nodes"] if n["kind"] == tdf.SNODE_CALL and not n["is_grad"])
    bwd = sorted(n["label"] for n in info["nodes"] if n["kind"] == tdf.SNODE_CALL and n["is_grad"])
    assert fwd == bwd == [0, 1, 2]
    entries = [i for i, n in enumerate(info["nodes"]) if n["kind"] == tdf.SNODE_MERGE_ENTRY and n["is_grad"]]
    assert len(entries) == 1
    assert sum(1 for e in info["edges"] if e["dst"] == entries[0]) == 3      # fed by the three Call^grad
    cell_grad = [i for i, n in enumerate(info["nodes"]) if n["kind"] == tdf.OP_RNN_CELL and n["is_grad"]]
    assert len(cell_grad) == 1
    assert sum(1 for e in info["edges"] if e["dst"] == cell_grad[0]) == 3    # (x_l, x_r, dy)


@pytest.mark.parametrize("functions,why", [
    ([("result", 0, [(tdf.OP_CONST, [], 1)])], "no OUT"),
    ([("result", 1, [(tdf.OP_IN, [], 0), (tdf.OP_CALLFN, [(0, 0)], 3), (tdf.OP_OUT, [(1, 0)], 0)])], "undefined callee"),
    ([("result", 1, [(tdf.OP_IN, [], 0), (tdf.OP_CALLFN, [(0, 0)], 1), (tdf.OP_OUT, [(1, 0)], 0)]),
      ("g", 2, [(tdf.OP_IN, [], 0), (tdf.OP_IN, [], 1), (tdf.OP_ADD, [(0, 0), (1, 0)], 0), (tdf.OP_OUT, [(2, 0)], 0)])],
     "arity mismatch"),
    ([("result", 1, [(tdf.OP_IN, [], 0), (tdf.OP_ADD, [(0, 0), (2, 0)], 0), (tdf.OP_OUT, [(1, 0)], 0)])], "forward reference"),
    ([("result", 1, [(tdf.OP_IN, [], 0), (tdf.OP_OUT, [(0, 0)], 0), (tdf.OP_OUT, [(0, 0)], 0)])], "two OUT"),
])
def test_malformed_programs_are_rejected(functions, why):
    with pytest.raises(tdf.TdfError) as ei:
        tdf.graph_build(functions, 0)
    assert ei.value.status == tdf.ERR_BAD_PROGRAM, why


def test_gradient_of_integer_program_is_rejected():
    fns, r = programs.fib()
    with pytest.raises(tdf.TdfError):
        tdf.graph_build(fns, r, want_grad=True)


def test_unused_state_row_is_rejected_in_a_gradient_graph():
    # a cell whose value nobody differentiates would fire, be logged, and its gradient row would be
    # read without ever having been written: such a program is refused when gradients are asked for
    T = tdf
    g = ("g", 1, [(T.OP_IN, [], 0), (T.OP_EMBED, [(0, 0)], 0), (T.OP_OUT, [(1, 0)], 0)])
    nodes = [(T.OP_IN, [], 0),                                   # 0: token id
             (T.OP_CALLFN, [(0, 0)], 1),                         # 1: row, used by the cell and by OUT
             (T.OP_CALLFN, [(0, 0)], 1),                         # 2: a second row
             (T.OP_RNN_CELL, [(1, 0), (2, 0)], 0),               # 3: a cell nobody consumes
             (T.OP_OUT, [(1, 0)], 0)]
    fns = [("result", 1, nodes), g]
    tdf.graph_build(fns, 0)                                      # fine without gradients
    with pytest.raises(tdf.TdfError) as ei:
        tdf.graph_build(fns, 0, want_grad=True)
    assert ei.value.status == tdf.ERR_BAD_PROGRAM
    assert "consumer" in str(ei.value) or "two differentiable" in str(ei.value)


def test_two_vector_values_under_one_tag_are_rejected():
    # a state row is named by the tag that produced it: operators that make rows must exclude each
    # other (the two sides of a Switch, as in the tree function) or sit in functions of their own
    T = tdf
    nodes = [(T.OP_IN, [], 0),
             (T.OP_EMBED, [(0, 0)], 0),
             (T.OP_EMBED, [(0, 0)], 0),
             (T.OP_RNN_CELL, [(1, 0), (2, 0)], 0),
             (T.OP_OUT, [(3, 0)], 0)]
    with pytest.raises(tdf.TdfError) as ei:
        tdf.graph_build([("result", 1, nodes)], 0)
    assert ei.value.status == tdf.ERR_BAD_PROGRAM and "one tag" in str(ei.value)
    for cell in ("rnn", "lstm"):                                 # embed and cell on opposite sides of the Switch
        for kw in ({}, {"head": True}, {"node_loss": True}):
            tdf.graph_build(*programs.tree(cell, **kw))


def test_workspace_size_grows_with_capacity():
    fns, r = programs.tree("lstm", head=True)
    g = tdf.graph_build(fns, r, want_grad=True)
    small = tdf.workspace_size(g, tdf.make_inputs(8, n_args=2, dtype=tdf.BF16, hidden=64, vocab=100,
                                                  n_classes=5, max_tags=1000), True)
    big = tdf.workspace_size(g, tdf.make_inputs(8, n_args=2, dtype=tdf.BF16, hidden=64, vocab=100,
                                                n_classes=5, max_tags=100000), True)
    assert 0 < small < big
    with pytest.raises(tdf.TdfError):
        tdf.workspace_size(g, tdf.make_inputs(8, n_args=1, max_tags=1000), True)   # wrong n_args


@pytest.mark.parametrize("name,prog,grad", [
    ("fact", programs.fact, False), ("fib", programs.fib, False),
    ("treernn", lambda: programs.tree("rnn", False), False),
    ("treelstm_head_grad", lambda: programs.tree("lstm", True), True),
    ("ack", programs.ack, False), ("tak", programs.tak, False),
    ("treelstm_node_loss_grad", lambda: programs.tree("lstm", node_loss=True), True),
])
def test_generated_step_kernels_compile_for_gfx950(name, prog, grad):
    # the firing tables of every workload turn into HIP source that the run-time compiler
    # accepts for gfx950 (no GPU needed); skipped where the run-time compiler is not installed
    fns, r = prog()
    g = tdf.graph_build(fns, r, want_grad=grad)
    try:
        n = tdf.graph_precompile(g, "gfx950")
    except tdf.TdfError as ex:
        if "hiprtc is not available" in str(ex):
            pytest.skip("hiprtc is not available")
        raise
    assert n > 1000


def test_precompile_rejects_missing_arguments():
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    with pytest.raises(tdf.TdfError):
        tdf.graph_precompile(g, "")


_KIND_NAMES = {tdf.OP_IN: "in", tdf.OP_OUT: "out", tdf.OP_CONST: "const", tdf.OP_ADD: "add", tdf.OP_SUB: "sub",
               tdf.OP_MUL: "mul", tdf.OP_EQ: "eq", tdf.OP_LT: "lt", tdf.OP_ID: "id", tdf.OP_SWITCH: "switch",
               tdf.OP_MERGE: "merge", tdf.SNODE_MERGE_ENTRY: "merge_entry", tdf.SNODE_CALL: "call",
               tdf.SNODE_RETURN: "return", tdf.SNODE_ENTER: "enter", tdf.SNODE_NEXT: "next", tdf.SNODE_EXIT: "exit"}


@pytest.mark.parametrize("name", ["sum_loop", "fib_loop", "gcd_loop", "nested_loop", "loop_of_calls", "loop_in_function"])
def test_static_graph_of_loops_is_the_oracles(name):
    # Section 2.3, figure of the while-loop: Enter and Next feed the variables' Merges, Exit hangs
    # on the value that leaves.  Same nodes and edges as the oracle's transformation.
    import oracle
    from oracle import programs as oprog
    from collections import Counter
    fns, r = getattr(programs, name)()
    g = tdf.graph_build(fns, r)
    info = tdf.graph_info(g)
    nodes = info["nodes"]
    got = Counter((_KIND_NAMES[nodes[e["src"]]["kind"]], _KIND_NAMES[nodes[e["dst"]]["kind"]],
                   "control" if e["is_control"] else "data") for e in info["edges"])
    sg = oracle.transform(getattr(oprog, name + "_program")())
    want = Counter((sg.nodes[s].op, sg.nodes[d].op, kind) for s, d, kind in sg.edge_list())
    assert got == want
    assert Counter(_KIND_NAMES[n["kind"]] for n in nodes) == Counter(nd.op for nd in sg.nodes)
    assert info["n_labels"] == len(sg.labels)
    assert tdf.graph_precompile(g, "gfx950") > 0


def test_node_loss_operator_in_the_static_and_the_joint_graph():
    # the per-node loss operator sits between the Merge of a node's state and the function output;
    # its gradient operator takes the two forward inputs and the output gradient (Section 4)
    import oracle
    from oracle import programs as oprog
    from collections import Counter
    names = dict(_KIND_NAMES)
    names.update({tdf.OP_TREE_ISLEAF: "isleaf", tdf.OP_TREE_LEFT: "left", tdf.OP_TREE_RIGHT: "right",
                  tdf.OP_TREE_TOKEN: "token", tdf.OP_EMBED: "embed", tdf.OP_RNN_CELL: "rnn_cell", tdf.OP_CE_NODE: "ce_node"})
    fns, r = programs.tree("rnn", node_loss=True)
    info = tdf.graph_info(tdf.graph_build(fns, r))
    nodes = info["nodes"]
    got = Counter((names[nodes[e["src"]]["kind"]], names[nodes[e["dst"]]["kind"]], "control" if e["is_control"] else "data")
                  for e in info["edges"])
    sg = oracle.transform(oprog.tree_program("rnn", node_loss=True))
    assert got == Counter((sg.nodes[s].op, sg.nodes[d].op, kind) for s, d, kind in sg.edge_list())
    joint = tdf.graph_info(tdf.graph_build(fns, r, want_grad=True))
    g = [i for i, n in enumerate(joint["nodes"]) if n["kind"] == tdf.OP_CE_NODE and n["is_grad"]]
    assert len(g) == 1
    ins = sorted((e["dst_slot"], names.get(joint["nodes"][e["src"]]["kind"]), joint["nodes"][e["src"]]["is_grad"])
                 for e in joint["edges"] if e["dst"] == g[0])
    assert ins == [(0, "merge", 0), (1, "merge_entry", 0), (2, "merge_entry", 1)]   # state, node, gradient of f's output
    fns2, r2 = programs.tree("rnn", head=True)
    with pytest.raises(tdf.TdfError, match="CE_HEAD and CE_NODE"):   # not together with the root-only head
        tdf.graph_build([fns2[0], fns[1]], r2)


def test_malformed_loops_are_rejected():
    T = tdf

    def build(result_nodes, loop_nodes, n_vars=2, want_grad=False):
        fns = [("result", 1, result_nodes), ("S", n_vars, loop_nodes)]
        with pytest.raises(tdf.TdfError) as e:
            tdf.graph_build(fns, 0, want_grad=want_grad)
        assert e.value.status == tdf.ERR_BAD_PROGRAM

    good_loop = programs.sum_loop()[0][1][2]
    n, zero = (0, 0), (1, 0)
    head = [(T.OP_IN, [], 0), (T.OP_CONST, [], 0)]
    build(head + [(T.OP_CALLFN, [n, zero], 1), (T.OP_OUT, [(2, 0)], 0)], good_loop)        # a loop graph is called
    build(head + [(T.OP_LOOP, [n], 1), (T.OP_OUT, [(2, 0)], 0)], good_loop)                # one initial value too few
    build(head + [(T.OP_LOOP, [n, zero], 1), (T.OP_LOOP, [n, zero], 1), (T.OP_ADD, [(2, 0), (3, 0)], 0),
                  (T.OP_OUT, [(4, 0)], 0)], good_loop)                                     # two LOOP nodes on one graph
    build(head + [(T.OP_OUT, [n], 0)], good_loop)                                          # ... and none
    no_next = [nd for nd in good_loop if nd[0] != T.OP_NEXT]
    build(head + [(T.OP_LOOP, [n, zero], 1), (T.OP_OUT, [(2, 0)], 0)], no_next)            # LOOP over a graph without NEXT
    two_next = good_loop[:-1] + [nd for nd in good_loop if nd[0] == T.OP_NEXT] + good_loop[-1:]
    build(head + [(T.OP_LOOP, [n, zero], 1), (T.OP_OUT, [(2, 0)], 0)], two_next)           # two NEXT nodes
    short_next = [(op, ins[:1], imm) if op == T.OP_NEXT else (op, ins, imm) for op, ins, imm in good_loop]
    build(head + [(T.OP_LOOP, [n, zero], 1), (T.OP_OUT, [(2, 0)], 0)], short_next)         # NEXT without a value for a variable
