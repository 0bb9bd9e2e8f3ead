"""ORACLE — test infrastructure only, never on the product path.

Program representation and the transformation of a set of function graphs into one
static tagged graph (paper Section 2.4 "Functions and Recursion" and Section 3
"A Tagged Implementation of Recursion").

A program is a set of named function graphs; one of them is `result`.  A function graph
has input nodes (one per formal parameter), processing nodes, one output node, and call
nodes that carry the name of the function they invoke (Section 2.4).  The transformation
of Section 3 numbers the call nodes, replaces call number i by one Call_i node per formal
parameter, replaces the callee's input nodes by Merge nodes fed by the Call_i nodes,
hangs Return_0..Return_{n-1} on the callee's output, wires Return_i to wherever call i's
result went, and adds a control edge from every Call_i to its Return_i.

Tagged iteration (Section 2.3, figure "Dataflow implementation of a while-loop"): a loop is
written as a graph of its own, the *loop graph*.  Its input nodes are the loop variables of
the current iteration (the Merge nodes of the figure, fed by Enter and by Next), its `next`
node takes the variables' values for the following iteration, and its output node is the value
that leaves the loop (it hangs on the false side of the Switch on the loop condition).  A
`loop` node in another graph supplies the initial values and stands for the value that leaves.
The static graph gets one Enter node per variable at the `loop` node's place, one Next node
per variable, and one Exit node on the loop graph's output value.

Readings where the paper is silent:
  * labels i are unique over the whole program, not per callee;
  * `result` may have input nodes of its own: they are the per-instance program inputs;
  * gradient inputs / outputs of a function (`gin`, `gout`, Section 4) are treated exactly
    like `in` / `out`, and a `callgrad` node shares the label of the call it belongs to;
  * a loop graph belongs to exactly one `loop` node (a while-loop is written in place, it is
    not a shared definition), so an Exit needs no label check; `loop` nodes are numbered
    together with the call nodes, the number only names the loop;
  * values of the enclosing scope that the loop reads are loop variables handed on unchanged;
  * Enter -> Exit control edges, as between Call_i and Return_i: a loop whose initial values
    are dead is not entered and its Exit emits a dead token (see interp.py).
"""
from dataclasses import dataclass, field

INT, FLOAT, VEC = "int", "float", "vec"
TWO_PORT_OPS = ("switch", "rnn_cell_grad", "lstm_cell_grad")


@dataclass
class Node:
    op: str
    ins: list            # list of (node_index, port)
    attr: dict = field(default_factory=dict)


class Function:
    """One named dataflow graph.  Nodes are appended through the helper methods; each helper
    returns a reference (node_index, port) usable as an input of later nodes."""

    def __init__(self, name, param_types, ret_type=INT):
        self.name = name
        self.param_types = list(param_types)
        self.ret_type = ret_type
        self.nodes = []
        self._params = [self._add("in", [], k=k) for k in range(len(self.param_types))]
        self.out = None

    def _add(self, op, ins, **attr):
        self.nodes.append(Node(op, list(ins), dict(attr)))
        return (len(self.nodes) - 1, 0)

    def param(self, k):
        return self._params[k]

    def const(self, value):
        return self._add("const", [], value=value)

    def op(self, name, *ins, **attr):
        return self._add(name, ins, **attr)

    def switch(self, pred, data):
        """Returns (true_side, false_side)."""
        n, _ = self._add("switch", [pred, data])
        return (n, 0), (n, 1)

    def merge(self, *ins):
        return self._add("merge", ins)

    def call(self, fn_name, *args):
        return self._add("call", args, fn=fn_name)

    def loop(self, loop_name, *inits):
        """The while-loop written as loop graph `loop_name`, started with `inits`."""
        return self._add("loop", inits, fn=loop_name)

    def next(self, *values):
        """In a loop graph: the loop variables' values for the next iteration."""
        return self._add("next", values)

    @property
    def is_loop(self):
        return any(nd.op == "next" for nd in self.nodes)

    def output(self, ref):
        self.out = self._add("out", [ref])[0]
        return self.out


class Program:
    def __init__(self, functions, result="result"):
        self.functions = {f.name: f for f in functions}
        self.result = result
        for f in functions:
            if f.out is None:
                raise ValueError("function %s has no output node" % f.name)
            for nd in f.nodes:
                if nd.op == "call":
                    g = self.functions.get(nd.attr["fn"])
                    if g is None:
                        raise ValueError("call to undefined function %s" % nd.attr["fn"])
                    if len(nd.ins) != len(g.param_types):
                        raise ValueError("arity mismatch calling %s" % g.name)
                    if g.is_loop:
                        raise ValueError("%s is a loop graph: it cannot be called" % g.name)
        users = {}
        for f in functions:
            if sum(nd.op == "next" for nd in f.nodes) > 1:
                raise ValueError("loop graph %s has two next nodes" % f.name)
            for nd in f.nodes:
                if nd.op == "next" and len(nd.ins) != len(f.param_types):
                    raise ValueError("next of %s needs one value per loop variable" % f.name)
                if nd.op == "loop":
                    g = self.functions.get(nd.attr["fn"])
                    if g is None or not g.is_loop:
                        raise ValueError("loop over %s, which is not a loop graph" % nd.attr["fn"])
                    if len(nd.ins) != len(g.param_types):
                        raise ValueError("loop %s needs one initial value per variable" % g.name)
                    users[g.name] = users.get(g.name, 0) + 1
        for f in functions:
            if f.is_loop and users.get(f.name, 0) != 1:
                raise ValueError("loop graph %s must belong to exactly one loop node" % f.name)
            if f.is_loop and f.name == result:
                raise ValueError("result cannot be a loop graph")


# --------------------------------------------------------------------------------------
# the static graph
# --------------------------------------------------------------------------------------
@dataclass
class SNode:
    op: str              # original op name, or "merge_entry", "call", "return"
    fn: str              # function graph the node came from
    attr: dict
    ins: list            # data inputs: (snode_index, port)
    ctl: list            # control inputs: snode_index
    outs: list = field(default_factory=list)      # data consumers: (port, dst, dst_slot)
    ctl_outs: list = field(default_factory=list)  # control consumers: (dst, dst_ctl_slot)


class StaticGraph:
    def __init__(self):
        self.nodes = []
        self.inputs = {}        # ("in"|"gin", k) of `result` -> snode index
        self.outputs = {}       # ("out",0) | ("gout",k) of `result` -> snode index
        self.labels = {}        # label -> (caller fn, callee fn)

    def add(self, op, fn, attr=None):
        self.nodes.append(SNode(op, fn, dict(attr or {}), [], []))
        return len(self.nodes) - 1

    def finish(self):
        for j, nd in enumerate(self.nodes):
            for slot, (src, port) in enumerate(nd.ins):
                self.nodes[src].outs.append((port, j, slot))
            for cslot, src in enumerate(nd.ctl):
                self.nodes[src].ctl_outs.append((j, cslot))

    def edge_list(self):
        """[(src_index, dst_index, "data"|"control")], for structural tests."""
        e = []
        for j, nd in enumerate(self.nodes):
            e += [(s, j, "data") for s, _ in nd.ins]
            e += [(s, j, "control") for s in nd.ctl]
        return e


def transform(program):
    """Section 3: turn the set of function graphs into one static graph."""
    g = StaticGraph()
    g.result_fn = program.result
    fns = program.functions
    # number the call nodes (labels) -- any numbering works as long as labels differ;
    # `result` is visited first so that its calls get the smallest labels.
    order = [program.result] + [n for n in fns if n != program.result]
    label_of = {}
    for fname in order:
        for idx, nd in enumerate(fns[fname].nodes):
            if nd.op in ("call", "loop"):
                label_of[(fname, idx)] = len(label_of)
                g.labels[label_of[(fname, idx)]] = (fname, nd.attr["fn"])

    # copy every node; input nodes of callees become Merge, call nodes vanish
    smap = {}                                  # (fname, node, port) -> (snode, port)
    entry = {}                                 # (fname, "in"|"gin", k) -> merge snode
    for fname in order:
        f = fns[fname]
        is_result = fname == program.result
        for idx, nd in enumerate(f.nodes):
            if nd.op in ("in", "gin"):
                k = nd.attr.get("k", 0)
                if is_result:
                    s = g.add(nd.op, fname, nd.attr)
                    g.inputs[(nd.op, k)] = s
                else:
                    s = g.add("merge_entry", fname, {"k": k, "kind": "loop" if f.is_loop else nd.op})
                    entry[(fname, nd.op, k)] = s
                smap[(fname, idx, 0)] = (s, 0)
            elif nd.op in ("call", "callgrad", "loop", "next"):
                continue
            else:
                s = g.add(nd.op, fname, nd.attr)
                if is_result and nd.op in ("out", "gout"):
                    g.outputs[(nd.op, nd.attr.get("k", 0))] = s
                nports = 2 if nd.op in TWO_PORT_OPS else 1
                for p in range(nports):
                    smap[(fname, idx, p)] = (s, p)

    # Call_i (one per formal parameter) and Return_i nodes
    pending_ret = []                           # (return snode, callee fname, kind, k)
    call_nodes = {}                            # (fname, idx) -> [call snodes]
    for fname in order:
        f = fns[fname]
        for idx, nd in enumerate(f.nodes):
            if nd.op == "call":
                lab, callee = label_of[(fname, idx)], nd.attr["fn"]
                cs = []
                for k in range(len(nd.ins)):
                    c = g.add("call", fname, {"label": lab, "k": k, "callee": callee, "kind": "in"})
                    cs.append(c)
                    g.nodes[entry[(callee, "in", k)]].ins.append((c, 0))
                r = g.add("return", fname, {"label": lab, "callee": callee, "kind": "out", "k": 0})
                g.nodes[r].ctl = list(cs)
                call_nodes[(fname, idx)] = cs
                pending_ret.append((r, callee, "out", 0))
                smap[(fname, idx, 0)] = (r, 0)
            elif nd.op == "loop":
                # Enter (one per loop variable) and Exit; the Exit hangs on the loop graph's output
                lab, callee = label_of[(fname, idx)], nd.attr["fn"]
                cs = []
                for k in range(len(nd.ins)):
                    c = g.add("enter", fname, {"label": lab, "k": k, "callee": callee})
                    cs.append(c)
                    g.nodes[entry[(callee, "in", k)]].ins.append((c, 0))
                r = g.add("exit", fname, {"label": lab, "callee": callee})
                g.nodes[r].ctl = list(cs)
                call_nodes[(fname, idx)] = cs
                pending_ret.append((r, callee, "out", 0))
                smap[(fname, idx, 0)] = (r, 0)
            elif nd.op == "next":
                # Next (one per loop variable) feeds the variable's Merge
                cs = []
                for k in range(len(nd.ins)):
                    c = g.add("next", fname, {"k": k})
                    cs.append(c)
                    g.nodes[entry[(fname, "in", k)]].ins.append((c, 0))
                call_nodes[(fname, idx)] = cs
            elif nd.op == "callgrad":
                pair = nd.attr["pair"]
                lab, callee = label_of[(fname, pair)], f.nodes[pair].attr["fn"]
                c = g.add("call", fname, {"label": lab, "k": 0, "callee": callee, "kind": "gin"})
                g.nodes[entry[(callee, "gin", 0)]].ins.append((c, 0))
                call_nodes[(fname, idx)] = [c]
                for port, k in enumerate(nd.attr["params"]):
                    r = g.add("return", fname, {"label": lab, "callee": callee, "kind": "gout", "k": k})
                    g.nodes[r].ctl = [c]
                    pending_ret.append((r, callee, "gout", k))
                    smap[(fname, idx, port)] = (r, 0)

    # wire ordinary data edges (Call_i takes the original argument edge)
    for fname in order:
        f = fns[fname]
        for idx, nd in enumerate(f.nodes):
            if nd.op in ("call", "callgrad", "loop", "next"):
                for k, (src, port) in enumerate(nd.ins):
                    g.nodes[call_nodes[(fname, idx)][k]].ins.append(smap[(fname, src, port)])
            elif nd.op not in ("in", "gin"):
                s, _ = smap[(fname, idx, 0)]
                g.nodes[s].ins = [smap[(fname, src, port)] for src, port in nd.ins]

    # every Return_i hangs on the value that fed the callee's out / gout node
    for r, callee, kind, k in pending_ret:
        f = fns[callee]
        src = None
        for idx, nd in enumerate(f.nodes):
            if nd.op == kind and nd.attr.get("k", 0) == k:
                src = nd.ins[0]
        if src is None:
            raise ValueError("function %s has no %s[%d]" % (callee, kind, k))
        g.nodes[r].ins = [smap[(callee, src[0], src[1])]]

    # out / gout nodes of callees are absorbed by the Return nodes; keep only result's
    keep = [j for j, nd in enumerate(g.nodes)
            if not (nd.op in ("out", "gout") and nd.fn != program.result)]
    remap = {old: new for new, old in enumerate(keep)}
    for nd in g.nodes:
        nd.ins = [(remap[s], p) for s, p in nd.ins]
        nd.ctl = [remap[s] for s in nd.ctl]
    g.nodes = [g.nodes[j] for j in keep]
    g.inputs = {k: remap[v] for k, v in g.inputs.items()}
    g.outputs = {k: remap[v] for k, v in g.outputs.items()}
    g.finish()
    return g
