"""ORACLE — test infrastructure only, never on the product path.

Reverse-mode automatic differentiation of a program of function graphs (paper Section 4).

For every operator y = op(x_1..x_n) the gradient graph gets an operator op^grad that takes
the forward inputs and the output gradient and yields the input gradients.  A function f is
differentiated as a graph; the result is *joined* with f: the joint function has the inputs
of f plus the gradient of its output (`gin`) and the outputs of f plus the gradients of its
differentiable parameters (`gout`).  A call of f and the matching call of f^grad (`callgrad`)
get the same label, so under equal tags the gradient operators inside f meet the forward
values produced by the same invocation.

Dead tokens make this work without extra machinery: the gradient of an untaken branch is
dead, `snd(x, dy)` (the gradient of a Merge input) is dead wherever x was dead, and `addn`
(the sum over the consumers of a value) waits for every term and adds the live ones.
"""
from .graph import Function, Program, INT, FLOAT, VEC

_INT_OPS = ("eq", "lt", "isleaf", "left", "right", "token")
_VEC_OPS = ("embed", "embed_lstm", "rnn_cell", "lstm_cell", "take_h", "ce_node")


def infer_types(program):
    types = {}
    for f in program.functions.values():
        t = {}
        for idx, nd in enumerate(f.nodes):
            if nd.op == "in":
                ty = f.param_types[nd.attr["k"]]
            elif nd.op == "const":
                ty = INT if isinstance(nd.attr["value"], int) else FLOAT
            elif nd.op in _INT_OPS:
                ty = INT
            elif nd.op in _VEC_OPS:
                ty = VEC
            elif nd.op == "ce_head":
                ty = FLOAT
            elif nd.op == "call":
                ty = program.functions[nd.attr["fn"]].ret_type
            elif nd.op == "switch":
                ty = t[nd.ins[1][0]]
            elif nd.op == "out":
                ty = t[nd.ins[0][0]]
            else:
                tys = [t[s] for s, _ in nd.ins]
                ty = VEC if VEC in tys else FLOAT if FLOAT in tys else INT
            t[idx] = ty
        types[f.name] = t
    return types


def differentiate(program):
    """Return the joint forward+gradient program."""
    types = infer_types(program)
    diff_params = {f.name: [k for k, ty in enumerate(f.param_types) if ty != INT]
                   for f in program.functions.values()}
    new_fns = []
    for f in program.functions.values():
        g = Function(f.name, f.param_types, f.ret_type)
        g.nodes = [type(nd)(nd.op, list(nd.ins), dict(nd.attr)) for nd in f.nodes]
        g.out = f.out
        g._params = list(f._params)
        if f.ret_type != INT:
            _add_gradient_nodes(g, types[f.name], diff_params)
        new_fns.append(g)
    return Program(new_fns, program.result)


def _add_gradient_nodes(g, ty, diff_params):
    n_orig = len(g.nodes)
    gin = g._add("gin", [], k=0)
    contrib = {g.nodes[g.out].ins[0]: [gin]}

    def push(ref, term):
        if ty[ref[0]] != INT and g.nodes[ref[0]].op != "const":
            contrib.setdefault(ref, []).append(term)

    def total(ref):
        terms = contrib.get(ref)
        if not terms:
            return None
        return terms[0] if len(terms) == 1 else g.op("addn", *terms)

    for idx in range(n_orig - 1, -1, -1):
        nd = g.nodes[idx]
        op = nd.op
        if op == "switch":
            dt, df = total((idx, 0)), total((idx, 1))
            if dt is None and df is None:
                continue
            d = g.merge(dt, df) if (dt is not None and df is not None) else (dt or df)
            push(nd.ins[1], d)
            continue
        dy = total((idx, 0))
        if dy is None or op in ("out", "const"):
            continue
        if op == "in":
            g._add("gout", [dy], k=nd.attr["k"])
        elif op == "id":
            push(nd.ins[0], dy)
        elif op == "add":
            push(nd.ins[0], dy)
            push(nd.ins[1], dy)
        elif op == "sub":
            push(nd.ins[0], dy)
            push(nd.ins[1], g.op("neg", dy))
        elif op == "mul":
            push(nd.ins[0], g.op("mul", dy, nd.ins[1]))
            push(nd.ins[1], g.op("mul", dy, nd.ins[0]))
        elif op == "tanh":
            push(nd.ins[0], g.op("tanh_grad", nd.ins[0], dy))
        elif op == "merge":
            for ref in nd.ins:
                push(ref, g.op("snd", ref, dy))
        elif op == "call":
            params = diff_params[nd.attr["fn"]]
            cg, _ = g._add("callgrad", [dy], pair=idx, params=list(params))
            for port, k in enumerate(params):
                push(nd.ins[k], (cg, port))
        elif op in ("embed", "embed_lstm"):
            g.op(op + "_grad", nd.ins[0], dy)
        elif op in ("rnn_cell", "lstm_cell"):
            n, _ = g.op(op + "_grad", nd.ins[0], nd.ins[1], dy)
            push(nd.ins[0], (n, 0))
            push(nd.ins[1], (n, 1))
        elif op == "take_h":
            push(nd.ins[0], g.op("take_h_grad", nd.ins[0], dy))
        elif op == "ce_head":
            push(nd.ins[0], g.op("ce_head_grad", nd.ins[0], nd.ins[1], dy))
        elif op == "ce_node":                       # the node's own loss term joins the gradient of the state
            push(nd.ins[0], g.op("ce_node_grad", nd.ins[0], nd.ins[1], dy))
        else:
            raise ValueError("no gradient operator for " + op)
