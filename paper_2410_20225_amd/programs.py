"""Program descriptions in the library's input language (a set of function graphs, one of
them `result`; paper Section 2.4), as plain tuples for tdf.graph_build:
(name, n_params, [(op, [(node, port), ...], imm), ...]).
"""
from . import tdf as T


class _Fn:
    def __init__(self, name, n_params):
        self.name, self.n_params, self.nodes = name, n_params, []

    def add(self, op, ins=(), imm=0):
        self.nodes.append((op, list(ins), imm))
        return (len(self.nodes) - 1, 0)

    def desc(self):
        return (self.name, self.n_params, self.nodes)


def fact():
    """result = fact(3)+5; fact(n) = if n==1 then n else n*fact(n-1)  (the paper's example)."""
    r = _Fn("result", 0)
    call = r.add(T.OP_CALLFN, [r.add(T.OP_CONST, imm=3)], imm=1)
    r.add(T.OP_OUT, [r.add(T.OP_ADD, [r.add(T.OP_CONST, imm=5), call])])
    f = _Fn("fact", 1)
    n = f.add(T.OP_IN, imm=0)
    sw = f.add(T.OP_SWITCH, [f.add(T.OP_EQ, [f.add(T.OP_CONST, imm=1), n]), n])
    then, other = (sw[0], 0), (sw[0], 1)
    rec = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [other, f.add(T.OP_CONST, imm=1)])], imm=1)
    f.add(T.OP_OUT, [f.add(T.OP_MERGE, [f.add(T.OP_ID, [then]), f.add(T.OP_MUL, [other, rec])])])
    return [r.desc(), f.desc()], 0


def fib():
    """result(n) = fib(n); fib(n) = if n<2 then n else fib(n-1)+fib(n-2)."""
    r = _Fn("result", 1)
    r.add(T.OP_OUT, [r.add(T.OP_CALLFN, [r.add(T.OP_IN, imm=0)], imm=1)])
    f = _Fn("fib", 1)
    n = f.add(T.OP_IN, imm=0)
    sw = f.add(T.OP_SWITCH, [f.add(T.OP_LT, [n, f.add(T.OP_CONST, imm=2)]), n])
    then, other = (sw[0], 0), (sw[0], 1)
    a = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [other, f.add(T.OP_CONST, imm=1)])], imm=1)
    b = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [other, f.add(T.OP_CONST, imm=2)])], imm=1)
    f.add(T.OP_OUT, [f.add(T.OP_MERGE, [f.add(T.OP_ID, [then]), f.add(T.OP_ADD, [a, b])])])
    return [r.desc(), f.desc()], 0


def tree(cell="rnn", head=False):
    """f(v) = if isleaf(v) then embed(token(v)) else cell(f(left v), f(right v));
    result(v) = f(v), or result(v, label) = ce_head(f(v), label)."""
    r = _Fn("result", 2 if head else 1)
    y = r.add(T.OP_CALLFN, [r.add(T.OP_IN, imm=0)], imm=1)
    if head:
        y = r.add(T.OP_CE_HEAD, [y, r.add(T.OP_IN, imm=1)])
    r.add(T.OP_OUT, [y])
    f = _Fn("f", 1)
    v = f.add(T.OP_IN, imm=0)
    sw = f.add(T.OP_SWITCH, [f.add(T.OP_TREE_ISLEAF, [v]), v])
    leaf, inner = (sw[0], 0), (sw[0], 1)
    e = f.add(T.OP_EMBED, [f.add(T.OP_TREE_TOKEN, [leaf])])
    hl = f.add(T.OP_CALLFN, [f.add(T.OP_TREE_LEFT, [inner])], imm=1)
    hr = f.add(T.OP_CALLFN, [f.add(T.OP_TREE_RIGHT, [inner])], imm=1)
    h = f.add(T.OP_RNN_CELL if cell == "rnn" else T.OP_LSTM_CELL, [hl, hr])
    f.add(T.OP_OUT, [f.add(T.OP_MERGE, [e, h])])
    return [r.desc(), f.desc()], 0
