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


def ack():
    """result(m,n) = ack(m,n); ack(m,n) = n+1 if m==0; ack(m-1,1) if n==0; else ack(m-1, ack(m,n-1))."""
    r = _Fn("result", 2)
    r.add(T.OP_OUT, [r.add(T.OP_CALLFN, [r.add(T.OP_IN, imm=0), r.add(T.OP_IN, imm=1)], imm=1)])
    f = _Fn("ack", 2)
    m, n = f.add(T.OP_IN, imm=0), f.add(T.OP_IN, imm=1)
    one, zero = f.add(T.OP_CONST, imm=1), f.add(T.OP_CONST, imm=0)
    p0 = f.add(T.OP_EQ, [m, zero])
    sm, sn = f.add(T.OP_SWITCH, [p0, m]), f.add(T.OP_SWITCH, [p0, n])
    m_e, n_t, n_e = (sm[0], 1), (sn[0], 0), (sn[0], 1)
    r0 = f.add(T.OP_ADD, [n_t, one])
    p1 = f.add(T.OP_EQ, [n_e, zero])
    sm1, sn1 = f.add(T.OP_SWITCH, [p1, m_e]), f.add(T.OP_SWITCH, [p1, n_e])
    m_et, m_ee, n_et, n_ee = (sm1[0], 0), (sm1[0], 1), (sn1[0], 0), (sn1[0], 1)
    r1 = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [m_et, one]), f.add(T.OP_ADD, [n_et, one])], imm=1)
    inner = f.add(T.OP_CALLFN, [m_ee, f.add(T.OP_SUB, [n_ee, one])], imm=1)
    r2 = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [m_ee, one]), inner], imm=1)
    f.add(T.OP_OUT, [f.add(T.OP_MERGE, [r0, f.add(T.OP_MERGE, [r1, r2])])])
    return [r.desc(), f.desc()], 0


def tak():
    """result(x,y,z) = tak(x,y,z); tak(x,y,z) = if y<x then tak(tak(x-1,y,z), tak(y-1,z,x), tak(z-1,x,y)) else z."""
    r = _Fn("result", 3)
    r.add(T.OP_OUT, [r.add(T.OP_CALLFN, [r.add(T.OP_IN, imm=k) for k in range(3)], imm=1)])
    f = _Fn("tak", 3)
    x, y, z = (f.add(T.OP_IN, imm=k) for k in range(3))
    one = f.add(T.OP_CONST, imm=1)
    p = f.add(T.OP_LT, [y, x])
    sx, sy, sz = (f.add(T.OP_SWITCH, [p, v]) for v in (x, y, z))
    x_t, y_t, z_t, z_e = (sx[0], 0), (sy[0], 0), (sz[0], 0), (sz[0], 1)
    a = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [x_t, one]), y_t, z_t], imm=1)
    b = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [y_t, one]), z_t, x_t], imm=1)
    c = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [z_t, one]), x_t, y_t], imm=1)
    top = f.add(T.OP_CALLFN, [a, b, c], imm=1)
    f.add(T.OP_OUT, [f.add(T.OP_MERGE, [top, f.add(T.OP_ID, [z_e])])])
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
