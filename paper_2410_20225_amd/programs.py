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


def tree(cell="rnn", head=False, node_loss=False):
    """f(v) = if isleaf(v) then embed(token(v)) else cell(f(left v), f(right v));
    result(v) = f(v), or result(v, label) = ce_head(f(v), label).  With node_loss every node
    has a loss term of its own: f(v) = ce_node(if ..., v)."""
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
    s = f.add(T.OP_MERGE, [e, h])
    f.add(T.OP_OUT, [f.add(T.OP_CE_NODE, [s, v]) if node_loss else s])
    return [r.desc(), f.desc()], 0


# ---- while-loops (tagged iteration, paper Section 2.3) -----------------------------------------
def _counting_loop(name, n_vars, step):
    """Loop graph: while 0 < v0: (v0, v1, ..) = step(g, v0, v1, ..); leaves with the last variable."""
    g = _Fn(name, n_vars)
    vs = [g.add(T.OP_IN, imm=k) for k in range(n_vars)]
    p = g.add(T.OP_LT, [g.add(T.OP_CONST, imm=0), vs[0]])
    sw = [g.add(T.OP_SWITCH, [p, v]) for v in vs]
    g.add(T.OP_NEXT, step(g, *[(s[0], 0) for s in sw]))
    g.add(T.OP_OUT, [(sw[-1][0], 1)])
    return g


def _sum_step(g, i, acc):
    return [g.add(T.OP_SUB, [i, g.add(T.OP_CONST, imm=1)]), g.add(T.OP_ADD, [acc, i])]


def sum_loop():
    """result(n) = { i = n; acc = 0; while 0 < i: acc = acc + i; i = i - 1 } acc."""
    r = _Fn("result", 1)
    r.add(T.OP_OUT, [r.add(T.OP_LOOP, [r.add(T.OP_IN, imm=0), r.add(T.OP_CONST, imm=0)], imm=1)])
    return [r.desc(), _counting_loop("S", 2, _sum_step).desc()], 0


def fib_loop():
    """result(n) = { i = n; b = 1; a = 0; while 0 < i: (i, b, a) = (i - 1, a + b, b) } a."""
    r = _Fn("result", 1)
    init = [r.add(T.OP_IN, imm=0), r.add(T.OP_CONST, imm=1), r.add(T.OP_CONST, imm=0)]
    r.add(T.OP_OUT, [r.add(T.OP_LOOP, init, imm=1)])
    f = _counting_loop("F", 3, lambda g, i, b, a: [g.add(T.OP_SUB, [i, g.add(T.OP_CONST, imm=1)]),
                                                   g.add(T.OP_ADD, [a, b]), g.add(T.OP_ID, [b])])
    return [r.desc(), f.desc()], 0


def gcd_loop():
    """result(a,b) = { while a != b: if a < b then b = b - a else a = a - b } a  (a, b >= 1)."""
    r = _Fn("result", 2)
    r.add(T.OP_OUT, [r.add(T.OP_LOOP, [r.add(T.OP_IN, imm=0), r.add(T.OP_IN, imm=1)], imm=1)])
    g = _Fn("G", 2)
    a, b = g.add(T.OP_IN, imm=0), g.add(T.OP_IN, imm=1)
    p = g.add(T.OP_EQ, [g.add(T.OP_EQ, [a, b]), g.add(T.OP_CONST, imm=0)])
    sa, sb = g.add(T.OP_SWITCH, [p, a]), g.add(T.OP_SWITCH, [p, b])
    a_t, a_f, b_t = (sa[0], 0), (sa[0], 1), (sb[0], 0)
    q = g.add(T.OP_LT, [a_t, b_t])
    qa, qb = g.add(T.OP_SWITCH, [q, a_t]), g.add(T.OP_SWITCH, [q, b_t])
    a_lt, a_ge, b_lt, b_ge = (qa[0], 0), (qa[0], 1), (qb[0], 0), (qb[0], 1)
    na = g.add(T.OP_MERGE, [g.add(T.OP_ID, [a_lt]), g.add(T.OP_SUB, [a_ge, b_ge])])
    nb = g.add(T.OP_MERGE, [g.add(T.OP_SUB, [b_lt, a_lt]), g.add(T.OP_ID, [b_ge])])
    g.add(T.OP_NEXT, [na, nb])
    g.add(T.OP_OUT, [a_f])
    return [r.desc(), g.desc()], 0


def nested_loop():
    """result(n) = { i = n; acc = 0; while 0 < i: acc = acc + { j = i; c = 0; while 0 < j:
    c = c + 1; j = j - 1 } c; i = i - 1 } acc."""
    r = _Fn("result", 1)
    r.add(T.OP_OUT, [r.add(T.OP_LOOP, [r.add(T.OP_IN, imm=0), r.add(T.OP_CONST, imm=0)], imm=1)])

    def outer_step(g, i, acc):
        c = g.add(T.OP_LOOP, [i, g.add(T.OP_SUB, [i, i])], imm=2)
        return [g.add(T.OP_SUB, [i, g.add(T.OP_CONST, imm=1)]), g.add(T.OP_ADD, [acc, c])]
    inner = _counting_loop("I", 2, lambda g, j, c: [g.add(T.OP_SUB, [j, g.add(T.OP_CONST, imm=1)]),
                                                    g.add(T.OP_ADD, [c, g.add(T.OP_CONST, imm=1)])])
    return [r.desc(), _counting_loop("O", 2, outer_step).desc(), inner.desc()], 0


def loop_of_calls():
    """result(n) = { i = n; acc = 0; while 0 < i: acc = acc + fib(i); i = i - 1 } acc."""
    r = _Fn("result", 1)
    r.add(T.OP_OUT, [r.add(T.OP_LOOP, [r.add(T.OP_IN, imm=0), r.add(T.OP_CONST, imm=0)], imm=1)])
    s = _counting_loop("L", 2, lambda g, i, acc: [g.add(T.OP_SUB, [i, g.add(T.OP_CONST, imm=1)]),
                                                  g.add(T.OP_ADD, [acc, g.add(T.OP_CALLFN, [i], imm=2)])])
    fns, _ = fib()
    name, n_params, nodes = fns[1]
    nodes = [(op, ins, 2 if op == T.OP_CALLFN else imm) for op, ins, imm in nodes]   # fib is function 2 here
    return [r.desc(), s.desc(), (name, n_params, nodes)], 0


def loop_in_function():
    """result(n) = tet(n); tet(n) = if n < 1 then n - n else { the sum loop over n } + tet(n - 1)."""
    r = _Fn("result", 1)
    r.add(T.OP_OUT, [r.add(T.OP_CALLFN, [r.add(T.OP_IN, imm=0)], imm=1)])
    f = _Fn("tet", 1)
    n = f.add(T.OP_IN, imm=0)
    sw = f.add(T.OP_SWITCH, [f.add(T.OP_LT, [n, f.add(T.OP_CONST, imm=1)]), n])
    t, e = (sw[0], 0), (sw[0], 1)
    tri = f.add(T.OP_LOOP, [e, f.add(T.OP_SUB, [e, e])], imm=2)
    rec = f.add(T.OP_CALLFN, [f.add(T.OP_SUB, [e, f.add(T.OP_CONST, imm=1)])], imm=1)
    f.add(T.OP_OUT, [f.add(T.OP_MERGE, [f.add(T.OP_SUB, [t, t]), f.add(T.OP_ADD, [tri, rec])])])
    return [r.desc(), f.desc(), _counting_loop("S", 2, _sum_step).desc()], 0
