"""ORACLE — test infrastructure only, never on the product path.

The programs of the workloads, written as sets of function graphs (paper Section 2.4).
Conditionals are Switch/Merge pairs exactly as in the paper's factorial example: the
predicate steers the parameter through a Switch and the two branch results meet in a Merge.
"""
from .graph import Function, Program, INT, FLOAT, VEC


def fact_program():
    """result = fact(3)+5 ; fact(n) = if n==1 then n else n*fact(n-1)   (Section 2.4)."""
    f = Function("fact", [INT], INT)
    n = f.param(0)
    t, e = f.switch(f.op("eq", f.const(1), n), n)
    rec = f.call("fact", f.op("sub", e, f.const(1)))
    f.output(f.merge(f.op("id", t), f.op("mul", e, rec)))
    r = Function("result", [], INT)
    r.output(r.op("add", r.const(5), r.call("fact", r.const(3))))
    return Program([r, f])


def fib_program():
    """result(n) = fib(n) ; fib(n) = if n<2 then n else fib(n-1)+fib(n-2)."""
    f = Function("fib", [INT], INT)
    n = f.param(0)
    t, e = f.switch(f.op("lt", n, f.const(2)), n)
    a = f.call("fib", f.op("sub", e, f.const(1)))
    b = f.call("fib", f.op("sub", e, f.const(2)))
    f.output(f.merge(f.op("id", t), f.op("add", a, b)))
    r = Function("result", [INT], INT)
    r.output(r.call("fib", r.param(0)))
    return Program([r, f])


def power_program():
    """result(x,n) = pw(x,n) ; pw(x,n) = if n==0 then 1.0 else x*pw(x,n-1): a float-valued
    recursion whose gradient has the closed form n*x^(n-1)."""
    f = Function("pw", [FLOAT, INT], FLOAT)
    x, n = f.param(0), f.param(1)
    p = f.op("eq", n, f.const(0))
    one, _ = f.switch(p, f.const(1.0))
    _, xe = f.switch(p, x)
    _, ne = f.switch(p, n)
    rec = f.call("pw", xe, f.op("sub", ne, f.const(1)))
    f.output(f.merge(one, f.op("mul", xe, rec)))
    r = Function("result", [FLOAT, INT], FLOAT)
    r.output(r.call("pw", r.param(0), r.param(1)))
    return Program([r, f])


def ack_program():
    """result(m,n) = ack(m,n) ; ack(m,n) = n+1 if m==0 ; ack(m-1,1) if n==0 ; else
    ack(m-1, ack(m,n-1)): two parameters per call (two Call_i nodes insert one tag) and a call
    whose argument is another call's result (Section 3, Section 6.1)."""
    f = Function("ack", [INT, INT], INT)
    m, n = f.param(0), f.param(1)
    p0 = f.op("eq", m, f.const(0))
    _, m_e = f.switch(p0, m)
    n_t, n_e = f.switch(p0, n)
    r0 = f.op("add", n_t, f.const(1))
    p1 = f.op("eq", n_e, f.const(0))
    m_et, m_ee = f.switch(p1, m_e)
    n_et, n_ee = f.switch(p1, n_e)
    r1 = f.call("ack", f.op("sub", m_et, f.const(1)), f.op("add", n_et, f.const(1)))
    inner = f.call("ack", m_ee, f.op("sub", n_ee, f.const(1)))
    r2 = f.call("ack", f.op("sub", m_ee, f.const(1)), inner)
    f.output(f.merge(r0, f.merge(r1, r2)))
    r = Function("result", [INT, INT], INT)
    r.output(r.call("ack", r.param(0), r.param(1)))
    return Program([r, f])


def tak_program():
    """result(x,y,z) = tak(x,y,z) ; tak(x,y,z) = if y<x then
    tak(tak(x-1,y,z), tak(y-1,z,x), tak(z-1,x,y)) else z: three parameters per call, three
    calls nested as arguments (Section 6.1)."""
    f = Function("tak", [INT, INT, INT], INT)
    x, y, z = f.param(0), f.param(1), f.param(2)
    p = f.op("lt", y, x)
    x_t, _ = f.switch(p, x)
    y_t, _ = f.switch(p, y)
    z_t, z_e = f.switch(p, z)
    a = f.call("tak", f.op("sub", x_t, f.const(1)), y_t, z_t)
    b = f.call("tak", f.op("sub", y_t, f.const(1)), z_t, x_t)
    c = f.call("tak", f.op("sub", z_t, f.const(1)), x_t, y_t)
    f.output(f.merge(f.call("tak", a, b, c), f.op("id", z_e)))
    r = Function("result", [INT, INT, INT], INT)
    r.output(r.call("tak", r.param(0), r.param(1), r.param(2)))
    return Program([r, f])


def tree_program(cell="rnn", head=False, node_loss=False):
    """f(v) = if isleaf(v) then embed(token(v)) else cell(f(left v), f(right v)).
    result(v) = f(v), or with `head`: result(v,label) = ce_head(f(v), label).
    With `node_loss` every node of a tree contributes a loss term (fully labelled trees,
    Section 6): f(v) = ce_node(if ... , v)."""
    f = Function("f", [INT], VEC)
    v = f.param(0)
    leaf, inner = f.switch(f.op("isleaf", v), v)
    e = f.op("embed" if cell == "rnn" else "embed_lstm", f.op("token", leaf))
    hl = f.call("f", f.op("left", inner))
    hr = f.call("f", f.op("right", inner))
    h = f.op(cell + "_cell", hl, hr)
    s = f.merge(e, h)
    f.output(f.op("ce_node", s, v) if node_loss else s)
    if head:
        r = Function("result", [INT, INT], FLOAT)
        y = r.call("f", r.param(0))
        if cell == "lstm":
            y = r.op("take_h", y)
        r.output(r.op("ce_head", y, r.param(1)))
    else:
        r = Function("result", [INT], VEC)
        r.output(r.call("f", r.param(0)))
    return Program([r, f])


# ---- tagged iteration (Section 2.3) -----------------------------------------------------------
# A while-loop is a loop graph: its parameters are the loop variables, the Switch on the loop
# condition sends them into the body (true side) or out of the loop (false side), `next` takes
# the body's results, the output hangs on the false side.
def _counting_loop(name, n_vars, step):
    """while 0 < v0: (v0, v1, ..) = step(g, v0_true, v1_true, ..); leaves with the last
    variable.  Returns the loop graph."""
    g = Function(name, [INT] * n_vars, INT)
    p = g.op("lt", g.const(0), g.param(0))
    sides = [g.switch(p, g.param(k)) for k in range(n_vars)]
    g.next(*step(g, *[t for t, _ in sides]))
    g.output(sides[-1][1])
    return g


def sum_loop_program():
    """result(n) = { i = n; acc = 0; while 0 < i: acc = acc + i; i = i - 1 } acc."""
    s = _counting_loop("S", 2, lambda g, i, acc: (g.op("sub", i, g.const(1)), g.op("add", acc, i)))
    r = Function("result", [INT], INT)
    r.output(r.loop("S", r.param(0), r.const(0)))
    return Program([r, s])


def fib_loop_program():
    """result(n) = { i = n; b = 1; a = 0; while 0 < i: (i, b, a) = (i - 1, a + b, b) } a."""
    f = _counting_loop("F", 3, lambda g, i, b, a: (g.op("sub", i, g.const(1)), g.op("add", a, b), g.op("id", b)))
    r = Function("result", [INT], INT)
    r.output(r.loop("F", r.param(0), r.const(1), r.const(0)))
    return Program([r, f])


def gcd_loop_program():
    """result(a,b) = { while a != b: if a < b then b = b - a else a = a - b } a  (a, b >= 1):
    a conditional inside the loop body, and a trip count that depends on the data."""
    g = Function("G", [INT, INT], INT)
    a, b = g.param(0), g.param(1)
    p = g.op("eq", g.op("eq", a, b), g.const(0))
    a_t, a_f = g.switch(p, a)
    b_t, _ = g.switch(p, b)
    q = g.op("lt", a_t, b_t)
    a_lt, a_ge = g.switch(q, a_t)
    b_lt, b_ge = g.switch(q, b_t)
    g.next(g.merge(g.op("id", a_lt), g.op("sub", a_ge, b_ge)),
           g.merge(g.op("sub", b_lt, a_lt), g.op("id", b_ge)))
    g.output(a_f)
    r = Function("result", [INT, INT], INT)
    r.output(r.loop("G", r.param(0), r.param(1)))
    return Program([r, g])


def nested_loop_program():
    """result(n) = { i = n; acc = 0; while 0 < i: acc = acc + { j = i; c = 0; while 0 < j:
    c = c + 1; j = j - 1 } c; i = i - 1 } acc: a loop in a loop body, tags two counters long."""
    inner = _counting_loop("I", 2, lambda g, j, c: (g.op("sub", j, g.const(1)), g.op("add", c, g.const(1))))

    def outer_step(g, i, acc):
        c = g.loop("I", i, g.op("sub", i, i))
        return g.op("sub", i, g.const(1)), g.op("add", acc, c)
    outer = _counting_loop("O", 2, outer_step)
    r = Function("result", [INT], INT)
    r.output(r.loop("O", r.param(0), r.const(0)))
    return Program([r, outer, inner])


def loop_of_calls_program():
    """result(n) = { i = n; acc = 0; while 0 < i: acc = acc + fib(i); i = i - 1 } acc: calls
    from inside a loop body, call labels pushed on top of an iteration counter."""
    fib = fib_program().functions["fib"]
    s = _counting_loop("L", 2, lambda g, i, acc: (g.op("sub", i, g.const(1)), g.op("add", acc, g.call("fib", i))))
    r = Function("result", [INT], INT)
    r.output(r.loop("L", r.param(0), r.const(0)))
    return Program([r, s, fib])


def loop_in_function_program():
    """result(n) = tet(n) ; tet(n) = if n < 1 then n - n else { the sum loop over n } +
    tet(n - 1): a loop in the body of a recursive function, iteration counters pushed on top
    of call labels; in the base case the loop's initial values are dead."""
    s = _counting_loop("S", 2, lambda g, i, acc: (g.op("sub", i, g.const(1)), g.op("add", acc, i)))
    f = Function("tet", [INT], INT)
    n = f.param(0)
    t, e = f.switch(f.op("lt", n, f.const(1)), n)
    tri = f.loop("S", e, f.op("sub", e, e))
    rec = f.call("tet", f.op("sub", e, f.const(1)))
    f.output(f.merge(f.op("sub", t, t), f.op("add", tri, rec)))
    r = Function("result", [INT], INT)
    r.output(r.call("tet", r.param(0)))
    return Program([r, f, s])


def sum_recursive_program():
    """result(n) = s(n, 0) ; s(i, acc) = if 0 < i then s(i - 1, acc + i) else acc: the sum loop
    written as a tail recursion, for comparison (same values, tags as long as the trip count)."""
    f = Function("s", [INT, INT], INT)
    i, acc = f.param(0), f.param(1)
    p = f.op("lt", f.const(0), i)
    i_t, _ = f.switch(p, i)
    a_t, a_f = f.switch(p, acc)
    f.output(f.merge(f.call("s", f.op("sub", i_t, f.const(1)), f.op("add", a_t, i_t)), f.op("id", a_f)))
    r = Function("result", [INT], INT)
    r.output(r.call("s", r.param(0), r.op("sub", r.param(0), r.param(0))))
    return Program([r, f])
