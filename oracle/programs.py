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


def tree_program(cell="rnn", head=False):
    """f(v) = if isleaf(v) then embed(token(v)) else cell(f(left v), f(right v)).
    result(v) = f(v), or with `head`: result(v,label) = ce_head(f(v), label)."""
    f = Function("f", [INT], VEC)
    v = f.param(0)
    leaf, inner = f.switch(f.op("isleaf", v), v)
    e = f.op("embed" if cell == "rnn" else "embed_lstm", f.op("token", leaf))
    hl = f.call("f", f.op("left", inner))
    hr = f.call("f", f.op("right", inner))
    h = f.op(cell + "_cell", hl, hr)
    f.output(f.merge(e, h))
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
