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
