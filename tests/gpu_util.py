"""Helpers for the GPU parity tests: upload a workload, call the library through its binding,
and run the oracle on the same inputs.  Nothing here computes expected values."""
import numpy as np
import torch

from paper_2410_20225_amd import tdf
from paper_2410_20225_amd.harness import TreeRun, DEV  # noqa: F401  (re-exported for the tests)
import oracle
from oracle import programs as oracle_programs



def rel_fro(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def assert_close_bf16(got, want, name, tol=2e-2):
    """The 16-bit path's bar for one tensor: relative Frobenius error within tol, and no single element
    further off than tol times the largest element of the oracle's tensor."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, name
    assert rel_fro(got, want) < tol, (name, rel_fro(got, want))
    worst = float(np.abs(got - want).max()) if want.size else 0.0
    assert worst <= tol * float(np.abs(want).max()), (name, worst, float(np.abs(want).max()))


def assert_rows_close_bf16(got, want, name, tol=2e-2, floor=0.05):
    """Row by row (a token's row of dE, a tree's root state): the row's error within tol of the row's own
    norm; rows whose norm is below `floor` times the largest row norm are held to tol times that instead
    (their entries are sums with cancellation, which has no relative bound)."""
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, name
    rn = np.linalg.norm(want, axis=1)
    err = np.linalg.norm(got - want, axis=1)
    bar = tol * np.maximum(rn, floor * rn.max())
    bad = np.nonzero(err > bar)[0]
    assert bad.size == 0, (name, bad[:8].tolist(), err[bad[:8]].tolist(), rn[bad[:8]].tolist())


def oracle_env(c):
    F = c["forest"]
    return dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"], U=c["U"], u0=c["u0"])


def run_oracle_tree(c, head, grad, dy=None, round_bf16=False):
    """Returns dict with out (list per instance), grads, interpreter.  round_bf16: the oracle's
    diagnostic variant with the roundings of a 16-bit state path (oracle/ops_bf16.py)."""
    F = c["forest"]
    B = F.n_trees
    prog = oracle_programs.tree_program(c["cell"], head=head)
    if grad:
        prog = oracle.differentiate(prog)
    env = oracle_env(c)
    env["round_bf16"] = round_bf16
    it = oracle.Interpreter(oracle.transform(prog), env)
    inputs = {("in", 0): F.roots.tolist()}
    if head:
        inputs[("in", 1)] = c["labels"].tolist()
    if grad:
        inputs[("gin", 0)] = list(dy)
    out = it.run(inputs, B)
    return dict(out=out[("out", 0)], grads=it.param_grad, it=it)


def run_oracle_node_loss(c, node_labels, dnode=None, dy=None, ids=None):
    """Per-node losses (and gradients when dnode is given) of the trees `ids` (default: all)."""
    F = c["forest"]
    roots = F.roots.tolist() if ids is None else [int(F.roots[b]) for b in ids]
    prog = oracle_programs.tree_program(c["cell"], node_loss=True)
    env = oracle_env(c)
    env["node_label"] = node_labels
    inputs = {("in", 0): roots}
    if dnode is not None:
        prog = oracle.differentiate(prog)
        env["dnode"] = dnode
        D = c["H"] * (2 if c["cell"] == "lstm" else 1)
        inputs[("gin", 0)] = list(np.zeros((len(roots), D)) if dy is None else dy)
    it = oracle.Interpreter(oracle.transform(prog), env)
    out = it.run(inputs, len(roots))
    return dict(out=out[("out", 0)], node_loss=it.node_loss, grads=it.param_grad, it=it)


def fire_counts(graph, stats):
    """{name: live firings} with the oracle's naming of static-graph nodes."""
    names = {tdf.OP_IN: "in", tdf.OP_OUT: "out", tdf.OP_ADD: "add", tdf.OP_SUB: "sub", tdf.OP_MUL: "mul",
             tdf.OP_EQ: "eq", tdf.OP_LT: "lt", tdf.OP_ID: "id", tdf.OP_SWITCH: "switch", tdf.OP_MERGE: "merge",
             tdf.SNODE_MERGE_ENTRY: "merge_entry", tdf.OP_TREE_ISLEAF: "isleaf", tdf.OP_TREE_LEFT: "left",
             tdf.OP_TREE_RIGHT: "right", tdf.OP_TREE_TOKEN: "token", tdf.OP_EMBED: "embed",
             tdf.OP_RNN_CELL: "rnn_cell", tdf.OP_LSTM_CELL: "lstm_cell", tdf.OP_CE_HEAD: "ce_head",
             tdf.OP_CE_NODE: "ce_node"}
    out = {}
    for i, n in enumerate(tdf.graph_info(graph)["nodes"]):
        if n["is_grad"] or n["kind"] == tdf.OP_CONST:
            continue
        if n["kind"] == tdf.SNODE_CALL:
            name = "call_%d" % n["label"]
        elif n["kind"] == tdf.SNODE_RETURN:
            name = "return_%d" % n["label"]
        elif n["kind"] == tdf.SNODE_ENTER:
            name = "enter_%d" % n["label"]
        elif n["kind"] == tdf.SNODE_EXIT:
            name = "exit_%d" % n["label"]
        elif n["kind"] == tdf.SNODE_NEXT:
            name = "next"
        else:
            name = names[n["kind"]]
        out[name] = out.get(name, 0) + stats.fire_count[i]
    return out
