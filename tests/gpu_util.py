"""Helpers for the GPU parity tests: upload a workload, call the library through its binding,
and run the oracle on the same inputs.  Nothing here computes expected values."""
import numpy as np
import torch

from paper_2410_20225_amd import tdf, programs as gpu_programs
import oracle
from oracle import programs as oracle_programs

DEV = "cuda:0"


def rel_fro(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


def oracle_env(c):
    F = c["forest"]
    return dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"], U=c["U"], u0=c["u0"])


def run_oracle_tree(c, head, grad, dy=None):
    """Returns dict with out (list per instance), grads, interpreter."""
    F = c["forest"]
    B = F.n_trees
    prog = oracle_programs.tree_program(c["cell"], head=head)
    if grad:
        prog = oracle.differentiate(prog)
    it = oracle.Interpreter(oracle.transform(prog), oracle_env(c))
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


class TreeRun:
    """One workload resident on the GPU plus the buffers of one evaluation."""

    def __init__(self, c, head, grad, max_tags=None, step_limit=0, stats_level=1, node_labels=None):
        F = c["forest"]
        self.c, self.head, self.grad = c, head, grad
        self.B, self.H = F.n_trees, c["H"]
        dt = torch.bfloat16 if c["bf16"] else torch.float32
        self.rows = (5 if c["cell"] == "lstm" else 1) * self.H
        fns, r = gpu_programs.tree(c["cell"], head=head, node_loss=node_labels is not None)
        self.graph = tdf.graph_build(fns, r, want_grad=grad)
        args = np.stack([F.roots, c["labels"]], 1) if head else F.roots[:, None]
        t = lambda a, d: torch.tensor(np.ascontiguousarray(a), dtype=d, device=DEV)
        self.t_args = t(args, torch.int64)
        self.t_left, self.t_right, self.t_token = (t(a, torch.int32) for a in (F.left, F.right, F.token))
        self.t_E, self.t_W = t(c["E"], dt), t(c["W"], dt)
        self.t_b, self.t_U, self.t_u0 = t(c["b"], torch.float32), t(c["U"], torch.float32), t(c["u0"], torch.float32)
        self.max_tags = F.n_nodes if max_tags is None else max_tags
        self.t_node_label = self.out_node_loss = self.t_dnode = self._dnode_src = self.t_dy = self._dy_src = None
        if node_labels is not None:
            self.t_node_label = t(node_labels, torch.int32)
            self.out_node_loss = torch.full((F.n_nodes,), -7.0, dtype=torch.float32, device=DEV)
        self.inputs = tdf.make_inputs(self.B, args=self.t_args, n_args=args.shape[1], left=self.t_left,
                                      right=self.t_right, token=self.t_token,
                                      dtype=tdf.BF16 if c["bf16"] else tdf.F32, hidden=self.H, vocab=c["V"],
                                      E=self.t_E, W=self.t_W, b=self.t_b, U=self.t_U, u0=self.t_u0,
                                      n_classes=5, max_tags=self.max_tags, step_limit=step_limit, stats_level=stats_level,
                                      node_label=self.t_node_label)
        nbytes = tdf.workspace_size(self.graph, self.inputs, grad)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
        self.out_f32 = torch.zeros(self.B, dtype=torch.float32, device=DEV)
        self.out_h = torch.zeros(self.B, self.H, dtype=torch.float32, device=DEV)
        self.out_c = torch.zeros(self.B, self.H, dtype=torch.float32, device=DEV)
        if grad:
            self.dW = torch.empty(self.rows, 2 * self.H, dtype=torch.float32, device=DEV)
            self.db = torch.empty(self.rows, dtype=torch.float32, device=DEV)
            self.dE = torch.empty(c["V"], self.H, dtype=torch.float32, device=DEV)

    def run(self, dy=None, check=True, dnode=None):
        if self.grad:
            f32 = lambda a: None if a is None else torch.tensor(np.ascontiguousarray(a), dtype=torch.float32, device=DEV)
            if dy is not self._dy_src:         # both stay resident while the caller passes the same arrays
                self._dy_src, self.t_dy = dy, f32(dy)
            if dnode is not self._dnode_src:   # stays resident while the caller passes the same array
                self._dnode_src, self.t_dnode = dnode, f32(dnode)
            st, stats = tdf.eval_grad(self.graph, self.inputs, self.t_dy, self.ws, self.dW, self.db, self.dE,
                                      out_f32=self.out_f32, out_h=self.out_h, out_c=self.out_c,
                                      out_node_loss=self.out_node_loss, dnode=self.t_dnode, check=check)
        else:
            st, stats = tdf.eval(self.graph, self.inputs, self.ws, out_f32=self.out_f32, out_h=self.out_h,
                                 out_c=self.out_c, out_node_loss=self.out_node_loss, check=check)
        torch.cuda.synchronize()
        return st, stats


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
