"""A workload resident on the GPU together with the buffers of one evaluation: uploads the forest
and the parameters once, builds the graph, sizes the workspace and calls tdf_eval / tdf_eval_grad.
Used by the benchmark and by the GPU tests; argument marshalling only."""
import numpy as np
import torch

from . import tdf, programs as gpu_programs

DEV = "cuda:0"


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
        torch.cuda.current_stream().synchronize()   # (the call has done so already; other streams may be busy with another evaluation)
        return st, stats
