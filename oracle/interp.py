"""ORACLE — test infrastructure only, never on the product path.

A plain interpreter of the tagged dataflow model (paper Sections 2.1-2.2 and 3).

Edges carry tokens <tag, data>.  A tag is a tuple whose first element is the most recent
call label (the paper's list i:t); the last element is the instance index, so instance b
of a batch runs under root tag (b,) and its first call under (0, b).  Data is an int, a
float, a float64 array, or DEAD (the hiaton, written * in the paper).

  ordinary node   fires when every input holds a token with the same tag; the output
                  keeps the tag; a DEAD input makes every output DEAD
  Switch          (<t,true>,<t,d>) -> (<t,d>,<t,*>); false mirrored
  Merge           forwards the live input; fires on the first live arrival for a tag
                  (the inputs of an entry Merge come from different Call nodes and never
                  share a tag); emits * only when every input delivered *
  Call_i          <t,d> -> <i:t,d> into the callee, plus a control token <i:t> to
                  Return_i; a DEAD input sends nothing into the callee and a DEAD control
                  token to Return_i
  Return_i        <i:t,d> -> <t,d> once its control tokens for i:t are there; data whose
                  head label is not i is dropped; DEAD control -> <t,*>
  Enter           <t,d> -> <0:t,d> into the loop (Section 2.3), plus a control token <t> to
                  the loop's Exit; a DEAD input sends nothing into the loop and a DEAD control
                  token to the Exit
  Next            <n:t,d> -> <(n+1):t,d>; a DEAD input ends there (the iteration after the
                  last one does not exist)
  Exit            <n:t,d> -> <t,d> once the control tokens for t are there; DEAD data ends
                  there (every iteration but the last sends one); DEAD control -> <t,*>
  constants       hold for all tags: they are immediates of the consuming node

A tag is one list for call labels and iteration counters alike (Section 5.1: loop scopes and
function scopes share one stack); which of the two an element is follows from the node that
handles the token, as in the paper.

Execution is in synchronous rounds: every (node, tag) that became ready in round r fires
in round r+1.  The paper's executor is asynchronous; results and counts do not depend on
the order because each (node, tag) fires at most once.

Parameter gradients (dW, db, dE, ...) are the sums over all tags of the per-tag terms,
accumulated in float64 in firing order (the paper leaves the cross-tag sum implicit:
parameters are input nodes visible under every tag).
"""
import numpy as np
from . import ops, ops_bf16
from .graph import TWO_PORT_OPS


class _Dead:
    def __repr__(self):
        return "*"


DEAD = _Dead()


def _truth(v):
    return bool(v)


class Interpreter:
    def __init__(self, sgraph, env=None):
        self.g = sgraph
        self.env = dict(env or {})
        nodes = sgraph.nodes
        self.const_fill = []
        self.n_wait = []
        for nd in nodes:
            fill = [(s, nodes[src].attr["value"]) for s, (src, _) in enumerate(nd.ins)
                    if nodes[src].op == "const"]
            self.const_fill.append(fill)
            self.n_wait.append(len(nd.ins) - len(fill) + len(nd.ctl))
        # the value every Return of a function hangs on, and its gradient entry
        self.body_out = set()
        for nd in nodes:
            if nd.op == "return" and nd.attr["kind"] == "out":
                self.body_out.add(nd.ins[0][0])
        self.reset()

    # ------------------------------------------------------------------------------
    def reset(self):
        self.slots = {}
        self.ready = []
        self.fire_count = [0] * len(self.g.nodes)
        self.tags = set()              # call-context tags created (entry Merge firings)
        self.iter_tags = set()         # (loop graph, tag) of every iteration entered
        self._entered_iters = set()    # the same tags without the graph
        self.fwd_body = {}             # tag -> live firings of the function's result value
        self.bwd_body = {}             # tag -> live firings of the gradient entry
        self.dropped = 0               # Return_i label mismatches
        self.rounds = 0
        self.peak_live_tags = 0        # most tags alive in one round (only with track_live)
        self.max_tag_len = 0
        self.outputs = {}
        self.param_grad = {}
        self.node_loss = {}            # tree node -> loss term of the ce_node firing there
        self._outer = {}               # name -> ([delta rows], [x rows]) awaiting a flush

    # ------------------------------------------------------------------------------
    def _slot(self, j, tag):
        key = (j, tag)
        rec = self.slots.get(key)
        if rec is None:
            nd = self.g.nodes[j]
            vals = [None] * len(nd.ins)
            for s, v in self.const_fill[j]:
                vals[s] = v
            rec = [vals, [None] * len(nd.ctl), self.n_wait[j], False]   # vals, ctl, waiting, fired
            self.slots[key] = rec
        return rec

    def _schedule(self, j, tag, rec):
        if not rec[3]:
            rec[3] = True
            self.ready.append((j, tag))

    def _deliver(self, j, slot, tag, value, control=False):
        nd = self.g.nodes[j]
        if nd.op == "return" and not control and tag[0] != nd.attr["label"]:
            self.dropped += 1                       # wrong frame label: no output
            return
        if nd.op == "exit":
            if not control:
                if value is DEAD:                   # an iteration that goes on: nothing leaves
                    return
                tag = tag[1:]                       # pop the iteration counter
            rec = self._slot(j, tag)
            (rec[1] if control else rec[0])[slot] = value
            ctl = rec[1]
            if all(c is not None for c in ctl):
                if any(c is DEAD for c in ctl) or rec[0][0] is not None:
                    self._schedule(j, tag, rec)
            return
        rec = self._slot(j, tag)
        if rec[3] and nd.op in ("merge", "merge_entry"):
            return
        (rec[1] if control else rec[0])[slot] = value
        rec[2] -= 1
        op = nd.op
        if op in ("merge", "merge_entry"):
            if value is not DEAD or rec[2] == 0:
                self._schedule(j, tag, rec)
        elif op == "return":
            ctl = rec[1]
            if all(c is not None for c in ctl):
                if any(c is DEAD for c in ctl) or rec[0][0] is not None:
                    self._schedule(j, tag, rec)
        elif rec[2] == 0:
            self._schedule(j, tag, rec)

    def _emit(self, j, port, tag, value):
        for p, dst, dslot in self.g.nodes[j].outs:
            if p == port:
                self._deliver(dst, dslot, tag, value)

    # ------------------------------------------------------------------------------
    def _fire(self, j, tag):
        nd = self.g.nodes[j]
        op = nd.op
        if op in ("merge", "merge_entry"):      # the record stays: later arrivals are ignored
            vals, ctl = self.slots[(j, tag)][0:2]
        else:
            vals, ctl = self.slots.pop((j, tag))[0:2]
        if op in ("merge", "merge_entry"):
            live = [v for v in vals if v is not None and v is not DEAD]
            out = live[0] if live else DEAD
            if out is not DEAD:
                self.fire_count[j] += 1
                if op == "merge_entry" and nd.attr["kind"] == "loop":
                    self.iter_tags.add((nd.fn, tag))
                    self._entered_iters.add(tag)
                    self.max_tag_len = max(self.max_tag_len, len(tag) - 1)
                elif op == "merge_entry":
                    self.tags.add(tag)
                    self.max_tag_len = max(self.max_tag_len, len(tag) - 1)
                    if nd.attr["kind"] == "gin":
                        self.bwd_body[tag] = self.bwd_body.get(tag, 0) + 1
            self._after(j, tag, out)
            self._emit(j, 0, tag, out)
            return
        if op == "call":
            v = vals[0]
            new = (nd.attr["label"],) + tag
            if v is not DEAD:
                self.fire_count[j] += 1
                self._emit(j, 0, new, v)
            for dst, cslot in nd.ctl_outs:
                self._deliver(dst, cslot, new, DEAD if v is DEAD else True, control=True)
            return
        if op == "return":
            dead = any(c is DEAD for c in ctl)
            out = DEAD if dead else vals[0]
            if not dead:
                self.fire_count[j] += 1
            self._emit(j, 0, tag[1:], out)
            return
        if op == "enter":
            v = vals[0]
            if v is not DEAD:
                self.fire_count[j] += 1
                self._emit(j, 0, (0,) + tag, v)
            for dst, cslot in nd.ctl_outs:
                self._deliver(dst, cslot, tag, DEAD if v is DEAD else True, control=True)
            return
        if op == "next":
            v = vals[0]
            if v is not DEAD:
                self.fire_count[j] += 1
                self._emit(j, 0, (tag[0] + 1,) + tag[1:], v)
            return
        if op == "exit":                            # `tag` is the enclosing scope's already
            dead = any(c is DEAD for c in ctl)
            if not dead:
                self.fire_count[j] += 1
            self._emit(j, 0, tag, DEAD if dead else vals[0])
            return
        if op == "addn":
            live = [v for v in vals if v is not DEAD]
            out = DEAD
            if live:
                out = live[0]
                for v in live[1:]:
                    out = out + v
                self.fire_count[j] += 1
            self._emit(j, 0, tag, out)
            return
        if any(v is DEAD for v in vals):
            for port in range(2 if op in TWO_PORT_OPS else 1):
                self._emit(j, port, tag, DEAD)
            return
        self.fire_count[j] += 1
        if op == "switch":
            t = _truth(vals[0])
            self._emit(j, 0, tag, vals[1] if t else DEAD)
            self._emit(j, 1, tag, DEAD if t else vals[1])
            return
        if op in ("out", "gout"):
            self.outputs.setdefault((op, nd.attr.get("k", 0)), {})[tag] = vals[0]
            return
        out = self._compute(nd, vals, tag)
        self._after(j, tag, out)
        if out is not None:
            self._emit(j, 0, tag, out[0] if isinstance(out, tuple) else out)
            if isinstance(out, tuple):
                for port in range(1, len(out)):
                    self._emit(j, port, tag, out[port])

    def _after(self, j, tag, out):
        if j in self.body_out and out is not DEAD:
            self.fwd_body[tag] = self.fwd_body.get(tag, 0) + 1

    # ------------------------------------------------------------------------------
    def _compute(self, nd, v, tag):
        op, env = nd.op, self.env
        if op == "add":
            return v[0] + v[1]
        if op == "sub":
            return v[0] - v[1]
        if op == "mul":
            return v[0] * v[1]
        if op == "neg":
            return -v[0]
        if op == "eq":
            return int(v[0] == v[1])
        if op == "lt":
            return int(v[0] < v[1])
        if op == "id":
            return v[0]
        if op == "snd":
            return v[1]
        if op == "tanh":
            return np.tanh(v[0])
        if op == "tanh_grad":                       # (x, dy) -> dx
            return v[1] * (1.0 - np.tanh(v[0]) ** 2)
        if op == "isleaf":
            return int(env["left"][v[0]] < 0)
        if op == "left":
            return int(env["left"][v[0]])
        if op == "right":
            return int(env["right"][v[0]])
        if op == "token":
            return int(env["token"][v[0]])
        if op == "embed":
            return env["E"][v[0]].astype(np.float64)
        if op == "embed_lstm":
            return ops.lstm_leaf(env["E"][v[0]].astype(np.float64))
        cells = ops_bf16 if env.get("round_bf16") else ops   # diagnostic: the roundings of a 16-bit state path
        if op == "rnn_cell":
            return cells.rnn_cell(env["W"], env["b"], v[0], v[1])
        if op == "lstm_cell":
            return cells.lstm_cell(env["W"], env["b"], v[0], v[1])
        if op == "take_h":
            return v[0][: v[0].shape[0] // 2]
        if op == "take_h_grad":                     # (s, dh) -> ds
            return np.concatenate([v[1], np.zeros_like(v[1])])
        if op == "ce_head":
            return ops.ce_head(env["U"], env["u0"], v[0], v[1])
        if op == "ce_head_grad":                    # (h, label, dloss) -> dh
            return ops.ce_head_grad(env["U"], env["u0"], v[0], v[1], v[2])
        if op == "ce_node":                         # (state, tree node) -> the same state
            lab = int(env["node_label"][v[1]])
            if lab >= 0:                            # the loss term of this firing, kept by node
                h = v[0][: env["U"].shape[1]]
                self.node_loss[v[1]] = ops.ce_head(env["U"], env["u0"], h, lab)
            return v[0]
        if op == "ce_node_grad":                    # (state, tree node, dstate) -> dstate
            lab = int(env["node_label"][v[1]])
            ds = np.array(v[2], dtype=np.float64)
            if lab >= 0:
                H = env["U"].shape[1]
                ds[:H] += ops.ce_head_grad(env["U"], env["u0"], v[0][:H], lab, float(env["dnode"][v[1]]))
            return ds
        if op == "embed_grad":                      # (token, dy) -> sink
            self._add_rows("dE", v[0], v[1])
            return None
        if op == "embed_lstm_grad":
            self._add_rows("dE", v[0], v[1][: v[1].shape[0] // 2])
            return None
        if op == "rnn_cell_grad":                   # (h_l, h_r, dh) -> (dh_l, dh_r)
            dl, dr, delta, x = cells.rnn_cell_grad(env["W"], env["b"], v[0], v[1], v[2])
            self._add_outer("dW", "db", delta, x)
            return (dl, dr)
        if op == "lstm_cell_grad":
            dl, dr, dz, x = cells.lstm_cell_grad(env["W"], env["b"], v[0], v[1], v[2])
            self._add_outer("dW", "db", dz, x)
            return (dl, dr)
        raise ValueError("unknown op " + op)

    def _add_rows(self, name, row, vec):
        g = self.param_grad.get(name)
        if g is None:
            g = self.param_grad[name] = np.zeros_like(self.env["E"], dtype=np.float64)
        g[row] += vec

    def _add_outer(self, wname, bname, delta, x):
        buf = self._outer.setdefault(wname, ([], [], bname))
        buf[0].append(delta)
        buf[1].append(x)
        if len(buf[0]) >= 2048:
            self._flush_outer()

    def _flush_outer(self):
        """sum_t delta_t x_t^T over the buffered tags, written as one matrix product."""
        for wname, (ds, xs, bname) in self._outer.items():
            if not ds:
                continue
            D, X = np.stack(ds), np.stack(xs)
            self.param_grad[wname] = self.param_grad.get(wname, 0.0) + D.T @ X
            self.param_grad[bname] = self.param_grad.get(bname, 0.0) + D.sum(axis=0)
            ds.clear()
            xs.clear()

    # ------------------------------------------------------------------------------
    def _live_tags(self):
        """Tags below the root that some node still holds an unconsumed token of: a pending operand of
        a node that has not fired, or a node about to fire.  (Section 5.1: the frame of a tag is needed
        exactly that long; Return_i deallocates it.)  A Merge keeps its record after firing only to
        ignore later arrivals: that is not a token."""
        live = set()
        for (j, tag), rec in self.slots.items():
            if len(tag) > 1 and not (rec[3] and self.g.nodes[j].op in ("merge", "merge_entry")):
                live.add(tag)
        for j, tag in self.ready:
            if len(tag) > 1:
                live.add(tag)
        # only scopes that were really entered: a dead Call sends a dead control token under the tag
        # of a call that never happens, and no frame exists for it
        return {t for t in live if t in self.tags or t in self._entered_iters}

    def run(self, inputs, n_instances, max_rounds=10 ** 7, track_live=False):
        """inputs: {("in"|"gin", k): sequence indexed by instance}.  Returns
        {("out"|"gout", k): list indexed by instance}.  track_live: also record in peak_live_tags the
        largest number of tags alive in one round (slow: every round looks at every pending token)."""
        self.reset()
        for (kind, k), seq in inputs.items():
            j = self.g.inputs[(kind, k)]
            for b in range(n_instances):
                self.fire_count[j] += 1
                self._emit(j, 0, (b,), seq[b])
        # a node fed by constants only can fire under the root tag of every instance
        # (constants hold for all tags); this is how `result = fact(3)+5` starts
        for j, nd in enumerate(self.g.nodes):
            if self.n_wait[j] == 0 and nd.op not in ("const", "in", "gin"):
                if nd.fn != self.g.result_fn:
                    raise ValueError("node %s of %s has only constant inputs" % (nd.op, nd.fn))
                for b in range(n_instances):
                    self._schedule(j, (b,), self._slot(j, (b,)))
        while self.ready:
            if self.rounds >= max_rounds:
                raise RuntimeError("round limit exceeded")
            if track_live:
                self.peak_live_tags = max(self.peak_live_tags, len(self._live_tags()))
            batch, self.ready = self.ready, []
            self.rounds += 1
            for j, tag in batch:
                self._fire(j, tag)
        self._flush_outer()
        res = {}
        for key, per_tag in self.outputs.items():
            res[key] = [per_tag.get((b,)) for b in range(n_instances)]
        return res

    # ------------------------------------------------------------------------------
    def count_by_op(self):
        out = {}
        for nd, c in zip(self.g.nodes, self.fire_count):
            name = nd.op
            if nd.op == "merge_entry" and nd.attr["kind"] == "gin":
                name = "merge_entry_grad"
            if nd.op in ("call", "return"):
                name = "%s_%d" % (nd.op, nd.attr["label"])
                if nd.attr["kind"] != ("in" if nd.op == "call" else "out"):
                    name += "_grad"
            if nd.op in ("enter", "exit"):
                name = "%s_%d" % (nd.op, nd.attr["label"])
            out[name] = out.get(name, 0) + c
        return out
