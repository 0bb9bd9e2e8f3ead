"""GPU parity, per-node losses of fully labelled trees (Section 6; gradient operators of Section
4): the loss term of every node and the parameter gradients of a weighted sum of the terms,
HIP path against the oracle on the same seeded inputs.  fp32 within rel 1e-5 (gradients 2e-5),
bf16 within rel 2e-2 (Frobenius); firing counts bit-exact."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from tdf_workloads import make_config, SplitMix64  # noqa: E402
from gpu_util import TreeRun, run_oracle_node_loss, rel_fro, fire_counts  # noqa: E402
from paper_2410_20225_amd import tdf  # noqa: E402

FP32_TOL, BF16_TOL = 1e-5, 2e-2


def _losses(ref, n_nodes):
    want = np.zeros(n_nodes)
    for v, l in ref["node_loss"].items():
        want[v] = l
    return want


@pytest.mark.parametrize("kernels", ["default", "tiled_gemm_only", "no_tail"])
@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
@pytest.mark.parametrize("with_dy", [False, True])
def test_fp32_losses_and_gradients(cell, cfg, kernels, with_dy, monkeypatch):
    if kernels == "tiled_gemm_only":
        monkeypatch.setenv("TDF_SMALL_LEVEL", "0")
    if kernels == "no_tail":
        monkeypatch.setenv("TDF_NO_DIE_LOCAL", "1")
    c = make_config(cfg, n_trees=24, max_leaves=20, hidden=48, vocab=200)
    c["bf16"] = False
    c["u0"] = SplitMix64(8).normal(5) * 0.3
    F, B, H = c["forest"], c["forest"].n_trees, c["H"]
    lab = c["node_labels"].copy()
    lab[2::5] = -1                                           # partly labelled
    dnode = SplitMix64(4).normal(F.n_nodes)
    dy = SplitMix64(5).normal(B * H).reshape(B, H) if with_dy else None
    run = TreeRun(c, head=False, grad=True, node_labels=lab)
    st, stats = run.run(dy, dnode=dnode)
    dy_o = None if dy is None else ([np.concatenate([d, np.zeros(H)]) for d in dy] if cell == "lstm" else list(dy))
    ref = run_oracle_node_loss(c, lab, dnode, dy_o)
    got = run.out_node_loss.cpu().numpy()
    want = _losses(ref, F.n_nodes)
    assert np.array_equal(got == 0.0, want == 0.0) and not got[lab < 0].any()
    assert np.abs(got - want).max() <= FP32_TOL * np.abs(want).max()
    assert rel_fro(run.out_h.cpu().numpy(), np.stack(ref["out"])[:, :H]) < FP32_TOL
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-5, name
    counts = fire_counts(run.graph, stats)
    assert counts["ce_node"] == ref["it"].count_by_op()["ce_node"] == F.n_nodes


@pytest.mark.parametrize("cfg,n_trees,max_leaves,hidden,vocab", [
    (3, 96, 60, 300, 2000),      # H not a multiple of 32
    (4, 128, 128, 256, 3000),    # TreeLSTM: wide levels and a tail
    (5, 6, 512, 512, 500),       # deep chains and complete trees
    (3, 5, 1, 24, 30),           # single-leaf trees: the root's row is a leaf's
])
def test_bf16_losses_and_gradients(cfg, n_trees, max_leaves, hidden, vocab):
    c = make_config(cfg, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden, vocab=vocab)
    F = c["forest"]
    lab = c["node_labels"]
    dnode = np.full(F.n_nodes, 1.0 / F.n_nodes)              # mean over all nodes of the batch
    run = TreeRun(c, head=False, grad=True, node_labels=lab)
    for rep in range(2):                                     # the row marks are cleared per evaluation
        st, stats = run.run(None, dnode=dnode)
    ref = run_oracle_node_loss(c, lab, dnode)
    assert rel_fro(run.out_node_loss.cpu().numpy(), _losses(ref, F.n_nodes)) < BF16_TOL
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        if name in ref["grads"]:
            assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < BF16_TOL, name
        else:                                                # no cell fired
            assert F.n_nodes == F.n_trees and name != "dE" and not t.cpu().numpy().any()
    assert stats.n_tags == F.n_nodes


def test_forward_only_and_missing_buffers():
    c = make_config(4, n_trees=32, max_leaves=40, hidden=64, vocab=300)
    F = c["forest"]
    lab = c["node_labels"]
    run = TreeRun(c, head=False, grad=False, node_labels=lab)
    st, stats = run.run()
    ref = run_oracle_node_loss(c, lab)
    assert rel_fro(run.out_node_loss.cpu().numpy(), _losses(ref, F.n_nodes)) < BF16_TOL
    keep = run.out_node_loss
    run.out_node_loss = None
    st, _ = run.run(check=False)
    assert st == tdf.ERR_BAD_ARG and "out_node_loss" in tdf.last_error()
    run.out_node_loss = keep
    bad = lab.copy()
    bad[5] = 9                                               # not a class: no term, like a negative label
    run2 = TreeRun(c, head=False, grad=False, node_labels=bad)
    run2.run()
    got = run2.out_node_loss.cpu().numpy()
    assert got[5] == 0.0 and rel_fro(np.delete(got, 5), np.delete(_losses(ref, F.n_nodes), 5)) < BF16_TOL


def test_full_size_workload_on_sampled_trees():
    # workload 4 at the size the benchmark times, every node labelled; the gradient weights are
    # zero outside a sample of trees, so the gradients are those of the sample alone
    c = make_config(4)
    F = c["forest"]
    ids = [0, 7, 513, 2047, 3333, 4095]
    lab = c["node_labels"]
    dnode = np.zeros(F.n_nodes)
    n_s = 0
    for b in ids:
        r, n = int(F.roots[b]), 2 * int(F.n_leaves[b]) - 1
        dnode[r:r + n] = 1.0
        n_s += n
    dnode /= n_s
    run = TreeRun(c, head=False, grad=True, node_labels=lab, stats_level=0)
    st, stats = run.run(None, dnode=dnode)
    assert stats.n_tags == F.n_nodes
    ref = run_oracle_node_loss(c, lab, dnode, ids=ids)
    got = run.out_node_loss.cpu().numpy()
    assert (got > 0).all()                                   # every node of the batch has its term
    sel = dnode > 0
    assert rel_fro(got[sel], _losses(ref, F.n_nodes)[sel]) < BF16_TOL
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < BF16_TOL, name


def test_node_outside_the_forest_is_reported_and_unreached_nodes_have_no_term():
    # result(v) = ce_node(embed(token(v)), v + k): with k = 0 only the roots (here: leaves) get a
    # term and every other node of the forest stays at zero; with k far beyond the forest the
    # device raises an error instead of writing outside its arrays.  The program has no cell, and
    # no W or b is passed: the library must not touch them.
    T = tdf

    def program(k):
        nodes = [(T.OP_IN, [], 0), (T.OP_TREE_TOKEN, [(0, 0)], 0), (T.OP_EMBED, [(1, 0)], 0), (T.OP_CONST, [], k),
                 (T.OP_ADD, [(0, 0), (3, 0)], 0), (T.OP_CE_NODE, [(2, 0), (4, 0)], 0), (T.OP_OUT, [(5, 0)], 0)]
        return [("result", 1, nodes)], 0

    c = make_config(3, n_trees=6, max_leaves=5, hidden=32, vocab=50)
    F = c["forest"]
    leaves = np.flatnonzero(F.left < 0)[:6].astype(np.int64)   # instances start at leaves: token ids exist there
    t = lambda a, d: torch.tensor(np.ascontiguousarray(a), dtype=d, device="cuda:0")
    bufs = dict(args=t(leaves, torch.int64), left=t(F.left, torch.int32), right=t(F.right, torch.int32),
                token=t(F.token, torch.int32), E=t(c["E"], torch.bfloat16), U=t(c["U"], torch.float32),
                u0=t(c["u0"], torch.float32), node_label=t(c["node_labels"], torch.int32))
    out_h = torch.zeros(6, 32, dtype=torch.float32, device="cuda:0")
    for k, want in ((0, tdf.OK), (10 ** 7, tdf.ERR_BAD_ARG), (-10 ** 7, tdf.ERR_BAD_ARG)):
        fns, r = program(k)
        g = tdf.graph_build(fns, r)
        inp = tdf.make_inputs(6, n_args=1, dtype=tdf.BF16, hidden=32, vocab=c["V"], n_classes=5, max_tags=64, **bufs)
        ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device="cuda:0")
        loss = torch.full((F.n_nodes,), -1.0, dtype=torch.float32, device="cuda:0")
        st, stats = tdf.eval(g, inp, ws, out_h=out_h, out_node_loss=loss, check=False)
        assert st == want
        if st == tdf.OK:
            got = loss.cpu().numpy()
            h = c["E"][F.token[leaves]]
            lg = h @ c["U"].T + c["u0"]
            ref = np.log(np.exp(lg - lg.max(1, keepdims=True)).sum(1)) + lg.max(1) - lg[np.arange(6), c["node_labels"][leaves]]
            # a library routine's definition of the loss on a single embedding row; the oracle's own
            # check of this operator is in the tests above
            assert np.allclose(got[leaves], ref, rtol=2e-2)
            rest = np.ones(F.n_nodes, bool)
            rest[leaves] = False
            assert not got[rest].any()
