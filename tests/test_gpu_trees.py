"""GPU parity, recursive tree networks: forward values and gradients of the HIP path against
the oracle on the same seeded inputs.  Tolerances: fp32 within rel 1e-5, bf16 within rel 2e-2
(Frobenius norm of the difference over the Frobenius norm of the oracle's tensor); tag and
firing counts bit-exact."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from tdf_workloads import make_config  # noqa: E402
from gpu_util import TreeRun, run_oracle_tree, rel_fro, fire_counts, assert_close_bf16, assert_rows_close_bf16  # noqa: E402

FP32_TOL, BF16_TOL = 1e-5, 2e-2


def _check_counts(run, stats, ref):
    F = run.c["forest"]
    L = int(F.n_leaves.sum())
    assert stats.n_tags == F.n_nodes == len(ref["it"].tags)
    assert stats.n_leaf_rows == L and stats.n_cell_rows == L - F.n_trees
    assert stats.max_tag_depth == ref["it"].max_tag_len
    got = fire_counts(run.graph, stats)
    want = {k.replace("embed_lstm", "embed"): v for k, v in ref["it"].count_by_op().items()
            if k != "const" and not k.endswith("_grad") and k not in ("addn", "snd", "gin", "gout", "take_h")}
    # the oracle's gradient graph adds Merge / Switch nodes of its own: compare forward ops only
    for k in ("merge_entry", "isleaf", "switch", "token", "embed", "left", "right", "call_0", "call_1",
              "call_2", "return_0", "return_1", "return_2", run.c["cell"] + "_cell"):
        assert got[k] == want[k], k


@pytest.mark.parametrize("n_trees,max_leaves,hidden", [(256, 50, 128), (37, 9, 40)])
def test_treernn_fp32_forward(n_trees, max_leaves, hidden):
    c = make_config(2, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden)
    run = TreeRun(c, head=False, grad=False)
    st, stats = run.run()
    ref = run_oracle_tree(c, head=False, grad=False)
    want = np.stack(ref["out"])
    got = run.out_h.cpu().numpy()
    assert rel_fro(got, want) < FP32_TOL
    assert np.abs(got - want).max() < 1e-5 * max(1.0, np.abs(want).max())
    _check_counts(run, stats, ref)


@pytest.mark.parametrize("cfg,n_trees,max_leaves,hidden,vocab", [
    (3, 96, 60, 300, 2000),      # H not a multiple of 32: padded lanes must stay zero
    (4, 128, 128, 256, 3000),    # TreeLSTM, Zipf tokens, 20 % left chains
    (5, 6, 512, 512, 500),       # deep chains and complete trees
    (3, 5, 4, 24, 30),           # tiny: a single ragged tile
    (3, 7, 1, 40, 30),           # single-leaf trees: no cell fires, the head reads leaves' rows, dW = db = 0
    (4, 300, 1, 64, 50),         # the same for the TreeLSTM, repeated tokens
    (4, 1, 30, 64, 50),          # a batch of one tree
    (4, 20, 12, 1100, 100),      # a padded width above 1024: the gradient kernels' lanes take several runs of units
])
def test_bf16_forward_backward(cfg, n_trees, max_leaves, hidden, vocab):
    c = make_config(cfg, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden, vocab=vocab)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    run = TreeRun(c, head=True, grad=True)
    st, stats = run.run(dy)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    assert_close_bf16(run.out_f32.cpu().numpy(), np.array(ref["out"]), "loss of every tree")
    if "dW" in ref["grads"]:
        assert_close_bf16(run.dW.cpu().numpy(), ref["grads"]["dW"], "dW")
        assert_close_bf16(run.db.cpu().numpy(), ref["grads"]["db"], "db")
    else:   # no cell fired: the oracle has no gradient for W and b, the library returns zeros
        assert (c["forest"].left < 0).all() and not run.dW.any() and not run.db.any()
    dE, dE_ref = run.dE.cpu().numpy(), ref["grads"]["dE"]
    assert_close_bf16(dE, dE_ref, "dE")
    untouched = np.ones(c["V"], bool)
    untouched[np.unique(c["forest"].token[c["forest"].token >= 0])] = False
    assert not dE[untouched].any()
    assert_rows_close_bf16(dE[~untouched], dE_ref[~untouched], "dE, token by token")
    _check_counts(run, stats, ref)
    # every tag's gradient body fired exactly once: marked and counted on the device, and the same
    # in the oracle (its per-tag counters of the gradient bodies)
    assert set(ref["it"].bwd_body.values()) == {1}
    assert stats.n_grad_firings == len(ref["it"].bwd_body) == stats.n_tags and stats.n_grad_not_once == 0


@pytest.mark.parametrize("cfg,n_trees,max_leaves,hidden,vocab", [
    (3, 96, 60, 300, 2000),
    (4, 128, 128, 256, 3000),
    (5, 4, 256, 512, 500),
])
@pytest.mark.parametrize("grad", [False, True], ids=["forward", "with_gradient"])
def test_bf16_root_states_against_oracle(cfg, n_trees, max_leaves, hidden, vocab, grad):
    # no head: the result is the root's state itself (h, and c of the TreeLSTM), 16-bit path
    c = make_config(cfg, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden, vocab=vocab)
    B, H = c["forest"].n_trees, c["H"]
    lstm = c["cell"] == "lstm"
    from tdf_workloads import SplitMix64
    dy = SplitMix64(11).normal(B * H).reshape(B, H) if grad else None
    run = TreeRun(c, head=False, grad=grad)
    st, stats = run.run(dy)
    dy_o = None
    if grad:
        dy_o = [np.concatenate([d, np.zeros(H)]) for d in dy] if lstm else list(dy)
    ref = run_oracle_tree(c, head=False, grad=grad, dy=dy_o)
    want = np.stack(ref["out"])
    assert_close_bf16(run.out_h.cpu().numpy(), want[:, :H], "root h")
    assert_rows_close_bf16(run.out_h.cpu().numpy(), want[:, :H], "root h, tree by tree")
    if lstm:
        assert_close_bf16(run.out_c.cpu().numpy(), want[:, H:], "root c")
        assert_rows_close_bf16(run.out_c.cpu().numpy(), want[:, H:], "root c, tree by tree")
    if grad:
        for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
            assert_close_bf16(t.cpu().numpy(), ref["grads"][name], name)
        assert stats.n_grad_firings == stats.n_tags and stats.n_grad_not_once == 0


@pytest.mark.parametrize("cfg,bf16", [(2, False), (4, True)])
def test_forest_with_permuted_node_numbers(cfg, bf16):
    # the trees' nodes scattered over the index space: trees interleave, children may come before
    # their parents.  Node numbers are only names; nothing may depend on their order.
    from tdf_workloads import SplitMix64, permuted
    c = make_config(cfg, n_trees=40, max_leaves=24, hidden=64, vocab=300)
    F = c["forest"]
    order = np.argsort(SplitMix64(5).uniform(F.n_nodes), kind="stable")
    c["forest"] = permuted(F, order)
    grad = bf16
    B = F.n_trees
    dy = np.full(B, 1.0 / B) if grad else None
    run = TreeRun(c, head=grad, grad=grad)
    st, stats = run.run(dy)
    ref = run_oracle_tree(c, head=grad, grad=grad, dy=dy)
    _check_counts(run, stats, ref)
    if grad:
        assert_close_bf16(run.out_f32.cpu().numpy(), np.array(ref["out"]), "loss of every tree")
        for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
            assert_close_bf16(t.cpu().numpy(), ref["grads"][name], name)
        # ... and the same numbers as with the original numbering (same trees, same tokens)
        c0 = dict(c)
        c0["forest"] = F
        ref0 = run_oracle_tree(c0, head=True, grad=True, dy=dy)
        assert np.allclose(np.array(ref["out"]), np.array(ref0["out"]), rtol=1e-12, atol=0)
    else:
        want = np.stack(ref["out"])
        assert rel_fro(run.out_h.cpu().numpy(), want) < FP32_TOL


def test_token_id_outside_the_vocabulary_is_an_error():
    from paper_2410_20225_amd import tdf
    c = make_config(2, n_trees=8, max_leaves=6, hidden=32, vocab=50)
    F = c["forest"]
    leaf = int(np.nonzero(F.token >= 0)[0][3])
    F.token[leaf] = 50                                   # one past the last row of E
    run = TreeRun(c, head=False, grad=False)
    st, stats = run.run(check=False)
    assert st == tdf.ERR_BAD_ARG and "token" in tdf.last_error()


@pytest.mark.parametrize("kernels", ["default", "tiled_gemm_only"])
@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
def test_vector_result_with_given_dy_fp32(cell, cfg, kernels, monkeypatch):
    # no head: the caller supplies dL/dh of every root; fp32 end to end, also with every level
    # through the tiled GEMM (fp32 MFMA, ragged tiles: H = 48 is padded to 64)
    if kernels != "default":
        monkeypatch.setenv("TDF_SMALL_LEVEL", "0")
    c = make_config(cfg, n_trees=24, max_leaves=20, hidden=48, vocab=200)
    c["bf16"] = False
    B, H = c["forest"].n_trees, c["H"]
    from tdf_workloads import SplitMix64
    dy = SplitMix64(4).normal(B * H).reshape(B, H)
    run = TreeRun(c, head=False, grad=True)
    st, stats = run.run(dy)
    dy_o = [np.concatenate([d, np.zeros(H)]) for d in dy] if cell == "lstm" else list(dy)
    ref = run_oracle_tree(c, head=False, grad=True, dy=dy_o)
    want = np.stack(ref["out"])
    assert rel_fro(run.out_h.cpu().numpy(), want[:, :H]) < FP32_TOL
    if cell == "lstm":
        assert rel_fro(run.out_c.cpu().numpy(), want[:, H:]) < FP32_TOL
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-5, name


def test_incomplete_forest_is_rejected_before_anything_runs():
    from paper_2410_20225_amd import tdf
    c = make_config(2, n_trees=4, max_leaves=6, hidden=32)
    run = TreeRun(c, head=False, grad=False)
    keep = run.inputs.right
    run.inputs.right = None
    st, _ = run.run(check=False)
    assert st == tdf.ERR_BAD_ARG and "forest" in tdf.last_error()
    run.inputs.right = keep
    run.inputs.n_tree_nodes = 0
    st, _ = run.run(check=False)
    assert st == tdf.ERR_BAD_ARG
    run.inputs.n_tree_nodes = c["forest"].n_nodes
    st, _ = run.run()
    assert st == tdf.OK


def test_state_rows_exhausted_is_reported():
    c = make_config(2, n_trees=16, max_leaves=20, hidden=32)
    run = TreeRun(c, head=False, grad=False, max_tags=c["forest"].n_nodes // 2)
    st, stats = run.run(check=False)
    from paper_2410_20225_amd import tdf
    assert st == tdf.ERR_TABLE_FULL


@pytest.mark.parametrize("cfg,ids", [
    (3, [0, 5, 77, 500, 901, 1023]),                  # TreeRNN, 1024 trees, H = 300
    (4, [0, 7, 513, 1024, 2047, 3000, 3333, 4095]),   # TreeLSTM, 4096 trees
    (5, [3, 100]),                                    # a left chain and a complete tree of 4096 leaves
])
def test_full_size_workload_on_sampled_trees(cfg, ids):
    # The workload at the size and in the launch configuration the benchmark times.  The oracle
    # cannot run all of it, but trees are independent: with dy zero outside a sample, the weight,
    # bias and embedding gradients of the whole batch are those of the sample alone, and the
    # sample's losses are the oracle's.
    c = make_config(cfg)
    F = c["forest"]
    B = F.n_trees
    dy = np.zeros(B)
    dy[ids] = 1.0 / len(ids)
    run = TreeRun(c, head=True, grad=True, stats_level=0)
    st, stats = run.run(dy)
    assert stats.n_tags == F.n_nodes
    L = int(F.n_leaves.sum())
    assert stats.n_leaf_rows == L and stats.n_cell_rows == L - B
    assert stats.max_tag_depth == int(F.n_leaves.max()) if cfg == 5 else stats.max_tag_depth >= 2
    sub = dict(c)
    sub["forest"] = F.subset(ids)
    sub["labels"] = c["labels"][ids]
    ref = run_oracle_tree(sub, head=True, grad=True, dy=dy[ids])
    assert_close_bf16(run.out_f32.cpu().numpy()[ids], np.array(ref["out"]), "losses of the sampled trees")
    assert_close_bf16(run.dW.cpu().numpy(), ref["grads"]["dW"], "dW")
    assert_close_bf16(run.db.cpu().numpy(), ref["grads"]["db"], "db")
    dE, dE_ref = run.dE.cpu().numpy(), ref["grads"]["dE"]
    assert_close_bf16(dE, dE_ref, "dE")
    untouched = np.ones(c["V"], bool)
    untouched[np.unique(sub["forest"].token[sub["forest"].token >= 0])] = False
    assert not dE_ref[untouched].any()
    assert np.abs(dE[untouched]).max() == 0.0          # rows of tokens outside the sample: exactly zero
    assert_rows_close_bf16(dE[~untouched], dE_ref[~untouched], "dE, token by token")
    assert stats.n_grad_firings == stats.n_tags and stats.n_grad_not_once == 0
    assert stats.generated == 1 and stats.die_local == 1 and stats.repeats == 0   # the way the benchmark takes
    del run
    # the root states themselves (no head), forward only, same batch: h (and c) of the sampled trees
    run = TreeRun(c, head=False, grad=False, stats_level=0)
    st, stats = run.run()
    ref = run_oracle_tree(sub, head=False, grad=False)
    want = np.stack(ref["out"])
    H = c["H"]
    assert_close_bf16(run.out_h.cpu().numpy()[ids], want[:, :H], "root h of the sampled trees")
    assert_rows_close_bf16(run.out_h.cpu().numpy()[ids], want[:, :H], "root h, tree by tree")
    if c["cell"] == "lstm":
        assert_close_bf16(run.out_c.cpu().numpy()[ids], want[:, H:], "root c of the sampled trees")
