"""GPU parity, recursive tree networks: forward values and gradients of the HIP path against
the oracle on the same seeded inputs.  Tolerances: fp32 within rel 1e-5, bf16 within rel 2e-2
(Frobenius norm of the difference over the Frobenius norm of the oracle's tensor); tag and
firing counts bit-exact."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from tdf_workloads import make_config  # noqa: E402
from gpu_util import TreeRun, run_oracle_tree, rel_fro, fire_counts  # noqa: E402

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
])
def test_bf16_forward_backward(cfg, n_trees, max_leaves, hidden, vocab):
    c = make_config(cfg, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden, vocab=vocab)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    run = TreeRun(c, head=True, grad=True)
    st, stats = run.run(dy)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    assert rel_fro(run.out_f32.cpu().numpy(), np.array(ref["out"])) < BF16_TOL
    assert rel_fro(run.dW.cpu().numpy(), ref["grads"]["dW"]) < BF16_TOL
    assert rel_fro(run.db.cpu().numpy(), ref["grads"]["db"]) < BF16_TOL
    dE, dE_ref = run.dE.cpu().numpy(), ref["grads"]["dE"]
    assert rel_fro(dE, dE_ref) < BF16_TOL
    untouched = np.ones(c["V"], bool)
    untouched[np.unique(c["forest"].token[c["forest"].token >= 0])] = False
    assert not dE[untouched].any()
    _check_counts(run, stats, ref)
    assert stats.n_grad_firings == stats.n_tags          # one gradient-body firing per tag
    assert set(ref["it"].bwd_body.values()) == {1} and len(ref["it"].bwd_body) == stats.n_tags


@pytest.mark.parametrize("kernels", ["default", "tiled_gemm_only", "tiled_gemm_four_waves"])
@pytest.mark.parametrize("cell,cfg", [("rnn", 3), ("lstm", 4)])
def test_vector_result_with_given_dy_fp32(cell, cfg, kernels, monkeypatch):
    # no head: the caller supplies dL/dh of every root; fp32 end to end, also with every level
    # through the tiled GEMM (fp32 MFMA, ragged tiles: H = 48 is padded to 64)
    if kernels != "default":
        monkeypatch.setenv("TDF_SMALL_LEVEL", "0")
    if kernels == "tiled_gemm_four_waves":
        monkeypatch.setenv("TDF_GEMM_WAVES", "4")
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
    assert rel_fro(run.out_f32.cpu().numpy()[ids], np.array(ref["out"])) < BF16_TOL
    assert rel_fro(run.dW.cpu().numpy(), ref["grads"]["dW"]) < BF16_TOL
    assert rel_fro(run.db.cpu().numpy(), ref["grads"]["db"]) < BF16_TOL
    dE, dE_ref = run.dE.cpu().numpy(), ref["grads"]["dE"]
    assert rel_fro(dE, dE_ref) < BF16_TOL
    untouched = np.ones(c["V"], bool)
    untouched[np.unique(sub["forest"].token[sub["forest"].token >= 0])] = False
    assert not dE_ref[untouched].any()
    assert np.abs(dE[untouched]).max() == 0.0          # rows of tokens outside the sample: exactly zero
