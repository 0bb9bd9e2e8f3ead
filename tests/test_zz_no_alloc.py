"""The entry point that allocates nothing (tdf_eval_static) against tdf_eval, through the C ABI:
same inputs, same results, bit for bit for integers and counts; twice in a row on the shared static
workspace, the second time with a smaller batch (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
from tdf_workloads import make_config  # noqa: E402

DEV = "cuda:0"


def _fib_both(g, ns):
    args = torch.tensor(ns, dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(len(ns), args=args, n_args=1, max_tags=22000)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    want = torch.full((len(ns),), -1, dtype=torch.int64, device=DEV)
    got = torch.full((len(ns),), -2, dtype=torch.int64, device=DEV)
    _, s_want = tdf.eval(g, inp, ws, out_i64=want)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    _, s_got = tdf.eval_static(g, inp, out_i64=got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert got.cpu().tolist() == want.cpu().tolist()
    assert s_got.n_tags == s_want.n_tags and s_got.n_tokens == s_want.n_tokens
    assert s_got.max_tag_depth == s_want.max_tag_depth
    assert list(s_got.fire_count) == list(s_want.fire_count)
    return got.cpu().tolist()


def test_static_workspace_entry_matches_tdf_eval_twice_in_a_row():
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    tdf.graph_prepare(g)
    big = _fib_both(g, list(range(19)))            # 21,873 tags
    assert big[18] == 2584
    small = _fib_both(g, [3, 9, 14, 2, 5])         # a smaller batch on the same array, right after
    assert small == [2, 34, 377, 1, 5]


def test_static_workspace_entry_on_a_tree_network():
    # forward TreeRNN (fp32): root states equal to those of tdf_eval on the same inputs, element by
    # element (same kernels, same order inside every sum), again with a smaller batch second
    from paper_2410_20225_amd.harness import TreeRun
    for n_trees in (48, 7):
        c = make_config(2, n_trees=n_trees, max_leaves=30, hidden=64, vocab=300)
        run = TreeRun(c, head=False, grad=False)
        run.run()
        want = run.out_h.clone()
        tdf.graph_prepare(run.graph)
        got = torch.zeros_like(want)
        st, stats = tdf.eval_static(run.graph, run.inputs, out_h=got)
        torch.cuda.synchronize()
        assert stats.n_tags == c["forest"].n_nodes
        assert torch.equal(got, want)


def test_static_workspace_entry_refuses_what_does_not_fit_or_was_not_prepared():
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    args = torch.arange(0, 4, dtype=torch.int64, device=DEV)
    out = torch.zeros(4, dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(4, args=args, n_args=1, max_tags=1000)
    st, _ = tdf.eval_static(g, inp, out_i64=out, check=False)
    assert st == tdf.ERR_BAD_ARG and "tdf_graph_prepare" in tdf.last_error()
    tdf.graph_prepare(g)
    huge = tdf.make_inputs(4, args=args, n_args=1, max_tags=50_000_000)
    assert tdf.workspace_size(g, huge) > tdf.STATIC_WORKSPACE_BYTES
    st, _ = tdf.eval_static(g, huge, out_i64=out, check=False)
    assert st == tdf.ERR_WORKSPACE and "static" in tdf.last_error()
    st, _ = tdf.eval_static(g, inp, out_i64=out)
    assert out.cpu().tolist() == [0, 1, 1, 2]
