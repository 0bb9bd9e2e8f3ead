"""GPU parity on seeded random cases: forests of random size, depth and hidden width (ragged
tiles, odd widths) for the three tree workloads, and integer programs (recursion, loops) on random
arguments; every case evaluated three times in a row on the same graph and workspace.  Same bars
as the other parity tests."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
import oracle  # noqa: E402
from oracle import programs as oprog  # noqa: E402
from tdf_workloads import make_config, SplitMix64  # noqa: E402
from gpu_util import DEV, TreeRun, run_oracle_tree, run_oracle_node_loss, rel_fro  # noqa: E402


@pytest.mark.parametrize("seed", range(9))
def test_random_forests(seed):
    r = SplitMix64(1000 + seed)
    cfg = [3, 4, 5][seed % 3]
    n_trees, max_leaves, hidden = (int(r.randint(lo, hi, 1)[0]) for lo, hi in ((1, 400), (2, 90), (8, 200)))
    if cfg == 5:                                     # a few deep chains and complete trees
        n_trees, max_leaves = int(r.randint(2, 12, 1)[0]), 2 ** int(r.randint(1, 8, 1)[0])
    c = make_config(cfg, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden, vocab=300, seed=seed * 7 + 1)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    run = TreeRun(c, head=True, grad=True)
    for _ in range(3):
        st, stats = run.run(dy)
        assert stats.n_tags == c["forest"].n_nodes == len(ref["it"].tags)
        assert stats.max_tag_depth == ref["it"].max_tag_len
        assert rel_fro(run.out_f32.cpu().numpy(), np.array(ref["out"])) < 2e-2
        for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
            assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-2, name


@pytest.mark.parametrize("seed", range(6))
def test_random_forests_with_a_loss_term_at_random_nodes(seed):
    r = SplitMix64(2000 + seed)
    cfg = [3, 4, 5][seed % 3]
    n_trees, max_leaves, hidden = (int(r.randint(lo, hi, 1)[0]) for lo, hi in ((1, 300), (1, 70), (8, 160)))
    if cfg == 5:
        n_trees, max_leaves = int(r.randint(2, 12, 1)[0]), 2 ** int(r.randint(1, 8, 1)[0])
    c = make_config(cfg, n_trees=n_trees, max_leaves=max_leaves, hidden=hidden, vocab=300, seed=seed * 11 + 3)
    F = c["forest"]
    lab = c["node_labels"].copy()
    lab[r.uniform(F.n_nodes) < 0.3] = -1                      # three nodes in ten carry no label
    dnode = r.normal(F.n_nodes) / F.n_nodes
    D = c["H"] * (2 if c["cell"] == "lstm" else 1)
    dy = r.normal(F.n_trees * c["H"]).reshape(F.n_trees, c["H"]) / F.n_nodes if seed % 2 else None
    dy_o = None if dy is None else [np.concatenate([d, np.zeros(D - c["H"])]) for d in dy]
    ref = run_oracle_node_loss(c, lab, dnode, dy_o)
    want = np.zeros(F.n_nodes)
    for v, l in ref["node_loss"].items():
        want[v] = l
    run = TreeRun(c, head=False, grad=True, node_labels=lab)
    for _ in range(3):
        st, stats = run.run(dy, dnode=dnode)
        got = run.out_node_loss.cpu().numpy()
        assert np.array_equal(got == 0.0, want == 0.0)
        assert rel_fro(got, want) < 2e-2
        for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
            if name in ref["grads"]:
                assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-2, name


INT_CASES = [("fib", programs.fib, oprog.fib_program, 1, 0, 17), ("tak", programs.tak, oprog.tak_program, 3, 0, 9),
             ("ack", programs.ack, oprog.ack_program, 2, 0, 3), ("gcd", programs.gcd_loop, oprog.gcd_loop_program, 2, 1, 200),
             ("nested", programs.nested_loop, oprog.nested_loop_program, 1, 0, 25),
             ("tet", programs.loop_in_function, oprog.loop_in_function_program, 1, 0, 30)]


@pytest.mark.parametrize("seed", range(2))
@pytest.mark.parametrize("case", INT_CASES, ids=[c[0] for c in INT_CASES])
def test_integer_programs_on_random_arguments(case, seed):
    name, gpu_prog, oracle_prog, n_args, lo, hi = case
    r = SplitMix64(5000 + seed)
    n = int(r.randint(1, 60, 1)[0])
    args = np.stack([r.randint(lo, hi, n) for _ in range(n_args)], 1).astype(np.int64)
    it = oracle.Interpreter(oracle.transform(oracle_prog()))
    want = it.run({("in", k): args[:, k].tolist() for k in range(n_args)}, n)[("out", 0)]
    n_tags = len(it.tags) + len(it.iter_tags)
    fns, res = gpu_prog()
    g = tdf.graph_build(fns, res)
    t_args = torch.tensor(args, dtype=torch.int64, device=DEV).reshape(-1)
    inp = tdf.make_inputs(n, args=t_args, n_args=n_args, max_tags=n_tags + 4)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    for _ in range(3):
        st, stats = tdf.eval(g, inp, ws, out_i64=out)
        assert out.cpu().tolist() == want
        assert stats.n_tags == n_tags and stats.max_tag_depth == it.max_tag_len
