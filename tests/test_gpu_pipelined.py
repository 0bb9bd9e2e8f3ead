"""Evaluations from two host threads at once, each with its own graph, workspace and stream: the
library lets one evaluation's tag machine run beside the data plane of the evaluation before it (the
control plane depends on the trees only) and serialises the rest.  Every evaluation must give what it
gives alone: counts and integers bit for bit, the losses bit for bit (one cell's arithmetic does not
depend on what else runs), the gradient sums within the summation-order bar of the other parity tests,
and the oracle's values within the workload's bar."""
import threading

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
from tdf_workloads import make_config  # noqa: E402
from gpu_util import DEV, TreeRun, run_oracle_tree, rel_fro  # noqa: E402


def _in_threads(fns):
    """Runs the callables at once, one thread and one stream each; re-raises what a thread raised."""
    gate = threading.Barrier(len(fns))
    errors = []

    def work(fn):
        try:
            with torch.cuda.stream(torch.cuda.Stream()):
                gate.wait()
                fn()
                torch.cuda.current_stream().synchronize()
        except BaseException as e:   # noqa: BLE001
            errors.append(e)
            gate.abort()

    threads = [threading.Thread(target=work, args=(fn,)) for fn in fns]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    if errors:
        raise errors[0]


def test_two_tree_evaluations_in_flight_give_what_one_gives_alone():
    c = make_config(4, n_trees=600, max_leaves=40, hidden=128, vocab=800)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    alone = TreeRun(c, head=True, grad=True)
    st, stats_alone = alone.run(dy)
    want = {k: getattr(alone, k).clone() for k in ("out_f32", "dW", "db", "dE")}
    runs = [TreeRun(c, head=True, grad=True) for _ in range(2)]
    got = [[] for _ in runs]

    def loop(i):
        for _ in range(6):
            st_i, stats = runs[i].run(dy)
            got[i].append((stats.n_tags, stats.n_steps, stats.n_grad_firings, stats.n_grad_not_once,
                           {k: getattr(runs[i], k).clone() for k in want}))

    _in_threads([lambda i=i: loop(i) for i in range(2)])
    for i in range(2):
        assert len(got[i]) == 6
        for n_tags, n_steps, n_gf, n_bad, t in got[i]:
            assert n_tags == stats_alone.n_tags == len(ref["it"].tags) and n_steps == stats_alone.n_steps
            assert n_gf == n_tags and n_bad == 0
            assert torch.equal(t["out_f32"], want["out_f32"])
            for k in ("dW", "db", "dE"):
                assert rel_fro(t[k].cpu().numpy(), want[k].cpu().numpy()) < 1e-5, k
    last = got[1][-1][4]
    assert rel_fro(last["out_f32"].cpu().numpy(), np.array(ref["out"])) < 2e-2
    for k in ("dW", "db", "dE"):
        assert rel_fro(last[k].cpu().numpy(), ref["grads"][k]) < 2e-2, k


def test_an_integer_program_beside_a_tree_network():
    c = make_config(3, n_trees=300, max_leaves=30, hidden=64, vocab=400)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    tree = TreeRun(c, head=True, grad=True)
    tree.run(dy)
    want_loss = tree.out_f32.clone()
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    args = torch.arange(0, 19, dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(19, args=args, n_args=1, max_tags=22000)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((19,), -1, dtype=torch.int64, device=DEV)
    fib = [0, 1]
    while len(fib) < 19:
        fib.append(fib[-1] + fib[-2])
    seen = []

    def ints():
        for _ in range(10):
            out.fill_(-1)
            st, stats = tdf.eval(g, inp, ws, out_i64=out)
            torch.cuda.current_stream().synchronize()
            seen.append((out.cpu().tolist(), stats.n_tags))

    def trees():
        for _ in range(10):
            tree.run(dy)
            assert torch.equal(tree.out_f32, want_loss)

    _in_threads([ints, trees])
    assert len(seen) == 10
    for values, n_tags in seen:
        assert values == fib and n_tags == sum(2 * f - 1 for f in fib[1:] + [fib[-1] + fib[-2]])


def test_one_graph_from_two_threads_takes_turns():
    # a graph owns streams, events and a host buffer: two threads that share it do not overlap
    c = make_config(3, n_trees=200, max_leaves=24, hidden=64, vocab=300)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    run = TreeRun(c, head=True, grad=True)
    st, stats = run.run(dy)
    want = {k: getattr(run, k).clone() for k in ("out_f32", "dW", "db", "dE")}
    counts = []

    def loop():
        for _ in range(5):
            st_i, s_i = run.run(dy)
            counts.append((s_i.n_tags, s_i.n_grad_firings, s_i.n_grad_not_once))

    _in_threads([loop, loop])
    assert counts == [(stats.n_tags, stats.n_tags, 0)] * 10
    assert torch.equal(run.out_f32, want["out_f32"])
    for k in ("dW", "db", "dE"):
        assert rel_fro(getattr(run, k).cpu().numpy(), want[k].cpu().numpy()) < 1e-5, k
