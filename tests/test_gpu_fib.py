"""GPU parity, integer recursion: values, tag counts and per-node firing counts of the HIP
tag machine against the oracle, bit-exact (workload 1: fib(n), n = 0..20)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
import oracle  # noqa: E402
from oracle import programs as oprog  # noqa: E402
from gpu_util import DEV, fire_counts  # noqa: E402


def _eval_int(fns, r, args, max_tags, n_args=1, step_limit=0, check=True):
    g = tdf.graph_build(fns, r)
    B = max(len(args), 1) if n_args else 1
    t_args = torch.tensor(args, dtype=torch.int64, device=DEV).reshape(-1) if n_args else None
    inp = tdf.make_inputs(B, args=t_args, n_args=n_args, max_tags=max_tags, step_limit=step_limit)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((B,), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out, check=check)
    return st, stats, out.cpu().numpy(), g


def test_fact_example():
    fns, r = programs.fact()
    st, stats, out, g = _eval_int(fns, r, [], 16, n_args=0)
    assert out.tolist() == [11]
    assert stats.n_tags == 3 and stats.max_tag_depth == 3


def test_fib_batch_matches_oracle_bit_exact():
    fns, r = programs.fib()
    st, stats, out, g = _eval_int(fns, r, list(range(21)), 57291)
    it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
    want = it.run({("in", 0): list(range(21))}, 21)[("out", 0)]
    assert out.tolist() == want
    assert stats.n_tags == len(it.tags) == 57291
    assert stats.max_tag_depth == it.max_tag_len == 20
    got = fire_counts(g, stats)
    ref = {k: v for k, v in it.count_by_op().items() if k != "const"}
    assert got == ref
    assert stats.max_probe < 64


def test_fib_separate_calls_equal_the_batch():
    fns, r = programs.fib()
    total = 0
    for n in (0, 1, 2, 7, 15):
        st, stats, out, _ = _eval_int(fns, r, [n], 4000)
        it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
        assert out.tolist() == it.run({("in", 0): [n]}, 1)[("out", 0)]
        assert stats.n_tags == len(it.tags)


def test_capacity_and_step_limit_are_reported_not_faulted():
    fns, r = programs.fib()
    st, stats, out, _ = _eval_int(fns, r, [18], 500, check=False)          # needs 8361 tags
    assert st == tdf.ERR_TABLE_FULL and stats.device_status == tdf.ERR_TABLE_FULL
    st, stats, out, _ = _eval_int(fns, r, [18], 10000, step_limit=10, check=False)
    assert st == tdf.ERR_STEP_LIMIT
    st, stats, out, _ = _eval_int(fns, r, [18], 10000)                      # and the library still works
    assert out.tolist() == [2584]


def test_fourteen_million_tags_in_one_batch():
    # fib(30), fib(31), fib(32) side by side: far beyond what the oracle can run, so the values are
    # checked against the Fibonacci numbers and the tag count against 2 F(n+1) - 1 invocations per
    # instance (the count the oracle is pinned to at small n); the longest tag is fib(32)'s chain
    # of 32 labels.  Instances of such different sizes also overflow the table part of a single
    # tag machine, which the library answers by running the batch on one machine.
    F = [0, 1]
    while len(F) < 40:
        F.append(F[-1] + F[-2])
    ns = [30, 31, 32]
    want_tags = sum(2 * F[n + 1] - 1 for n in ns)
    assert want_tags == 14098309
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    t_args = torch.tensor(ns, dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(3, args=t_args, n_args=1, max_tags=15_000_000, stats_level=0)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((3,), -1, dtype=torch.int64, device=DEV)
    for rep in range(2):
        st, stats = tdf.eval(g, inp, ws, out_i64=out)
        assert out.cpu().tolist() == [F[n] for n in ns]
        assert stats.n_tags == want_tags and stats.max_tag_depth == 32
    del ws
    torch.cuda.empty_cache()
