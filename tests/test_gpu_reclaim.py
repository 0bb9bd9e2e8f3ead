"""GPU parity with frames given back on Return (Section 5.1: Return_i checks the label and
deallocates the frame): forward evaluation of integer programs with stats_level 0.  Values and tag
counts bit-exact; max_tags is then a bound on the tags alive at once, taken from the interval model
that the oracle's own live-tag count is pinned to (tests/live_model.py,
tests/test_oracle_live_tags.py), evaluated with this executor's step constants."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
import oracle  # noqa: E402
from oracle import programs as oprog  # noqa: E402
from tdf_workloads import make_config  # noqa: E402
from live_model import fib_peak_live  # noqa: E402
from gpu_util import DEV  # noqa: E402

# a frame is created in the step after its caller's sweep, a base case is complete (and given back)
# in its first sweep, a caller one step after its deeper call: A : c : r = 2 : 1 : 1.  Lanes that go
# on with the frame they created in the same step (chains of first calls) run ahead of that
# schedule, so the engine may hold somewhat more: a quarter more is allowed.
ENGINE = (2, 1, 1)
SLACK = 1.25


def _run(fns, r, args, n_args, max_tags, stats_level=0, check=True):
    g = tdf.graph_build(fns, r)
    B = len(args)
    t_args = torch.tensor(args, dtype=torch.int64, device=DEV).reshape(-1)
    inp = tdf.make_inputs(B, args=t_args, n_args=n_args, max_tags=max_tags, stats_level=stats_level)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((B,), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out, check=check)
    return st, stats, out.cpu().tolist()


def test_fib_batch_in_a_table_of_its_live_tags():
    ns = list(range(21))
    it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
    want = it.run({("in", 0): ns}, len(ns))[("out", 0)]
    # (machines run at their own pace: the bound is the sum of the instances' own peaks)
    bound = int(SLACK * sum(fib_peak_live([n], *ENGINE) for n in ns))
    assert bound < len(it.tags)
    fns, r = programs.fib()
    for rep in range(2):
        st, stats, out = _run(fns, r, ns, 1, bound)
        assert out == want
        assert stats.n_tags == len(it.tags) == 57291 and stats.max_tag_depth == it.max_tag_len
        assert stats.frames_reclaimed == 1 and stats.peak_frames <= bound
    # the same table is too small when every frame is kept (per-node counts are asked for)
    st, stats, out = _run(fns, r, ns, 1, bound, stats_level=1, check=False)
    assert st == tdf.ERR_TABLE_FULL and stats.frames_reclaimed == 0


def test_fourteen_million_tags_in_a_table_of_their_live_tags():
    F = [0, 1]
    while len(F) < 40:
        F.append(F[-1] + F[-2])
    ns = [30, 31, 32]
    want_tags = sum(2 * F[n + 1] - 1 for n in ns)
    bound = int(SLACK * sum(fib_peak_live([n], *ENGINE) for n in ns))
    assert bound < want_tags
    fns, r = programs.fib()
    st, stats, out = _run(fns, r, ns, 1, bound)
    assert out == [F[n] for n in ns]
    assert stats.n_tags == want_tags and stats.max_tag_depth == 32
    assert stats.frames_reclaimed == 1 and stats.peak_frames <= bound
    print("fib(30..32): %d tags, %d frame records used (bound %d)" % (stats.n_tags, stats.peak_frames, bound))
    torch.cuda.empty_cache()


def test_loops_run_in_a_few_frames_per_instance():
    # workload 6 at full size: 65,536 subtractive-gcd loops, about two million iterations, in a table
    # of four tags per instance (the oracle: at most two alive per loop instance)
    c = make_config(6)
    ab = c["args"]
    fns, r = programs.gcd_loop()
    B = len(ab)
    st, stats, out = _run(fns, r, ab.tolist(), 2, 4 * B)
    assert out == np.gcd(ab[:, 0], ab[:, 1]).tolist()
    it = oracle.Interpreter(oracle.transform(oprog.gcd_loop_program()))
    sub = ab[:256]
    it.run({("in", 0): sub[:, 0].tolist(), ("in", 1): sub[:, 1].tolist()}, len(sub), track_live=True)
    assert it.peak_live_tags <= 2 * len(sub)
    assert stats.frames_reclaimed == 1 and stats.peak_frames <= 4 * B < stats.n_tags
    print("gcd loops: %d tags, %d frame records used" % (stats.n_tags, stats.peak_frames))


@pytest.mark.parametrize("name", ["ack", "tak", "loop_of_calls", "nested_loop", "loop_in_function"])
def test_frames_given_back_in_every_kind_of_scope(name):
    # several parameters per call, calls as arguments of calls, loops in functions and functions in
    # loops: same values and tag counts as with every frame kept
    cases = {"ack": (programs.ack, oprog.ack_program, [(2, 3), (3, 3), (3, 4), (1, 0), (0, 5)]),
             "tak": (programs.tak, oprog.tak_program, [(7, 4, 2), (12, 8, 4), (1, 2, 3), (14, 8, 3)]),
             "loop_of_calls": (programs.loop_of_calls, oprog.loop_of_calls_program, [(9,), (1,), (14,)]),
             "nested_loop": (programs.nested_loop, oprog.nested_loop_program, [(12,), (0,), (40,)]),
             "loop_in_function": (programs.loop_in_function, oprog.loop_in_function_program, [(10,), (3,), (25,)])}
    gpu_prog, oracle_prog, args = cases[name]
    n_args = len(args[0])
    it = oracle.Interpreter(oracle.transform(oracle_prog()))
    want = it.run({("in", k): [a[k] for a in args] for k in range(n_args)}, len(args))[("out", 0)]
    total = len(it.tags) + len(it.iter_tags)
    fns, r = gpu_prog()
    st, kept, out_kept = _run(fns, r, args, n_args, total + 8, stats_level=1)
    st, stats, out = _run(fns, r, args, n_args, total + 8)
    assert out == out_kept == want
    assert stats.n_tags == kept.n_tags == total and stats.max_tag_depth == kept.max_tag_depth == it.max_tag_len
    assert stats.frames_reclaimed == 1 and kept.frames_reclaimed == 0
    assert stats.peak_frames <= kept.peak_frames
