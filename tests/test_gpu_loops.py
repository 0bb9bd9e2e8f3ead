"""GPU parity, tagged iteration (Section 2.3: Enter, Next, Exit) on the same frames as call labels
(Section 5.1): while-loops, a loop in a loop, calls from a loop body, a loop in a recursive
function and a loop that is not entered.  Values, tag counts (function invocations plus loop
iterations), tag depth and per-node firing counts against the oracle, bit-exact, through every
step kernel of the library."""
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
import oracle  # noqa: E402
from oracle import programs as oprog  # noqa: E402
from gpu_util import DEV, fire_counts  # noqa: E402

CASES = {
    "sum_loop": (programs.sum_loop, oprog.sum_loop_program, [(n,) for n in (0, 1, 2, 7, 40, 300, 3, 0, 129)]),
    "fib_loop": (programs.fib_loop, oprog.fib_loop_program, [(n,) for n in range(0, 91, 6)]),
    "gcd_loop": (programs.gcd_loop, oprog.gcd_loop_program,
                 [(a, b) for a in (1, 2, 9, 12, 35, 64, 1071) for b in (1, 3, 12, 18, 49, 462)]),
    "nested_loop": (programs.nested_loop, oprog.nested_loop_program, [(n,) for n in (0, 1, 2, 5, 17, 30)]),
    "loop_of_calls": (programs.loop_of_calls, oprog.loop_of_calls_program, [(n,) for n in (0, 1, 2, 3, 9, 14)]),
    "loop_in_function": (programs.loop_in_function, oprog.loop_in_function_program, [(n,) for n in (0, 1, 2, 6, 25, 0, 40)]),
}

MODES = {"generated": {}, "interpreter": {"TDF_NO_JIT": "1"},
         "grid_kernel_only": {"TDF_SMALL_LIMIT": "1"}, "grid_kernel_device_scope": {"TDF_SMALL_LIMIT": "1", "TDF_NO_DIE_LOCAL": "1"},
         "single_workgroup_no_follow": {"TDF_SMALL_LIMIT": "100000000", "TDF_FOLLOW_LIMIT": "0"}}


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("name", list(CASES))
def test_loops(name, mode, monkeypatch):
    for k, v in MODES[mode].items():
        monkeypatch.setenv(k, v)
    gpu_prog, oracle_prog, args = CASES[name]
    n_args = len(args[0])
    it = oracle.Interpreter(oracle.transform(oracle_prog()))
    want = it.run({("in", k): [a[k] for a in args] for k in range(n_args)}, len(args))[("out", 0)]
    n_tags = len(it.tags) + len(it.iter_tags)
    fns, r = gpu_prog()
    g = tdf.graph_build(fns, r)
    t_args = torch.tensor(args, dtype=torch.int64, device=DEV).reshape(-1)
    inp = tdf.make_inputs(len(args), args=t_args, n_args=n_args, max_tags=n_tags + 8)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((len(args),), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out)
    assert out.cpu().tolist() == want
    assert stats.n_tags == n_tags
    assert stats.max_tag_depth == it.max_tag_len
    assert fire_counts(g, stats) == {k: v for k, v in it.count_by_op().items() if k != "const"}


def test_a_batch_of_loops_with_very_different_trip_counts():
    # 4096 instances on eight machines; trip counts from 1 to 5001
    ns = [(7 * b) % 5001 for b in range(4096)]
    fns, r = programs.sum_loop()
    g = tdf.graph_build(fns, r)
    n_tags = sum(n + 1 for n in ns)
    t_args = torch.tensor(ns, dtype=torch.int64, device=DEV)      # make_inputs keeps the pointer, not the tensor
    inp = tdf.make_inputs(len(ns), args=t_args, n_args=1, max_tags=n_tags)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((len(ns),), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out)
    assert out.cpu().tolist() == [n * (n + 1) // 2 for n in ns]      # the closed form the oracle is pinned to
    assert stats.n_tags == n_tags and stats.max_tag_depth == 1


def test_workload_6_at_full_size():
    # the benchmark's loop workload as the benchmark launches it: every output against math.gcd,
    # the tag count against the trip counts of subtractive Euclid counted here
    import math
    from tdf_workloads import make_config
    c = make_config(6)
    ab = c["args"]
    fns, r = programs.gcd_loop()
    g = tdf.graph_build(fns, r)
    t_args = torch.tensor(ab, dtype=torch.int64, device=DEV).reshape(-1)
    inp = tdf.make_inputs(len(ab), args=t_args, n_args=2, max_tags=c["max_tags"], stats_level=0)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((len(ab),), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out)
    assert out.cpu().tolist() == [math.gcd(int(a), int(b)) for a, b in ab]
    trips = 0
    for a, b in ab.tolist():
        while a != b:
            a, b = (a, b - a) if a < b else (a - b, b)
            trips += 1
        trips += 1
    assert stats.n_tags == trips and stats.max_tag_depth == 1


def test_a_loop_that_never_leaves_is_reported():
    # while 0 < i: i = i + 1, started at 1: the table fills up, the run ends with an error status
    T = tdf
    loop = [(T.OP_IN, [], 0), (T.OP_CONST, [], 0), (T.OP_LT, [(1, 0), (0, 0)], 0), (T.OP_SWITCH, [(2, 0), (0, 0)], 0),
            (T.OP_CONST, [], 1), (T.OP_ADD, [(3, 0), (4, 0)], 0), (T.OP_NEXT, [(5, 0)], 0), (T.OP_OUT, [(3, 1)], 0)]
    res = [(T.OP_IN, [], 0), (T.OP_LOOP, [(0, 0)], 1), (T.OP_OUT, [(1, 0)], 0)]
    g = tdf.graph_build([("result", 1, res), ("W", 1, loop)], 0)
    t_args = torch.tensor([1, 5, 0, 1], dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(4, args=t_args, n_args=1, max_tags=3000)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((4,), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out, check=False)
    assert st == tdf.ERR_TABLE_FULL and stats.device_status == tdf.ERR_TABLE_FULL
    inp = tdf.make_inputs(4, args=t_args, n_args=1, max_tags=100000, step_limit=50)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out, check=False)
    assert st in (tdf.ERR_STEP_LIMIT, tdf.ERR_TABLE_FULL)
    t_args = torch.tensor([0, -3, 0, 0], dtype=torch.int64, device=DEV)      # these leave at once
    inp = tdf.make_inputs(4, args=t_args, n_args=1, max_tags=64)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out)
    assert out.cpu().tolist() == [0, -3, 0, 0] and stats.n_tags == 4
