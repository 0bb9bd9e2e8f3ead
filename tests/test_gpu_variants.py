"""GPU parity of the library's alternative code paths, each forced by its environment switch:
the table interpreter instead of generated step kernels, grid-wide steps synchronised through
memory instead of one die's L2, every level through the tiled GEMM or through the small-level
kernel, every step through the grid-wide kernel (on eight machines and on one) or through the
single-workgroup kernel, the repetition of a run whose die-private kernels did not keep to their
dies (the host is told they did not: that switch exists only in the library's build for the tests,
libtdf_hooks.so, which these two cases load), and steps in which no lane goes on with the frame it
created.  Every case asserts through tdf_stats that the requested path is the one that ran.  Same
bars as the main parity tests: integers and counts bit-exact, bf16 within rel 2e-2 (Frobenius)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
import oracle  # noqa: E402
from oracle import programs as oprog  # noqa: E402
from tdf_workloads import make_config  # noqa: E402
from gpu_util import DEV, TreeRun, run_oracle_tree, rel_fro, fire_counts  # noqa: E402

VARIANTS = [{"TDF_NO_JIT": "1"}, {"TDF_NO_DIE_LOCAL": "1"}, {"TDF_NO_JIT": "1", "TDF_NO_DIE_LOCAL": "1"},
            {"TDF_SMALL_LEVEL": "0"}, {"TDF_SMALL_LEVEL": "100000000"},
            {"TDF_SMALL_LIMIT": "1"}, {"TDF_SMALL_LIMIT": "1", "TDF_DIES": "1"}, {"TDF_SMALL_LIMIT": "100000000"},
            {"TDF_TEST_MIXED_DIES": "1"}, {"TDF_TEST_MIXED_DIES": "2"},
            {"TDF_FOLLOW_LIMIT": "0"},
            {"TDF_SMALL_LEVEL": "0", "TDF_TEST_WIDE_OFFSETS": "1"}]
IDS = ["interpreter", "device_scope", "interpreter_device_scope", "tiled_gemm_only", "small_level_only",
       "grid_kernel_only", "grid_kernel_only_one_machine", "single_workgroup_only",
       "repeat_after_machines_left_their_dies", "repeat_after_tail_left_its_dies",
       "no_follow", "tiled_gemm_with_64_bit_offsets"]


@pytest.fixture(scope="module")
def lstm_case():
    # 1500 trees: the first steps touch more than 1024 frames, so the grid-wide kernel runs too
    c = make_config(4, n_trees=1500, max_leaves=20, hidden=96, vocab=500)
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    return c, dy, run_oracle_tree(c, head=True, grad=True, dy=dy)


@pytest.fixture(scope="module")
def hooks_library():
    import os
    path = os.path.join(os.path.dirname(tdf.__file__), "libtdf_hooks.so")
    assert os.path.exists(path), "libtdf_hooks.so is not built: run `python -m paper_2410_20225_amd.build`"
    return tdf.load_library(path)


@pytest.mark.parametrize("env", VARIANTS, ids=IDS)
def test_treelstm_variants(env, lstm_case, hooks_library, monkeypatch):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    c, dy, ref = lstm_case
    if any(k.startswith("TDF_TEST_") for k in env):   # switches that only the build for the tests reads
        with tdf.use_library(hooks_library):
            run = TreeRun(c, head=True, grad=True)
    else:
        run = TreeRun(c, head=True, grad=True)      # a fresh graph: the switches are read per graph / per call
    st, stats = run.run(dy)
    assert stats.n_tags == c["forest"].n_nodes == len(ref["it"].tags)
    assert stats.max_tag_depth == ref["it"].max_tag_len
    assert rel_fro(run.out_f32.cpu().numpy(), np.array(ref["out"])) < 2e-2
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-2, name
    got = fire_counts(run.graph, stats)
    want = ref["it"].count_by_op()
    for k in ("merge_entry", "isleaf", "switch", "call_0", "call_1", "return_0", "return_1", "lstm_cell"):
        assert got[k] == want[k], k
    # the call reports which way it took: the variant that was asked for is the one that ran
    assert stats.generated == (0 if env.get("TDF_NO_JIT") == "1" else 1)
    assert stats.die_local == (0 if env.get("TDF_NO_DIE_LOCAL") == "1" or "TDF_TEST_MIXED_DIES" in env else 1)
    assert stats.n_machines == (1 if env.get("TDF_DIES") == "1" or stats.die_local == 0 else 8)
    assert stats.repeats == (1 if "TDF_TEST_MIXED_DIES" in env else 0)
    assert stats.n_grad_firings == stats.n_tags and stats.n_grad_not_once == 0
    if env.get("TDF_SMALL_LEVEL") == "0":
        assert stats.tail_used == 0 and stats.n_wide_waves == stats.n_waves


@pytest.mark.parametrize("env", VARIANTS[:3] + VARIANTS[-2:-1], ids=IDS[:3] + IDS[-2:-1])
def test_fib_variants(env, monkeypatch):
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    args = torch.arange(0, 21, dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(21, args=args, n_args=1, max_tags=57291)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((21,), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out)
    it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
    want = it.run({("in", 0): list(range(21))}, 21)[("out", 0)]
    assert out.cpu().tolist() == want
    assert stats.n_tags == len(it.tags)
    assert fire_counts(g, stats) == {k: v for k, v in it.count_by_op().items() if k != "const"}


@pytest.mark.parametrize("local", ["0", "1"], ids=["die_local", "device_scope"])
def test_grid_barrier_wait_is_bounded(local, lstm_case, monkeypatch):
    # A wait limit of zero makes every workgroup that has to wait at the grid barrier give up:
    # the call reports a device error (or finishes, if nobody had to wait), every kernel exits,
    # and the next call with the normal limit is correct.
    c, dy, ref = lstm_case
    monkeypatch.setenv("TDF_NO_DIE_LOCAL", local)
    monkeypatch.setenv("TDF_GRID_WAIT_MS", "0")
    run = TreeRun(c, head=True, grad=True)
    st, stats = run.run(dy, check=False)
    assert st in (tdf.OK, tdf.ERR_DEVICE)
    monkeypatch.delenv("TDF_GRID_WAIT_MS")
    st, stats = run.run(dy)
    assert st == tdf.OK and stats.n_tags == c["forest"].n_nodes
    assert rel_fro(run.dW.cpu().numpy(), ref["grads"]["dW"]) < 2e-2


def test_one_huge_instance_among_small_ones():
    # Eight trees dealt to eight machines, one of them holding nearly all tags: that machine's
    # part of the tag table fills up although the whole table has room.  The library repeats the
    # run with one machine; values and counts are the oracle's.
    from tdf_workloads import SplitMix64
    from tdf_workloads.trees import left_chain_tree, random_split_tree, build_forest
    c = make_config(3, n_trees=8, max_leaves=6, hidden=64, vocab=200)
    rng = SplitMix64(77)
    shapes = [left_chain_tree(300)] + [random_split_tree(3 + b % 3, rng.fork(b)) for b in range(7)]
    c["forest"] = build_forest(shapes, lambda n: rng.randint(0, 199, n))
    B = 8
    dy = np.full(B, 1.0 / B)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    run = TreeRun(c, head=True, grad=True)                 # max_tags = exactly the number of tags
    for _ in range(2):                                     # the second call starts with one machine
        st, stats = run.run(dy)
        assert stats.n_tags == c["forest"].n_nodes == len(ref["it"].tags)
        assert stats.max_tag_depth == ref["it"].max_tag_len
        assert rel_fro(run.out_f32.cpu().numpy(), np.array(ref["out"])) < 2e-2
        for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
            assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-2, name


@pytest.mark.parametrize("follow", ["default", "0"])
def test_chains_leaning_either_way(follow, monkeypatch):
    # Chains deeper than one lane follows in a step (256), leaning left (the first call of a frame
    # is the deep one) and right (the second is), next to bushy trees.
    if follow != "default":
        monkeypatch.setenv("TDF_FOLLOW_LIMIT", follow)
    from tdf_workloads import SplitMix64
    from tdf_workloads.trees import left_chain_tree, right_chain_tree, random_split_tree, build_forest
    c = make_config(3, n_trees=12, max_leaves=6, hidden=64, vocab=200)
    rng = SplitMix64(78)
    shapes = [left_chain_tree(300), right_chain_tree(290), left_chain_tree(2), right_chain_tree(3)]
    shapes += [random_split_tree(10 + 5 * b, rng.fork(b)) for b in range(8)]
    c["forest"] = build_forest(shapes, lambda n: rng.randint(0, 199, n))
    B = len(shapes)
    c["labels"] = rng.randint(0, 4, B)
    dy = np.full(B, 1.0 / B)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    run = TreeRun(c, head=True, grad=True)
    st, stats = run.run(dy)
    assert stats.n_tags == c["forest"].n_nodes == len(ref["it"].tags)
    assert stats.max_tag_depth == ref["it"].max_tag_len
    assert rel_fro(run.out_f32.cpu().numpy(), np.array(ref["out"])) < 2e-2
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-2, name
    got = fire_counts(run.graph, stats)
    want = ref["it"].count_by_op()
    for k in ("merge_entry", "isleaf", "switch", "call_0", "call_1", "return_0", "return_1"):
        assert got[k] == want[k], k


def test_evaluations_from_several_threads_take_turns(lstm_case):
    # Four host threads, each with its own graph, workspace and stream, evaluate at the same time.
    # The persistent kernels of one evaluation need the whole GPU, so the library lets one
    # evaluation run at a time; every call must succeed and give the oracle's result.
    import threading
    c, dy, ref = lstm_case
    n = 4
    streams = [torch.cuda.Stream() for _ in range(n)]
    runs, errors = [], []
    for s in streams:
        with torch.cuda.stream(s):
            runs.append(TreeRun(c, head=True, grad=True))

    def worker(i):
        try:
            with torch.cuda.stream(streams[i]):
                for _ in range(3):
                    st, stats = runs[i].run(dy)
                    assert st == tdf.OK and stats.n_tags == c["forest"].n_nodes
        except Exception as ex:          # noqa: BLE001 -- reported below, from the main thread
            errors.append(repr(ex))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(n)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for r in runs:
        assert rel_fro(r.dW.cpu().numpy(), ref["grads"]["dW"]) < 2e-2
        assert rel_fro(r.out_f32.cpu().numpy(), np.array(ref["out"])) < 2e-2


@pytest.mark.parametrize("wide", ["600", "5000", "0", None], ids=["above_600", "above_5000", "off", "default"])
@pytest.mark.parametrize("jit", [True, False], ids=["generated", "interpreter"])
def test_few_instances_use_the_whole_gpu_for_wide_steps(wide, jit, monkeypatch):
    # Three instances are dealt to two tag machines, which leaves six dies without one: a machine's
    # steps above a limit then run in the device-wide kernel, the others in the die-local and the
    # single-workgroup kernel.  fib(17), fib(20), fib(19) pass through all three several times.
    if wide is not None:
        monkeypatch.setenv("TDF_WIDE_LIMIT", wide)
    if not jit:
        monkeypatch.setenv("TDF_NO_JIT", "1")
    ns = [17, 20, 19]
    fns, r = programs.fib()
    g = tdf.graph_build(fns, r)
    t_args = torch.tensor(ns, dtype=torch.int64, device=DEV)
    inp = tdf.make_inputs(3, args=t_args, n_args=1, max_tags=41000)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((3,), -1, dtype=torch.int64, device=DEV)
    it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
    want = it.run({("in", 0): ns}, 3)[("out", 0)]
    for rep in range(2):
        st, stats = tdf.eval(g, inp, ws, out_i64=out)
        assert out.cpu().tolist() == want
        assert stats.n_tags == len(it.tags) and stats.max_tag_depth == it.max_tag_len
        got = fire_counts(g, stats)
        ref = it.count_by_op()
        for k in got:
            assert got[k] == ref[k], k


@pytest.mark.parametrize("wide", ["300", None], ids=["above_300", "default"])
def test_three_large_trees_with_wide_steps(wide, monkeypatch):
    if wide is not None:
        monkeypatch.setenv("TDF_WIDE_LIMIT", wide)
        monkeypatch.setenv("TDF_SMALL_LIMIT", "128")
    c = make_config(5, n_trees=3, max_leaves=512, hidden=64, vocab=300)   # a left chain and two complete trees
    B = c["forest"].n_trees
    dy = np.full(B, 1.0 / B)
    ref = run_oracle_tree(c, head=True, grad=True, dy=dy)
    run = TreeRun(c, head=True, grad=True)
    st, stats = run.run(dy)
    assert stats.n_tags == c["forest"].n_nodes == len(ref["it"].tags)
    assert rel_fro(run.out_f32.cpu().numpy(), np.array(ref["out"])) < 2e-2
    for name, t in (("dW", run.dW), ("db", run.db), ("dE", run.dE)):
        assert rel_fro(t.cpu().numpy(), ref["grads"][name]) < 2e-2, name
