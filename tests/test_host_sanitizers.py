"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer: the graph
compiler (validation, Section 3 transformation, gradient graph, firing tables) is built from the same
source with g++ -fsanitize=address,undefined and driven through the C ABI over every program of the
test-suite and the malformed ones.  No GPU code is involved (GPU sanitizers are not available)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
tdf = pytest.importorskip("paper_2410_20225_amd.tdf")
from paper_2410_20225_amd import programs  # noqa: E402

T = tdf
GOOD = [("fact", programs.fact, 0), ("fib", programs.fib, 0), ("ack", programs.ack, 0), ("tak", programs.tak, 0),
        ("treernn", lambda: programs.tree("rnn", False), 0), ("treernn_grad", lambda: programs.tree("rnn", True), 1),
        ("treelstm_grad", lambda: programs.tree("lstm", True), 1),
        ("treelstm_node_loss_grad", lambda: programs.tree("lstm", node_loss=True), 1),
        ("sum_loop", programs.sum_loop, 0), ("fib_loop", programs.fib_loop, 0), ("gcd_loop", programs.gcd_loop, 0),
        ("nested_loop", programs.nested_loop, 0), ("loop_of_calls", programs.loop_of_calls, 0),
        ("loop_in_function", programs.loop_in_function, 0)]
BAD = [("no_out", [("result", 0, [(T.OP_CONST, [], 1)])], 0, 0),
       ("undefined_callee", [("result", 1, [(T.OP_IN, [], 0), (T.OP_CALLFN, [(0, 0)], 3), (T.OP_OUT, [(1, 0)], 0)])], 0, 0),
       ("forward_reference", [("result", 1, [(T.OP_IN, [], 0), (T.OP_ADD, [(0, 0), (2, 0)], 0), (T.OP_OUT, [(1, 0)], 0)])], 0, 0),
       ("bad_operator", [("result", 1, [(T.OP_IN, [], 0), (99, [(0, 0)], 0), (T.OP_OUT, [(1, 0)], 0)])], 0, 0),
       ("negative_input", [("result", 1, [(T.OP_IN, [], 0), (T.OP_ID, [(-5, 0)], 0), (T.OP_OUT, [(1, 0)], 0)])], 0, 0),
       ("bad_port", [("result", 1, [(T.OP_IN, [], 0), (T.OP_ID, [(0, 7)], 0), (T.OP_OUT, [(1, 0)], 0)])], 0, 0),
       ("result_out_of_range", [("result", 1, [(T.OP_IN, [], 0), (T.OP_OUT, [(0, 0)], 0)])], 5, 0),
       ("huge_param_index", [("result", 1, [(T.OP_IN, [], 1 << 40), (T.OP_OUT, [(0, 0)], 0)])], 0, 0),
       ("grad_of_integers", None, 0, 1),
       ("unused_cell_grad", [("result", 1, [(T.OP_IN, [], 0), (T.OP_EMBED, [(0, 0)], 0), (T.OP_EMBED, [(0, 0)], 0),
                                            (T.OP_RNN_CELL, [(1, 0), (2, 0)], 0), (T.OP_OUT, [(1, 0)], 0)])], 0, 1)]


def _write(f, name, fns, result_fn, want_grad):
    f.write("program %s %d %d %d\n" % (name, want_grad, result_fn, len(fns)))
    for fname, n_params, nodes in fns:
        f.write("function %s %d %d\n" % (fname, n_params, len(nodes)))
        for op, ins, imm in nodes:
            f.write("node %d %d %d %s\n" % (op, imm, len(ins), " ".join("%d %d" % (n, p) for n, p in ins)))


def test_graph_compiler_is_clean_under_address_and_undefined_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if not gxx:
        pytest.skip("no host compiler")
    exe = str(tmp_path / "driver")
    csrc = os.path.join(ROOT, "paper_2410_20225_amd", "csrc")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
           "-I", os.path.join(ROOT, "include"), "-I", csrc, os.path.join(csrc, "graph_build.cpp"),
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    path = str(tmp_path / "programs.txt")
    with open(path, "w") as f:
        for name, prog, grad in GOOD:
            fns, r = prog()
            _write(f, name, fns, r, grad)
        for name, fns, r, grad in BAD:
            if fns is None:
                fns, r = programs.fib()
            _write(f, name, fns, r, grad)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe, path], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "Sanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-4000:]
    lines = dict(l.split(" ", 1) for l in res.stdout.strip().splitlines())
    for name, _, _ in GOOD:
        assert lines[name].startswith("0 nodes"), (name, lines[name])
    for name, _, _, _ in BAD:
        assert lines[name].startswith("%d " % tdf.ERR_BAD_PROGRAM), (name, lines[name])
    # the same static graph as the library proper builds (node and edge counts of the paper's example)
    info = tdf.graph_info(tdf.graph_build(*programs.fact()))
    assert lines["fact"].startswith("0 nodes %d edges %d labels %d" % (len(info["nodes"]), len(info["edges"]), info["n_labels"]))
