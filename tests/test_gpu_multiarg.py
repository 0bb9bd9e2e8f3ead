"""GPU parity, recursion with several parameters per call (Ackermann: two Call_i nodes insert one
tag, a call's argument is another call's result; Takeuchi: three parameters, three nested calls):
values, tag counts, tag depth and per-node firing counts against the oracle, bit-exact, through
every step kernel of the library."""
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2410_20225_amd import tdf, programs  # noqa: E402
import oracle  # noqa: E402
from oracle import programs as oprog  # noqa: E402
from gpu_util import DEV, fire_counts  # noqa: E402

CASES = {
    "ack": (programs.ack, oprog.ack_program, [(0, 0), (1, 2), (2, 3), (3, 3), (3, 4), (2, 0), (0, 7), (3, 1), (1, 0)]),
    "tak": (programs.tak, oprog.tak_program, [(7, 4, 2), (12, 8, 4), (1, 2, 3), (9, 5, 1), (14, 8, 3), (3, 2, 1)]),
}


MODES = {"generated": {}, "interpreter": {"TDF_NO_JIT": "1"},
         "grid_kernel_only": {"TDF_SMALL_LIMIT": "1"}, "grid_kernel_device_scope": {"TDF_SMALL_LIMIT": "1", "TDF_NO_DIE_LOCAL": "1"},
         "single_workgroup_only": {"TDF_SMALL_LIMIT": "100000000"}}


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("name", ["ack", "tak"])
def test_multi_parameter_recursion(name, mode, monkeypatch):
    # frames of these programs receive their arguments in different steps and are swept in between:
    # every step kernel must see what another compute unit wrote into a frame it has read before
    for k, v in MODES[mode].items():
        monkeypatch.setenv(k, v)
    gpu_prog, oracle_prog, args = CASES[name]
    n_args = len(args[0])
    it = oracle.Interpreter(oracle.transform(oracle_prog()))
    want = it.run({("in", k): [a[k] for a in args] for k in range(n_args)}, len(args))[("out", 0)]
    fns, r = gpu_prog()
    g = tdf.graph_build(fns, r)
    t_args = torch.tensor(args, dtype=torch.int64, device=DEV).reshape(-1)
    inp = tdf.make_inputs(len(args), args=t_args, n_args=n_args, max_tags=len(it.tags) + 8)
    ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=DEV)
    out = torch.full((len(args),), -1, dtype=torch.int64, device=DEV)
    st, stats = tdf.eval(g, inp, ws, out_i64=out)
    assert out.cpu().tolist() == want
    assert stats.n_tags == len(it.tags)
    assert stats.max_tag_depth == it.max_tag_len
    assert fire_counts(g, stats) == {k: v for k, v in it.count_by_op().items() if k != "const"}
