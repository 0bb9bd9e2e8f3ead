#!/usr/bin/env python3
"""Benchmark of the tagged-dataflow hot path on one MI355X.

A step is one tdf_eval_grad (or tdf_eval for forward-only workloads) over the whole synthetic
batch: tag machine, cell firings level by level, and the reversed gradient schedule.  Inputs
are resident in HBM before the timed region.  Prints one JSON line.

  metric  tagged node firings/s: one body firing per call-context tag per pass
          (forward: n_tags per step; forward + gradient: 2 n_tags per step)
"""
import argparse
import json
import os
import sys
import time

# Two evaluations in flight use six streams (the caller's and the graph's two, each); HIP multiplexes
# streams onto GPU_MAX_HW_QUEUES hardware queues (4 unless set), and streams that share a queue run one
# after the other: which ones do would depend on the order in which they were created.  Eight queues give
# every stream its own.  (Read when the HIP runtime starts, so before torch is imported.)
if int(os.environ.get("GPU_MAX_HW_QUEUES", "4") or 4) < 8:
    os.environ["GPU_MAX_HW_QUEUES"] = "8"

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16 = 2.5e15      # dense bf16 MFMA, FLOP/s
PEAK_F32 = 157.3e12     # fp32 MFMA / vector
PEAK_HBM = 8.0e12       # B/s
COPY_BYTES = 1 << 30    # calibration copy: 1 GiB read + 1 GiB written

# HBM bytes per evaluation from the FETCH_SIZE / WRITE_SIZE counter passes (see
# profiles/bench_workload4_hbm_traffic.md), with the hash of the kernel source they were taken on:
# reported as `traffic` only while that source is unchanged.
MEASURED_TRAFFIC = {
    4: {"cells": ("paper_2410_20225_amd/csrc/cells.hip", "dda69c6299073a74", 1925062852.9),
        "steps": ("paper_2410_20225_amd/csrc/step_device.h", "2fd8b76edf21f18c", 337757515.5)},
}


def measured_traffic(cfg, which):
    import hashlib
    ent = MEASURED_TRAFFIC.get(cfg, {}).get(which)
    if not ent:
        return None
    path, sha, nbytes = ent
    try:
        now = hashlib.sha256(open(os.path.join(ROOT, path), "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    return nbytes if now == sha else None


def cpu_baseline(cfg, budget_trees, node_loss=False):
    """The oracle, as it stands, on the first trees of the same workload."""
    import numpy as np
    import oracle
    from oracle import programs as oprog
    from tdf_workloads import make_config
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas = 1
    if cfg == 1:
        it = oracle.Interpreter(oracle.transform(oprog.fib_program()))
        t0 = time.perf_counter()
        it.run({("in", 0): list(range(21))}, 21)
        dt = time.perf_counter() - t0
        return {"value": len(it.tags) / dt, "unit": "firings/s", "cores": 1, "kind": "oracle",
                "sample": "fib(0..20), one batch, %d tags, %.1f s" % (len(it.tags), dt)}
    if cfg == 6:
        ab = make_config(6)["args"][:budget_trees]
        it = oracle.Interpreter(oracle.transform(oprog.gcd_loop_program()))
        t0 = time.perf_counter()
        it.run({("in", 0): ab[:, 0].tolist(), ("in", 1): ab[:, 1].tolist()}, len(ab))
        dt = time.perf_counter() - t0
        return {"value": len(it.iter_tags) / dt, "unit": "firings/s", "cores": 1, "kind": "oracle",
                "sample": "first %d instances of the workload, %d loop iterations, %.1f s" % (len(ab), len(it.iter_tags), dt)}
    c = make_config(cfg)
    F = c["forest"].subset(range(budget_trees))
    grad = c["grad"]
    prog = oprog.tree_program(c["cell"], head=grad and not node_loss, node_loss=node_loss)
    if grad:
        prog = oracle.differentiate(prog)
    env = dict(left=F.left, right=F.right, token=F.token, E=c["E"], W=c["W"], b=c["b"], U=c["U"], u0=c["u0"])
    B = F.n_trees
    inputs = {("in", 0): F.roots.tolist()}
    if node_loss:     # the first trees' nodes are the first nodes of the forest
        env["node_label"] = c["node_labels"][:F.n_nodes]
        env["dnode"] = np.full(F.n_nodes, 1.0 / F.n_nodes)
        inputs[("gin", 0)] = list(np.zeros((B, c["H"] * (2 if c["cell"] == "lstm" else 1))))
    elif grad:
        inputs[("in", 1)] = c["labels"][:B].tolist()
        inputs[("gin", 0)] = [1.0 / B] * B
    it = oracle.Interpreter(oracle.transform(prog), env)
    t0 = time.perf_counter()
    it.run(inputs, B)
    dt = time.perf_counter() - t0
    firings = F.n_nodes * (2 if grad else 1)
    return {"value": firings / dt, "unit": "firings/s", "cores": blas, "kind": "oracle",
            "sample": "first %d trees of the workload (%d tags), %s, %.1f s; interpreter single-threaded, "
                      "BLAS threads %d of %d host cores" % (B, F.n_nodes, "forward+gradient" if grad else "forward",
                                                            dt, blas, len(os.sched_getaffinity(0)))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload 1..6 (default 4: TreeLSTM forward+gradient)")
    ap.add_argument("--node-loss", action="store_true",
                    help="workloads 3..5 with a loss term at every tree node instead of the root only")
    ap.add_argument("--scale", type=int, default=1,
                    help="workloads 2..5: this many times the workload's trees, same recipe (saturation sweep; the headline is --scale 1)")
    ap.add_argument("--fib", type=str, default="",
                    help="workload 1 with these arguments instead of 0..20, e.g. 30,31,32 (a large batch for the tag machine "
                         "alone; frames are kept, as in the counter runs of the same batch)")
    ap.add_argument("--pipeline", type=int, default=2,
                    help="tree workloads: after the headline measurement (one evaluation at a time) the same number of "
                         "evaluations with this many in flight, each from a host thread of its own with its own graph, "
                         "workspace and stream, reported as `pipelined` (1 = leave that out)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-trees", type=int, default=0, help="trees in the oracle's sample (0 = auto)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this engine has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2410_20225_amd import tdf, programs
    from tdf_workloads import make_config, CONFIG_NAMES

    cfg = a.config
    dev = "cuda:0"
    if a.node_loss and cfg not in (3, 4, 5):
        print("--node-loss applies to workloads 3, 4 and 5", file=sys.stderr)
        sys.exit(2)
    if cfg == 1:
        fns, r = programs.fib()
        g = tdf.graph_build(fns, r)
        ns = [int(x) for x in a.fib.split(",")] if a.fib else list(range(21))
        fibs = [0, 1]
        while len(fibs) < max(ns) + 2:
            fibs.append(fibs[-1] + fibs[-2])
        n_calls = sum(2 * fibs[n + 1] - 1 for n in ns)   # invocations of fib(n): 2 F(n+1) - 1
        args = torch.tensor(ns, dtype=torch.int64, device=dev)
        inp = tdf.make_inputs(len(ns), args=args, n_args=1, max_tags=n_calls, stats_level=1 if a.fib else 0)
        ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=dev)
        out = torch.zeros(len(ns), dtype=torch.int64, device=dev)
        step = lambda: tdf.eval(g, inp, ws, out_i64=out)[1]
        passes, dtype, flops_fwd, cell = 1, "int64", 0.0, None
    elif cfg == 6:
        c = make_config(6)
        fns, r = programs.gcd_loop()
        g = tdf.graph_build(fns, r)
        n_inst = len(c["args"])
        args = torch.tensor(c["args"], dtype=torch.int64, device=dev).reshape(-1)
        inp = tdf.make_inputs(n_inst, args=args, n_args=2, max_tags=c["max_tags"], stats_level=0)
        ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=dev)
        out = torch.zeros(n_inst, dtype=torch.int64, device=dev)
        step = lambda: tdf.eval(g, inp, ws, out_i64=out)[1]
        passes, dtype, flops_fwd, cell = 1, "int64", 0.0, None
    else:
        from paper_2410_20225_amd.harness import TreeRun
        if a.scale != 1:
            base_trees = {2: 256, 3: 1024, 4: 4096, 5: 128}[cfg]
            c = make_config(cfg, n_trees=base_trees * a.scale)
        else:
            c = make_config(cfg)
        grad = c["grad"]
        B = c["forest"].n_trees
        n_pipe = max(1, a.pipeline)
        if a.node_loss:
            runs = [TreeRun(c, head=False, grad=True, stats_level=0, node_labels=c["node_labels"]) for _ in range(n_pipe)]
            dnode = np.full(c["forest"].n_nodes, 1.0 / c["forest"].n_nodes)
            steps_of = [lambda r=r: r.run(None, dnode=dnode)[1] for r in runs]
        else:
            runs = [TreeRun(c, head=grad, grad=grad, stats_level=0) for _ in range(n_pipe)]
            dy = np.full(B, 1.0 / B)
            steps_of = [lambda r=r: r.run(dy if grad else None)[1] for r in runs]
        run, step = runs[0], steps_of[0]
        passes = 2 if grad else 1
        dtype = "bf16" if c["bf16"] else "f32"
        cell = c["cell"]
        rows = (5 if cell == "lstm" else 1) * c["H"]
        n_cell = int(c["forest"].n_leaves.sum()) - B
        flops_fwd = 2.0 * n_cell * rows * 2 * c["H"]

    # a plain device copy of known size, outside the timed region: what this machine's HBM delivers to a
    # simple kernel, and the reference that the FETCH_SIZE / WRITE_SIZE counter passes are scaled by
    copy_src = torch.empty(COPY_BYTES, dtype=torch.uint8, device=dev)
    copy_dst = torch.empty_like(copy_src)
    copy_dst.copy_(copy_src)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        copy_dst.copy_(copy_src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2.0 * COPY_BYTES / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del copy_src, copy_dst

    if cfg in (1, 6):
        steps_of = [step]
    import threading

    def timed(fns, n_steps):
        """Exactly n_steps evaluations, dealt in turn to one host thread per entry of fns (each with its own
        graph, workspace and stream).  Every evaluation is complete (control plane, data plane,
        gradients); with several in flight the library runs one's tag machine beside the previous one's
        data plane.  Returns (seconds, [(seconds from call to return, stats)])."""
        n = len(fns)
        streams = [torch.cuda.Stream() for _ in range(n)]   # (default priority)
        for fn, sm in zip(fns, streams):
            with torch.cuda.stream(sm):
                for _ in range(a.warmup):
                    fn()
        torch.cuda.synchronize()
        results = [[] for _ in range(n)]
        gate = threading.Barrier(n + 1)

        def worker(i):
            with torch.cuda.stream(streams[i]):
                gate.wait()
                for _ in range(i, n_steps, n):
                    t_call = time.perf_counter()
                    st_i = fns[i]()
                    results[i].append((time.perf_counter() - t_call, st_i))
                streams[i].synchronize()

        threads = [threading.Thread(target=worker, args=(i,)) for i in range(n)]
        for t in threads:
            t.start()
        gate.wait()
        t_begin = time.perf_counter()
        for t in threads:
            t.join()
        torch.cuda.synchronize()
        return time.perf_counter() - t_begin, [x for r in results for x in r]

    # the headline: one evaluation at a time
    dt, res = timed(steps_of[:1], a.steps)
    phase = np.zeros(len(tdf.PHASES))
    launches = np.zeros(len(tdf.PHASES))
    span_ms = 0.0
    for _, st in res:
        phase += np.array(list(st.phase_ms))
        launches += np.array(list(st.phase_launches))
        span_ms += st.fwd_cells_span_ms
    assert len(res) == a.steps
    latency_ms = 1e3 * float(np.mean([lat for lat, _ in res]))
    n_tags = int(st.n_tags)
    # and the same number of evaluations with several in flight (tree workloads)
    pipelined = None
    if len(steps_of) > 1:
        n_p = 3 * a.steps   # (more of them: the first tag machine and the last data plane have nothing beside them)
        dt_p, res_p = timed(steps_of, n_p)
        ph_p = np.zeros(len(tdf.PHASES))
        for _, st_p in res_p:
            ph_p += np.array(list(st_p.phase_ms))
        pipelined = {"evaluations_in_flight": len(steps_of), "steps": n_p, "ms_per_step": 1e3 * dt_p / n_p,
                     "value": n_tags * passes * n_p / dt_p, "unit": "firings/s",
                     "latency_ms": round(1e3 * float(np.mean([lat for lat, _ in res_p])), 4),
                     "phase_ms": {n: round(float(x) / n_p, 4) for n, x in zip(tdf.PHASES, ph_p)},
                     "how": "one host thread, graph, workspace and stream per evaluation in flight; the library runs an "
                            "evaluation's tag machine (which depends on the trees only) beside the previous evaluation's "
                            "data plane; every evaluation is complete"}
    # one more evaluation, outside the timed region, with the tag machines' step records switched on
    widest = []
    if cfg in (1, 6):
        inp.stats_level = 2
        ws = torch.empty(tdf.workspace_size(g, inp), dtype=torch.uint8, device=dev)
        st2 = step()
    else:
        run.inputs.stats_level = 2
        run.ws = torch.empty(tdf.workspace_size(run.graph, run.inputs, run.grad), dtype=torch.uint8, device=dev)
        st2 = step()
    for k in range(8):
        if st2.wide_step_frames[k] > 0 and st2.wide_step_us[k] > 0:
            fr, cr, us = int(st2.wide_step_frames[k]), int(st2.wide_step_created[k]), float(st2.wide_step_us[k])
            widest.append({"frames": fr, "tags_created": cr, "us": round(us, 2),
                           "useful_GBps": round(72.0 * max(cr, fr // 3) / (us * 1e-6) / 1e9, 2)})
    firings = n_tags * passes
    value = firings * a.steps / dt
    phase_ms = {n: round(float(p) / a.steps, 4) for n, p in zip(tdf.PHASES, phase)}

    # tag machine: algorithmic bytes per tag of matching + compaction (table entry and frame record
    # written, frame read on return, operand slot, arrival word, ready id, schedule-log entry): 72 B
    tag_bytes = 72.0 * n_tags
    tag_ms = phase[0] / a.steps
    roof_tags = {"bound": "hbm", "kernel": "tag machine step kernels (all steps)",
                 "achieved": tag_bytes / (tag_ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                 "launches_per_step": launches[0] / a.steps, "traffic": measured_traffic(cfg, "steps")}
    roof_tags["frac"] = roof_tags["achieved"] / roof_tags["peak"]
    roof_tags["copy_kernel_GBps"] = copy_gbps   # measured read + write rate of a plain 1 GiB device copy
    # the widest steps of a single tag machine (one of up to eight running side by side): frames that
    # received a token, tags the step created, duration; useful bytes = 72 B per tag created
    roof_tags["widest_steps_of_one_machine"] = widest
    if cfg in (1, 6):
        roof = roof_tags
    else:
        i_fwd, i_tail = tdf.PHASES.index("cells_fwd"), tdf.PHASES.index("tail_fwd")
        # forward cell kernels of all levels.  Where deep instances run beside the others the two groups of
        # launches overlap: the time is the span from the first launch to the last end over both streams
        ms = span_ms / a.steps if st.deep_split == 2 else (phase[i_fwd] + phase[i_tail]) / a.steps
        n_launch = (launches[i_fwd] + launches[i_tail]) / a.steps
        peak = PEAK_BF16 if dtype == "bf16" else PEAK_F32
        per_cell = 2.0 * rows * 2 * c["H"]
        roof = {"bound": "mfma", "kernel": "k_gemm + k_cell_small + k_tail_fwd <%s,%s_FWD> (forward cells of all levels)" % (dtype, cell.upper()),
                "achieved": flops_fwd / (ms * 1e-3) / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s",
                "launches_per_step": n_launch, "avg_launch_us": 1e3 * ms / max(n_launch, 1),
                "traffic": None if a.node_loss else measured_traffic(cfg, "cells")}
        # the same, split by level width: one launch per wide level, one launch for the whole narrow tail
        wide_ms, tail_ms = phase[i_fwd] / a.steps, phase[i_tail] / a.steps
        wide_cells = int(st.n_wide_cells)
        roof["wide_levels"] = {"levels": int(st.n_wide_waves), "cells": wide_cells, "ms": wide_ms,
                               "achieved": per_cell * wide_cells / max(wide_ms, 1e-9) / 1e9,
                               "frac": per_cell * wide_cells / max(wide_ms, 1e-9) / 1e9 / (peak / 1e12)}
        # the same kernels against the HBM roof: algorithmic bytes per cell (children's h, and c for
        # the LSTM, read; h, c and, in a gradient run, the five gate activations written)
        elt = 2 if dtype == "bf16" else 4
        H = c["H"]
        # (a leaf has no cell state: c is read only for the children that are cells, and every cell but an
        # instance's root is the child of exactly one cell)
        F = c["forest"]
        n_root_cells = int((F.left[F.roots] >= 0).sum())
        c_read = 4.0 * H * max(n_cell - n_root_cells, 0) / max(n_cell, 1)
        cell_bytes = 3 * H * elt + (4 * H + c_read + (5 * H * elt if grad or a.node_loss else 0) if cell == "lstm" else 0)
        roof["against_hbm"] = {"bytes_per_cell": cell_bytes, "flop_per_byte": per_cell / cell_bytes,
                               "machine_flop_per_byte": peak / PEAK_HBM,
                               "achieved": cell_bytes * n_cell / (ms * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                               "frac": cell_bytes * n_cell / (ms * 1e-3) / PEAK_HBM,
                               "wide_levels_frac": cell_bytes * wide_cells / max(wide_ms * 1e-3, 1e-12) / PEAK_HBM}
        roof["narrow_tail"] = {"levels": int(st.n_waves) - int(st.n_wide_waves), "cells": n_cell - wide_cells, "ms": tail_ms,
                               "achieved": per_cell * (n_cell - wide_cells) / max(tail_ms, 1e-9) / 1e9,
                               "frac": per_cell * (n_cell - wide_cells) / max(tail_ms, 1e-9) / 1e9 / (peak / 1e12)}
    roof["frac"] = roof["achieved"] / roof["peak"]

    rec = {"metric": "tagged node firings/sec at 1 GPU", "value": value, "unit": "firings/s", "n_gpus": 1,
           "steps": a.steps, "warmup": a.warmup, "ms_per_step": 1e3 * dt / a.steps, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
           "config": {"workload": "config %d: %s%s%s" % (cfg, CONFIG_NAMES[cfg], ", a loss term at every node" if a.node_loss else "",
                                                        ", arguments %s" % a.fib if (cfg == 1 and a.fib) else ""),
                      "n_tags": n_tags,
                      "firings_per_step": firings, "n_steps_tag_machine": int(st.n_steps),
                      "n_levels": int(st.n_waves), "max_tag_depth": int(st.max_tag_depth), "scale": a.scale,
                      "latency_ms": round(latency_ms, 4),   # mean time of one evaluation from call to return
                      # which way the evaluation took
                      "n_machines": int(st.n_machines), "die_local": int(st.die_local), "generated_step_kernels": int(st.generated),
                      "repeats": int(st.repeats), "tail_used": int(st.tail_used), "deep_split": int(st.deep_split),
                      "deep_cells": int(st.deep_cells), "frames_reclaimed": int(st.frames_reclaimed),
                      "peak_frames": int(st.peak_frames)},
           "phase_ms": phase_ms, "roofline": roof}
    if cfg not in (1, 6):
        rec["roofline_tag_machine"] = roof_tags
    if pipelined:
        rec["pipelined"] = pipelined
    if not a.no_cpu_baseline and not (cfg == 1 and a.fib):   # (the oracle does not finish a batch of that size)
        trees = a.cpu_trees or {1: 0, 2: 256, 3: 1024, 4: 1024, 5: 2, 6: 2048}[cfg]
        rec["cpu_baseline"] = cpu_baseline(cfg, trees, a.node_loss)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
