"""ctypes binding of include/tdf.h.  Same names as the C entry points, without the prefix.

Tensors are torch tensors on the GPU; the binding passes their data pointers and the current
HIP stream.  No computation happens here.
"""
import ctypes as C
import os

# torch ships its own copy of the HIP runtime; it must be loaded before libtdf.so so that the
# library binds to the same runtime (one context, shared streams) instead of loading a second one
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtdf.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError("libtdf.so is not built: run `python -m paper_2410_20225_amd.build` "
                      "(there is no fallback path)")
lib = C.CDLL(_LIB_PATH)

OK, ERR_BAD_PROGRAM, ERR_BAD_ARG, ERR_WORKSPACE, ERR_TABLE_FULL, ERR_STEP_LIMIT, ERR_DEVICE = 0, -1, -2, -3, -4, -5, -6
ERR_UNSUPPORTED = -7
F32, BF16 = 0, 1
(OP_IN, OP_OUT, OP_CONST, OP_ADD, OP_SUB, OP_MUL, OP_EQ, OP_LT, OP_ID, OP_SWITCH, OP_MERGE, OP_CALLFN,
 OP_TREE_ISLEAF, OP_TREE_LEFT, OP_TREE_RIGHT, OP_TREE_TOKEN, OP_EMBED, OP_RNN_CELL, OP_LSTM_CELL,
 OP_CE_HEAD, OP_LOOP, OP_NEXT, OP_CE_NODE) = range(23)
SNODE_MERGE_ENTRY, SNODE_CALL, SNODE_RETURN, SNODE_ENTER, SNODE_NEXT, SNODE_EXIT = 100, 101, 102, 103, 104, 105
MAX_INPUTS = 4
STATS_MAX_COUNTS = 256
PHASES = ("tags", "leaves", "levels", "cells_fwd", "head", "cells_bwd", "weight_grad", "embed_grad", "tail_fwd", "tail_bwd")


class Ref(C.Structure):
    _fields_ = [("node", C.c_int32), ("port", C.c_int32)]


class NodeDesc(C.Structure):
    _fields_ = [("op", C.c_int32), ("n_in", C.c_int32), ("inp", Ref * MAX_INPUTS), ("imm", C.c_int64)]


class FunctionDesc(C.Structure):
    _fields_ = [("name", C.c_char_p), ("n_params", C.c_int32), ("n_nodes", C.c_int32),
                ("nodes", C.POINTER(NodeDesc))]


class ProgramDesc(C.Structure):
    _fields_ = [("n_functions", C.c_int32), ("functions", C.POINTER(FunctionDesc)), ("result_fn", C.c_int32)]


class SNode(C.Structure):
    _fields_ = [("kind", C.c_int32), ("fn", C.c_int32), ("label", C.c_int32), ("param", C.c_int32),
                ("is_grad", C.c_int32), ("imm", C.c_int64)]


class SEdge(C.Structure):
    _fields_ = [("src", C.c_int32), ("src_port", C.c_int32), ("dst", C.c_int32), ("dst_slot", C.c_int32),
                ("is_control", C.c_int32)]


class GraphInfo(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_edges", C.c_int32), ("n_labels", C.c_int32),
                ("nodes", C.POINTER(SNode)), ("edges", C.POINTER(SEdge))]


class Inputs(C.Structure):
    _fields_ = [("n_instances", C.c_int32), ("n_args", C.c_int32), ("args", C.c_void_p),
                ("n_tree_nodes", C.c_int32), ("left", C.c_void_p), ("right", C.c_void_p), ("token", C.c_void_p),
                ("node_label", C.c_void_p),
                ("dtype", C.c_int32), ("hidden", C.c_int32), ("vocab", C.c_int32),
                ("E", C.c_void_p), ("W", C.c_void_p), ("b", C.c_void_p),
                ("n_classes", C.c_int32), ("U", C.c_void_p), ("u0", C.c_void_p),
                ("max_tags", C.c_int64), ("step_limit", C.c_int32), ("stats_level", C.c_int32)]


class Outputs(C.Structure):
    _fields_ = [("out_i64", C.c_void_p), ("out_f32", C.c_void_p), ("out_h", C.c_void_p), ("out_c", C.c_void_p),
                ("out_node_loss", C.c_void_p)]


class Seed(C.Structure):
    _fields_ = [("dy", C.c_void_p), ("dnode", C.c_void_p)]


class Grads(C.Structure):
    _fields_ = [("dW", C.c_void_p), ("db", C.c_void_p), ("dE", C.c_void_p)]


class Stats(C.Structure):
    _fields_ = [("n_tags", C.c_int64), ("n_steps", C.c_int64), ("n_tokens", C.c_int64),
                ("n_leaf_rows", C.c_int64), ("n_cell_rows", C.c_int64), ("n_waves", C.c_int64),
                ("n_wide_waves", C.c_int64), ("n_wide_cells", C.c_int64), ("deep_cells", C.c_int64),
                ("n_grad_firings", C.c_int64), ("n_grad_not_once", C.c_int64),
                ("max_tag_depth", C.c_int64), ("table_capacity", C.c_int64),
                ("max_probe", C.c_int64), ("peak_frames", C.c_int64), ("frames_reclaimed", C.c_int64), ("phase_ms", C.c_double * len(PHASES)), ("phase_launches", C.c_int64 * len(PHASES)),
                ("fwd_cells_span_ms", C.c_double), ("wide_step_frames", C.c_int64 * 8), ("wide_step_created", C.c_int64 * 8),
                ("wide_step_us", C.c_double * 8),
                ("device_status", C.c_int32), ("n_counts", C.c_int32),
                ("n_machines", C.c_int32), ("die_local", C.c_int32), ("generated", C.c_int32),
                ("repeats", C.c_int32), ("tail_used", C.c_int32), ("deep_split", C.c_int32),
                ("fire_count", C.c_int64 * STATS_MAX_COUNTS)]


def _declare(l):
    """Argument and result types of every entry point of a loaded library."""
    l.tdf_graph_build.argtypes = [C.POINTER(ProgramDesc), C.c_int, C.POINTER(C.c_void_p)]
    l.tdf_graph_build.restype = C.c_int
    l.tdf_graph_destroy.argtypes = [C.c_void_p]
    l.tdf_graph_destroy.restype = None
    l.tdf_graph_info.argtypes = [C.c_void_p, C.POINTER(GraphInfo)]
    l.tdf_graph_info.restype = C.c_int
    l.tdf_graph_precompile.argtypes = [C.c_void_p, C.c_char_p, C.POINTER(C.c_size_t)]
    l.tdf_graph_precompile.restype = C.c_int
    l.tdf_workspace_size.argtypes = [C.c_void_p, C.POINTER(Inputs), C.c_int, C.POINTER(C.c_size_t)]
    l.tdf_workspace_size.restype = C.c_int
    l.tdf_eval.argtypes = [C.c_void_p, C.POINTER(Inputs), C.POINTER(Outputs), C.c_void_p, C.c_size_t,
                             C.c_void_p, C.POINTER(Stats)]
    l.tdf_eval.restype = C.c_int
    l.tdf_eval_grad.argtypes = [C.c_void_p, C.POINTER(Inputs), C.POINTER(Seed), C.POINTER(Outputs),
                                  C.POINTER(Grads), C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(Stats)]
    l.tdf_eval_grad.restype = C.c_int
    l.tdf_graph_prepare.argtypes = [C.c_void_p]
    l.tdf_graph_prepare.restype = C.c_int
    l.tdf_eval_static.argtypes = [C.c_void_p, C.POINTER(Inputs), C.POINTER(Outputs), C.c_void_p, C.POINTER(Stats)]
    l.tdf_eval_static.restype = C.c_int
    l.tdf_last_error.argtypes = []
    l.tdf_last_error.restype = C.c_char_p
    return l


def load_library(path):
    """Another build of the library (the tests load the one with the test hooks compiled in); a graph
    built while it is current (use_library) keeps calling it."""
    return _declare(C.CDLL(path))


class use_library:
    """with use_library(l): graph_build and last_error go to `l` instead of the default library."""

    def __init__(self, l):
        self.l = l

    def __enter__(self):
        global lib
        self.prev, lib = lib, self.l
        return self.l

    def __exit__(self, *exc):
        global lib
        lib = self.prev


_declare(lib)
STATIC_WORKSPACE_BYTES = 64 << 20


class TdfError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib.tdf_last_error()
        super().__init__("%s failed with status %d: %s" % (where, status, msg.decode() if msg else ""))


def last_error():
    msg = lib.tdf_last_error()
    return msg.decode() if msg else ""


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Graph:
    """Owns a tdf_graph*; destroyed with the object."""

    def __init__(self, handle, library):
        self.handle = handle
        self.lib = library      # the library that built the graph serves every later call on it

    def __del__(self):
        if getattr(self, "handle", None) and getattr(self, "lib", None) is not None and C is not None:
            self.lib.tdf_graph_destroy(self.handle)
            self.handle = None


def graph_build(functions, result_fn, want_grad=False):
    """functions: list of (name, n_params, [(op, [(node, port), ...], imm), ...])."""
    keep = []
    fdescs = (FunctionDesc * len(functions))()
    for i, (name, n_params, nodes) in enumerate(functions):
        arr = (NodeDesc * max(len(nodes), 1))()
        for j, (op, ins, imm) in enumerate(nodes):
            arr[j].op, arr[j].n_in, arr[j].imm = op, len(ins), imm
            for k, (n, p) in enumerate(ins[:MAX_INPUTS]):
                arr[j].inp[k].node, arr[j].inp[k].port = n, p
        keep.append(arr)
        fdescs[i].name, fdescs[i].n_params, fdescs[i].n_nodes = name.encode(), n_params, len(nodes)
        fdescs[i].nodes = C.cast(arr, C.POINTER(NodeDesc))
    prog = ProgramDesc(len(functions), C.cast(fdescs, C.POINTER(FunctionDesc)), result_fn)
    handle = C.c_void_p()
    st = lib.tdf_graph_build(C.byref(prog), int(bool(want_grad)), C.byref(handle))
    if st != OK:
        raise TdfError(st, "tdf_graph_build")
    return Graph(handle, lib)


def graph_info(graph):
    info = GraphInfo()
    st = graph.lib.tdf_graph_info(graph.handle, C.byref(info))
    if st != OK:
        raise TdfError(st, "tdf_graph_info")
    nodes = [dict(kind=n.kind, fn=n.fn, label=n.label, param=n.param, is_grad=n.is_grad, imm=n.imm)
             for n in (info.nodes[i] for i in range(info.n_nodes))]
    edges = [dict(src=e.src, src_port=e.src_port, dst=e.dst, dst_slot=e.dst_slot, is_control=e.is_control)
             for e in (info.edges[i] for i in range(info.n_edges))]
    return dict(nodes=nodes, edges=edges, n_labels=info.n_labels)


def graph_precompile(graph, arch="gfx950"):
    """Compiles the specialised step kernels of `graph` for `arch`; returns the code size in bytes."""
    n = C.c_size_t()
    st = graph.lib.tdf_graph_precompile(graph.handle, arch.encode(), C.byref(n))
    if st != OK:
        raise TdfError(st, "tdf_graph_precompile")
    return n.value


def make_inputs(n_instances, args=None, n_args=0, left=None, right=None, token=None, dtype=F32, hidden=0,
                vocab=0, E=None, W=None, b=None, U=None, u0=None, n_classes=0, max_tags=0, step_limit=0, stats_level=1,
                node_label=None):
    n_tree = 0 if left is None else int(left.numel())
    return Inputs(n_instances, n_args, _ptr(args), n_tree, _ptr(left), _ptr(right), _ptr(token), _ptr(node_label), dtype, hidden,
                  vocab, _ptr(E), _ptr(W), _ptr(b), n_classes, _ptr(U), _ptr(u0), max_tags, step_limit, stats_level)


def workspace_size(graph, inputs, with_grad=False):
    n = C.c_size_t()
    st = graph.lib.tdf_workspace_size(graph.handle, C.byref(inputs), int(bool(with_grad)), C.byref(n))
    if st != OK:
        raise TdfError(st, "tdf_workspace_size")
    return n.value


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def eval(graph, inputs, workspace, out_i64=None, out_f32=None, out_h=None, out_c=None, out_node_loss=None, check=True):
    """Returns (status, Stats)."""
    outs = Outputs(_ptr(out_i64), _ptr(out_f32), _ptr(out_h), _ptr(out_c), _ptr(out_node_loss))
    stats = Stats()
    st = graph.lib.tdf_eval(graph.handle, C.byref(inputs), C.byref(outs), _ptr(workspace),
                      workspace.numel() * workspace.element_size(), _stream(), C.byref(stats))
    if check and st != OK:
        raise TdfError(st, "tdf_eval")
    return st, stats


def graph_prepare(graph):
    st = graph.lib.tdf_graph_prepare(graph.handle)
    if st != OK:
        raise TdfError(st, "tdf_graph_prepare")


def eval_static(graph, inputs, out_i64=None, out_f32=None, out_h=None, out_c=None, out_node_loss=None, check=True):
    """tdf_eval in the library's static workspace (no allocation).  Returns (status, Stats)."""
    outs = Outputs(_ptr(out_i64), _ptr(out_f32), _ptr(out_h), _ptr(out_c), _ptr(out_node_loss))
    stats = Stats()
    st = graph.lib.tdf_eval_static(graph.handle, C.byref(inputs), C.byref(outs), _stream(), C.byref(stats))
    if check and st != OK:
        raise TdfError(st, "tdf_eval_static")
    return st, stats


def eval_grad(graph, inputs, dy, workspace, dW, db, dE, out_f32=None, out_h=None, out_c=None, out_node_loss=None,
              dnode=None, check=True):
    outs = Outputs(None, _ptr(out_f32), _ptr(out_h), _ptr(out_c), _ptr(out_node_loss))
    seed = Seed(_ptr(dy), _ptr(dnode))
    grads = Grads(_ptr(dW), _ptr(db), _ptr(dE))
    stats = Stats()
    st = graph.lib.tdf_eval_grad(graph.handle, C.byref(inputs), C.byref(seed), C.byref(outs), C.byref(grads),
                           _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(),
                           C.byref(stats))
    if check and st != OK:
        raise TdfError(st, "tdf_eval_grad")
    return st, stats
