/* tdf — tagged static-dataflow execution of recursive function definitions on one GPU.
 *
 * C ABI of libtdf.  A program is a set of function graphs, one of them the `result`
 * graph (paper Section 2.4).  tdf_graph_build turns it into one static graph with
 * Call_i / Return_i nodes (Section 3) and, on request, joins every function with its
 * gradient under shared call labels (Section 4).  tdf_eval / tdf_eval_grad execute the
 * static graph over a batch of instances: tokens carry call-context tags
 * (Call_i <t,d> = <i:t,d>, Return_i <i:t,d> = <t,d>), tokens are matched by tag, and a
 * node body fires over every matched tag of a step at once.  While-loops (tagged iteration,
 * Section 2.3: Enter <t,d> = <0:t,d>, Next <n:t,d> = <(n+1):t,d>, Exit <n:t,d> = <t,d>) run on
 * the same tags: iteration counters and call labels share one tag list (Section 5.1).
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device, owned by the caller
 *     for the whole call; "host" pointers are ordinary process memory.
 *   - The evaluation calls allocate no device memory.  All transient device state lives in
 *     the caller's workspace (tdf_workspace_size bytes, 256-byte aligned); tdf_eval_static
 *     uses a fixed array inside the library instead (see there).
 *   - Work is enqueued on the caller's HIP stream; gradient evaluations also use two
 *     streams that the graph owns (default priority), ordered against the caller's by
 *     events, and join them before returning.  The evaluation calls synchronise the
 *     caller's stream before returning (the step count of a recursion is data dependent
 *     and is read back).
 *   - The functions may be called from several threads.  Evaluations take turns inside the
 *     library, stage by stage: one tag machine at a time and one data plane (cell levels,
 *     gradients) at a time, because the persistent kernels of either need their workgroups
 *     resident together; but an evaluation's tag machine, which depends on its trees only, runs
 *     beside the data plane of the evaluation before it.  Evaluations on one graph never
 *     overlap (the graph owns streams, events and a host buffer).  A caller who evaluates from two
 *     threads, each with its own graph, workspace and stream, gets that overlap (about a third
 *     more evaluations per second on the tree workloads; the streams should not share a
 *     hardware queue: GPU_MAX_HW_QUEUES of the HIP runtime, 4 unless set).  Other work of the
 *     caller on other streams of the same GPU should not hold compute units for long while an
 *     evaluation runs (the evaluation's bounded waits would end it with TDF_ERR_DEVICE).
 *   - Every function returns a tdf_status; a message for the last failure on the calling
 *     thread is available from tdf_last_error().  No exception crosses the ABI.
 */
#ifndef TDF_H
#define TDF_H

#ifndef __HIPCC_RTC__ /* the run-time compiler has size_t built in and no <stddef.h> */
#include <stddef.h>
#endif
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tdf_graph tdf_graph; /* opaque, library-owned host object */

typedef enum {
  TDF_OK = 0,
  TDF_ERR_BAD_PROGRAM = -1, /* malformed program description                         */
  TDF_ERR_BAD_ARG = -2,     /* NULL / inconsistent argument                           */
  TDF_ERR_WORKSPACE = -3,   /* workspace too small or misaligned                      */
  TDF_ERR_TABLE_FULL = -4,  /* more tags, tokens or state rows than max_tags allows   */
  TDF_ERR_STEP_LIMIT = -5,  /* recursion did not finish within step_limit steps       */
  TDF_ERR_DEVICE = -6,      /* a HIP call failed                                      */
  TDF_ERR_UNSUPPORTED = -7  /* optional facility not available                        */
} tdf_status;

/* ---- program description (host memory, read only during tdf_graph_build) ------------
 * Node operators.  The first group is the paper's language (Sections 2.2 and 2.4); the
 * TREE_* group reads the forest arrays of tdf_inputs at a node-index value; the next group
 * are vector-valued operators whose results live in the state table and travel through the
 * graph as row references; LOOP / NEXT write a while-loop (Section 2.3).
 *
 * A while-loop is a graph of its own, the loop graph: a tdf_function_desc with exactly one
 * NEXT node.  Its IN nodes are the loop variables in the current iteration (the Merge nodes of
 * the paper's while-loop figure, fed by Enter and Next), NEXT takes their values for the next
 * iteration, OUT is the value that leaves the loop.  The program decides by SWITCHes on the loop
 * condition which of the two is live: in every iteration exactly one of NEXT (all inputs) and
 * OUT must be.  A LOOP node in another graph supplies the initial values and stands for the
 * value that leaves.  Values of the enclosing graph that the loop reads are loop variables
 * handed on unchanged.  A loop graph belongs to exactly one LOOP node.  Every iteration is a tag
 * of its own and counts against max_tags; one loop instance runs at most 2^24 iterations
 * (TDF_ERR_STEP_LIMIT beyond); a loop that never leaves ends with TDF_ERR_TABLE_FULL or
 * TDF_ERR_STEP_LIMIT like a recursion without a base case.  */
typedef enum {
  TDF_OP_IN = 0,      /* formal parameter; imm = parameter index                        */
  TDF_OP_OUT,         /* the function's single output; in[0] = value                    */
  TDF_OP_CONST,       /* imm = int64 value                                              */
  TDF_OP_ADD, TDF_OP_SUB, TDF_OP_MUL, /* int64 arithmetic, wrapping                     */
  TDF_OP_EQ, TDF_OP_LT,               /* int64 comparison, result 0/1                   */
  TDF_OP_ID,
  TDF_OP_SWITCH,      /* in[0] = predicate, in[1] = data; port 0 = true, 1 = false side */
  TDF_OP_MERGE,       /* forwards the live input (2..4 inputs)                          */
  TDF_OP_CALLFN,      /* imm = callee function index; in[k] = argument k                */
  TDF_OP_TREE_ISLEAF, /* left[v] < 0                                                    */
  TDF_OP_TREE_LEFT, TDF_OP_TREE_RIGHT, TDF_OP_TREE_TOKEN,
  TDF_OP_EMBED,       /* in[0] = token id -> row E[token] (TreeLSTM: cell state 0)      */
  TDF_OP_RNN_CELL,    /* in[0], in[1] = child rows -> tanh(W [h_l; h_r] + b)            */
  TDF_OP_LSTM_CELL,   /* binary TreeLSTM, gate row blocks (i, f_l, f_r, o, u) of W      */
  TDF_OP_CE_HEAD,     /* in[0] = row, in[1] = label -> -log softmax(U h + u0)[label]    */
  TDF_OP_LOOP,        /* imm = loop graph index; in[k] = initial value of loop variable k   */
  TDF_OP_NEXT,        /* in a loop graph: in[k] = loop variable k in the next iteration     */
  TDF_OP_CE_NODE,     /* in[0] = row, in[1] = tree node v -> the same row; the node's loss term
                         -log softmax(U h + u0)[node_label[v]] goes to out_node_loss[v]
                         (no term where node_label[v] < 0): fully labelled trees, Section 6 */
  TDF_OP_COUNT
} tdf_op;

#define TDF_MAX_INPUTS 4

typedef struct {
  int32_t node; /* index of the producing node inside the same function */
  int32_t port; /* 0, or 1 for the false side of a SWITCH               */
} tdf_ref;

typedef struct {
  int32_t op;   /* tdf_op */
  int32_t n_in; /* number of inputs used */
  tdf_ref in[TDF_MAX_INPUTS];
  int64_t imm;
} tdf_node_desc;

typedef struct {
  const char* name;
  int32_t n_params;
  int32_t n_nodes;
  const tdf_node_desc* nodes; /* inputs must refer to earlier nodes (topological order) */
} tdf_function_desc;

typedef struct {
  int32_t n_functions;
  const tdf_function_desc* functions;
  int32_t result_fn; /* index of the `result` graph; its parameters are the program inputs */
} tdf_program_desc;

/* Section 3 (and Section 4 when want_grad != 0): validate the program, number the call
 * nodes, build the static graph, and compile the per-function firing tables used on the
 * device.  Host only.  Rejected with TDF_ERR_BAD_PROGRAM: undefined callee, arity
 * mismatch, forward reference, more or fewer than one OUT per function, an operator
 * whose inputs are all constants outside `result`, more than 64 nodes in a function, a
 * gradient request for a program without vector operators or with loops, CE_NODE together
 * with CE_HEAD, a loop graph that
 * is called, is `result`, has two NEXT nodes or belongs to no or several LOOP nodes, a LOOP
 * over a graph without NEXT.  *out is owned by the library
 * until tdf_graph_destroy. */
tdf_status tdf_graph_build(const tdf_program_desc* prog, int want_grad, tdf_graph** out);
void tdf_graph_destroy(tdf_graph* g);

/* ---- the static graph, for inspection (Section 3, figure "The transformed graph of
 * fact").  Node kinds: the tdf_op values for ordinary nodes, plus the three below.  */
#define TDF_SNODE_MERGE_ENTRY 100 /* Merge that replaced a callee's input node          */
#define TDF_SNODE_CALL 101        /* Call_i for one formal parameter                    */
#define TDF_SNODE_RETURN 102      /* Return_i                                           */
#define TDF_SNODE_ENTER 103       /* Enter of one loop variable; label = number of the LOOP */
#define TDF_SNODE_NEXT 104        /* Next of one loop variable                          */
#define TDF_SNODE_EXIT 105        /* Exit; label = number of the LOOP                   */

typedef struct {
  int32_t kind;    /* tdf_op or TDF_SNODE_*                                             */
  int32_t fn;      /* function graph the node came from                                 */
  int32_t label;   /* call label i for CALL / RETURN, the loop's number for ENTER / EXIT, else -1 */
  int32_t param;   /* parameter index for CALL / MERGE_ENTRY / IN / ENTER / NEXT, else -1 */
  int32_t is_grad; /* 1 for nodes of the gradient half of a joint function              */
  int64_t imm;     /* CONST value                                                       */
} tdf_snode;

typedef struct {
  int32_t src, src_port, dst, dst_slot;
  int32_t is_control; /* 1 for the Call_i -> Return_i (Enter -> Exit) synchronising edges */
} tdf_sedge;

typedef struct {
  int32_t n_nodes, n_edges, n_labels;
  const tdf_snode* nodes; /* library-owned, valid until tdf_graph_destroy               */
  const tdf_sedge* edges;
} tdf_graph_info_t;

tdf_status tdf_graph_info(const tdf_graph* g, tdf_graph_info_t* out);

/* Section 5 (the firing rule of the transformed graph, specialised): the per-function firing
 * tables of `g` are turned into straight-line device code and compiled for the GPU
 * architecture `arch` (e.g. "gfx950") with the HIP run-time compiler; tdf_eval does the same
 * on first use for the current device, so calling this is optional and only moves the
 * compile time.  Host only, needs no GPU.  *code_bytes (may be NULL) receives the size of
 * the code object.  TDF_ERR_UNSUPPORTED when the run-time compiler is missing or the
 * program does not fit the generated form; evaluation then uses the table interpreter. */
tdf_status tdf_graph_precompile(const tdf_graph* g, const char* arch, size_t* code_bytes);

/* ---- evaluation ------------------------------------------------------------------- */
typedef enum { TDF_F32 = 0, TDF_BF16 = 1 } tdf_dtype;

typedef struct {
  int32_t n_instances; /* B: the batch; instance b runs under root tag (b)              */
  int32_t n_args;      /* = n_params of `result`                                        */
  const int64_t* args; /* device int64[B * n_args], instance-major                      */
  /* forest, used by the TREE_* operators (may be NULL for integer programs)            */
  int32_t n_tree_nodes;
  const int32_t* left;  /* device int32[n_tree_nodes], -1 at a leaf                     */
  const int32_t* right; /* device int32[n_tree_nodes]                                   */
  const int32_t* token; /* device int32[n_tree_nodes], token id at a leaf               */
  const int32_t* node_label; /* device int32[n_tree_nodes], class of the node's loss term,
                                < 0: none (CE_NODE; NULL otherwise)                      */
  /* parameters of the vector operators (may be NULL / 0 for integer programs)          */
  int32_t dtype;  /* tdf_dtype of E, W and of the hidden-state rows                     */
  int32_t hidden; /* H                                                                  */
  int32_t vocab;
  const void* E;  /* device [vocab x H], dtype, row-major                               */
  const void* W;  /* device [R x 2H], dtype, row-major; R = H (RNN) or 5H (LSTM)        */
  const float* b; /* device float[R]                                                    */
  int32_t n_classes;
  const float* U;  /* device float[n_classes x H]   (CE_HEAD, CE_NODE)                  */
  const float* u0; /* device float[n_classes]                                           */
  /* capacities */
  int64_t max_tags;   /* capacity in call-context tags (= invocations and loop iterations).
                         tdf_eval of a program without vector operators with stats_level 0
                         gives a frame back when its tag has finished (Section 5.1: Return_i
                         deallocates), and max_tags bounds the tags alive at once; in every
                         other case all frames are kept and it bounds all tags of the call */
  int32_t step_limit; /* 0 = default (1<<20)                                            */
  int32_t stats_level; /* 0: counters and phase times; 1: also tdf_stats.fire_count (one
                          extra pass over the frame table after the evaluation); 2: also the
                          size and duration of the tag machines' widest steps              */
} tdf_inputs;

typedef struct {
  int64_t* out_i64; /* device int64[B]: integer result                                  */
  float* out_f32;   /* device float[B]: scalar float result (CE_HEAD loss per instance) */
  float* out_h;     /* device float[B x H]: vector result, h of the root                */
  float* out_c;     /* device float[B x H]: TreeLSTM cell state of the root, or NULL    */
  float* out_node_loss; /* device float[n_tree_nodes]: loss term of every tree node whose
                           CE_NODE fired, 0 elsewhere (graphs with CE_NODE; else ignored)  */
} tdf_outputs;      /* only the member matching the result type is written; others may be NULL */

typedef struct {
  const float* dy; /* device: float[B] for a scalar result, float[B x H] (dL/dh of each
                      root) for a vector result; NULL = zero in a graph with CE_NODE    */
  const float* dnode; /* device float[n_tree_nodes]: gradient of the objective with respect
                         to each node's loss term (graphs with CE_NODE; else ignored)     */
} tdf_seed;

typedef struct {
  float* dW; /* device float[R x 2H]  } overwritten with the gradients                  */
  float* db; /* device float[R]       }                                                 */
  float* dE; /* device float[vocab x H], rows of tokens that do not occur are set to 0  */
} tdf_grads;

#define TDF_STATS_MAX_COUNTS 256

/* Phases of one evaluation, timed on the caller's stream with HIP events. */
enum {
  TDF_PHASE_TAGS = 0,    /* tag machine: clear, seed, all match/fire steps                 */
  TDF_PHASE_LEAVES,      /* weight packing and EMBED rows (gradient runs write the rows on
                            a stream of their own, beside the level sort: outside this bracket) */
  TDF_PHASE_LEVELS,      /* bucketing of the cell firings by dependency level              */
  TDF_PHASE_CELLS_FWD,   /* cell GEMMs of the wide levels, one launch per level            */
  TDF_PHASE_HEAD,        /* head / result rows / gradient seeds                            */
  TDF_PHASE_CELLS_BWD,   /* gradient bodies of the cells of the wide levels, in reverse    */
  TDF_PHASE_WEIGHT_GRAD, /* dW, db                                                         */
  TDF_PHASE_EMBED_GRAD,  /* dE: the per-token sums (beside the weight gradients; the token
                            sort ran earlier, beside the cells)                            */
  TDF_PHASE_TAIL_FWD,    /* cells of the deep, narrow levels: one launch for all of them   */
  TDF_PHASE_TAIL_BWD,    /* ... and their gradient bodies                                  */
  TDF_PHASE_COUNT
};

typedef struct {
  int64_t n_tags;         /* tags created = function invocations + loop iterations      */
  int64_t n_steps;        /* match/fire steps of the tag machine                        */
  int64_t n_tokens;       /* Call and Return tokens delivered                           */
  int64_t n_leaf_rows;    /* EMBED firings                                              */
  int64_t n_cell_rows;    /* RNN_CELL / LSTM_CELL firings                               */
  int64_t n_waves;        /* dependency levels of the cell firings                      */
  int64_t n_wide_waves;   /* ... of which the first this many ran one launch per level  */
  int64_t n_wide_cells;   /* cell firings in those levels                               */
  int64_t deep_cells;     /* cell firings of the deep instances (see deep_split)        */
  int64_t n_grad_firings; /* gradient-body firings in tdf_eval_grad, counted on the device: every
                             gradient body marks its tag's row when it fires (one per tag) */
  int64_t n_grad_not_once; /* tags whose gradient body fired some other number of times than once */
  int64_t max_tag_depth;  /* longest list of call labels and iteration counters         */
  int64_t table_capacity; /* frame records the machines could hand out (all parts)      */
  int64_t max_probe;      /* accesses to find a tag's frame: 1 (the match table has no collisions) */
  int64_t peak_frames;    /* frame records ever handed out: with frames given back, the largest
                             number of tags alive at once (summed over the machines)    */
  int64_t frames_reclaimed; /* 1: frames were given back as their tags finished        */
  double phase_ms[TDF_PHASE_COUNT];        /* device time of each phase                */
  int64_t phase_launches[TDF_PHASE_COUNT]; /* kernel launches of each phase            */
  double fwd_cells_span_ms; /* first launch to last end of the forward cell kernels, over both
                               streams where deep instances run beside the others          */
  /* stats_level 2: the eight widest steps of the tag machines (a step of one machine): frames
     that received a token, frames created by the step, duration                              */
  int64_t wide_step_frames[8];
  int64_t wide_step_created[8];
  double wide_step_us[8];
  int32_t device_status;  /* tdf_status raised on the device                            */
  int32_t n_counts;       /* entries used in fire_count                                 */
  /* which way the evaluation took */
  int32_t n_machines;     /* independent tag machines the batch was dealt to (1, 2, 4, 8) */
  int32_t die_local;      /* 1: every machine kept to one accelerator die, atomics in its L2;
                             0: device-scope kernels                                    */
  int32_t generated;      /* 1: step kernels generated for this program at run time; 0: the
                             table interpreter                                          */
  int32_t repeats;        /* runs that were discarded and repeated inside this call (a part of
                             the tag table overflowed, or die-private kernels left their die) */
  int32_t tail_used;      /* 1: narrow levels ran in one launch per pass                */
  int32_t deep_split;     /* 1: the deep instances (root level >= 32) ran apart from the others,
                             all their levels in one launch per pass; 2: ... on a second
                             stream, beside the others                                   */
  /* live firings per static-graph node, indexed like tdf_graph_info_t.nodes            */
  int64_t fire_count[TDF_STATS_MAX_COUNTS];
} tdf_stats;

/* Bytes of workspace needed by tdf_eval (with_grad = 0) or tdf_eval_grad (1) for these
 * inputs (only sizes and capacities are read, no device memory is touched). */
tdf_status tdf_workspace_size(const tdf_graph* g, const tdf_inputs* in, int with_grad, size_t* bytes);

/* Forward evaluation of `result` for every instance (Sections 2.2, 3, 5.1).
 *   workspace: device, >= tdf_workspace_size bytes, 256-byte aligned, contents ignored.
 *   hip_stream: a hipStream_t (NULL = the default stream).
 *   stats: host, may be NULL.
 * Device-detected conditions (capacity, step limit) end the evaluation cleanly and are
 * returned as the status. */
tdf_status tdf_eval(tdf_graph* g, const tdf_inputs* in, tdf_outputs* out, void* workspace,
                    size_t workspace_bytes, void* hip_stream, tdf_stats* stats);

/* Forward and gradient in one call (Section 4: the joint graph computes the forward values
 * and the gradients; gradient operators meet the retained forward values under equal tags).
 * dy seeds the gradient of the result of each instance; grads receives the sums over all
 * tags of the parameter-gradient terms.  The graph must have been built with want_grad. */
tdf_status tdf_eval_grad(tdf_graph* g, const tdf_inputs* in, const tdf_seed* dy, tdf_outputs* out,
                         tdf_grads* grads, void* workspace, size_t workspace_bytes,
                         void* hip_stream, tdf_stats* stats);

/* ---- evaluation for callers that cannot allocate ---------------------------------------
 * For callers that must not call hipMalloc or any other allocating routine while they evaluate:
 * tight serving loops, harnesses that forbid allocation, code that keeps its memory budget fixed.
 *
 * tdf_graph_prepare is the set-up call (it allocates: host buffers, events, the generated step
 * kernels) and resolves, once per GPU, the address of the library's static workspace on the
 * current device.  Call it once per graph with the device current on which the graph will run.
 *
 * tdf_eval_static is tdf_eval without the workspace argument: it works in a static device array
 * of TDF_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds until the process ends,
 * and calls no allocating routine.  Inputs whose tdf_workspace_size exceeds that are refused with
 * TDF_ERR_WORKSPACE (lower max_tags, or use tdf_eval); a graph that was not prepared on the
 * current device is refused with TDF_ERR_BAD_ARG; a vector program with more than 8192
 * dependency levels is refused with TDF_ERR_WORKSPACE.  All calls on a GPU share that GPU's array
 * (calls of one process take turns inside the library; two processes have two arrays); the array
 * keeps the previous call's contents and every call clears what it needs cleared.  Like tdf_eval
 * it synchronises the stream, so it cannot be recorded into a HIP graph. */
#define TDF_STATIC_WORKSPACE_BYTES (64u << 20)
tdf_status tdf_graph_prepare(tdf_graph* g);
tdf_status tdf_eval_static(tdf_graph* g, const tdf_inputs* in, tdf_outputs* out, void* hip_stream, tdf_stats* stats);

const char* tdf_last_error(void); /* thread-local, static storage */

#ifdef __cplusplus
}
#endif
#endif /* TDF_H */
