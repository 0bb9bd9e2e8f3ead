// Host-side graph object shared by graph_build.cpp, jit.cpp and eval.hip.
#pragma once
#include <stdint.h>

#include <mutex>
#include <string>
#include <vector>

#include "tdf.h"
#include "tdf_tables.h"

namespace tdf {

// ---- host graph object ----------------------------------------------------------------
struct Graph {
  std::vector<tdf_snode> snodes;
  std::vector<tdf_sedge> sedges;
  DevProgram prog;
  int n_labels = 0;
  int n_result_params = 0;
  int cell_kind = 0;        // 0 none, 1 RNN, 2 LSTM
  bool has_embed = false, has_head = false, has_node_loss = false, want_grad = false;
  int out_type = T_INT;     // type of result's output
};

void set_error(const std::string& msg);

// Run-time generated step kernels for one program (jit.cpp).  Returns false (and leaves the
// handles null) when the run-time compiler is unavailable, disabled (TDF_NO_JIT=1) or fails;
// the table interpreter is used then.
struct JitKernels {
  void* module = nullptr;   // hipModule_t
  void* step = nullptr;     // hipFunction_t of the grid-wide step kernel
  void* step_local = nullptr;   // ... and of its variant that keeps to one accelerator die
  void* small = nullptr;    // hipFunction_t of the single-workgroup kernel
  bool tried = false;
};
bool jit_compile(const DevProgram& P, JitKernels& out, std::string& log);
void jit_release(JitKernels& k);

}  // namespace tdf

struct tdf_graph {
  tdf::Graph g;
  tdf::JitKernels jit;
  bool die_local = true;    // tag machines keep to one accelerator die each (cleared if the GPU spreads them)
  uint32_t max_dies = 8;    // tag machines a batch is dealt to (set to 1 after a part of the table overflowed)
  void* events[2 * TDF_PHASE_COUNT] = {nullptr};   // hipEvent_t pairs, created on first use
  void* side_stream = nullptr;                     // hipStream_t for work beside the caller's stream
  void* fork_event = nullptr, *join_event = nullptr;   // embedding gradient beside the weight gradients
  void* fork_deep = nullptr, *join_deep = nullptr;     // deep instances beside the others
  void* sort_stream = nullptr;                     // hipStream_t for the embedding gradient's token sort
  void* fork_sort = nullptr, *join_sort = nullptr;     // ... which starts once the leaves are known
  void* leaves_done = nullptr;                     // the leaves' rows, written on that stream too
  // pinned host memory for what an evaluation reads back or sends (control blocks, level offsets,
  // barrier records, the firing tables): copies to and from pageable memory are staged and slower
  void* pinned = nullptr;
  size_t pinned_bytes = 0;
  std::mutex busy;          // one evaluation at a time uses the graph's streams, events and host buffer
  bool prepared = false;    // tdf_graph_prepare has run: kernels compiled, events and host buffers exist
  int prepared_device = -1;
  ~tdf_graph();
};
