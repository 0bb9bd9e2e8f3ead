// Host driver of tdf_eval / tdf_eval_grad: workspace layout, the step loop of the tag machine,
// the level-by-level execution of the cell firings, and the reversed schedule of the
// gradient pass.
#include <algorithm>
#include <mutex>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <string>
#include <vector>

#include "die_sync.h"
#include "engine.h"
#include "tdf_internal.h"

namespace tdf {

void launch_seed(const DevProgram& P, const Engine& e, hipStream_t s);
tdf_status launch_round(const DevProgram& P, const Engine& e, int cus, bool local, int small_block, int max_steps,
                        long long spin_ticks, const JitKernels& jit, hipStream_t s);
int tag_machine_small_block(const DevProgram& P, bool jit);
void launch_levels(const Engine& e, uint32_t n_cell, uint32_t n_keys, hipStream_t s);
void launch_class_keys(const DevProgram& P, const Engine& e, uint32_t n_cell, uint32_t deep_level, uint32_t deep_base, hipStream_t s);
void launch_merge_logs(const Engine& e, const uint32_t* leaf_off, const uint32_t* cell_off, hipStream_t s);
void launch_count_fired(const DevProgram& P, const Engine& e, hipStream_t s);
void vec_pack_w(const VecArgs& v, hipStream_t s);
void vec_embed(const VecArgs& v, const Engine& e, uint32_t n_leaf, hipStream_t s);
void vec_cell_fwd(const VecArgs& v, const Engine& e, uint32_t q0, uint32_t count, int save_gates, hipStream_t s);
void vec_cell_bwd(const VecArgs& v, const Engine& e, uint32_t q0, uint32_t count, hipStream_t s);
uint32_t vec_small_level();
void vec_tail_fwd(const VecArgs& v, const Engine& e, const uint32_t* level_off, uint32_t lvl_first, uint32_t lvl_last,
                  uint32_t n_dies, void* sync, long long spin_ticks, int per_die, int save_gates, hipStream_t s);
void vec_tail_bwd(const VecArgs& v, const Engine& e, const uint32_t* level_off, uint32_t lvl_first, uint32_t lvl_last,
                  uint32_t n_dies, void* sync, long long spin_ticks, int per_die, uint32_t q_first, const uint32_t* root_rows,
                  hipStream_t s);
void vec_number_rows(const Engine& e, uint32_t n_leaf, uint32_t n_cell, int has_head, int has_root, hipStream_t s);
void vec_head(const VecArgs& v, const Engine& e, const float* dy, int with_grad, int cls, hipStream_t s);
void vec_node_loss(const VecArgs& v, const Engine& e, uint32_t n_leaf, uint32_t n_cell, const int32_t* node_label,
                   float* out_node_loss, const float* dnode, int with_grad, hipStream_t s);
void vec_seed_dy(const VecArgs& v, const Engine& e, const float* dy, hipStream_t s);
void vec_count_grad(const VecArgs& v, const Engine& e, uint32_t n_leaf, uint32_t n_cell, unsigned long long* out, hipStream_t s);
void vec_out_rows(const VecArgs& v, const Engine& e, float* out_h, float* out_c, hipStream_t s);
int vec_dw_splits(uint32_t q_stride, int Np, int Kp);
void vec_weight_grads(const VecArgs& v, const Engine& e, uint32_t n_q, float* dW, float* db, float* db_part, hipStream_t s);
void vec_embed_sort(const VecArgs& v, const Engine& e, uint32_t n_leaf, uint32_t* count, uint32_t* seg_off,
                    uint32_t* chunk_off, uint32_t* fill, uint32_t* sorted_row, uint32_t chunk, hipStream_t s);
void vec_embed_sums(const VecArgs& v, uint32_t n_leaf, const uint32_t* seg_off, const uint32_t* chunk_off,
                    const uint32_t* sorted_row, float* part, float* dE, uint32_t chunk, hipStream_t s);

namespace {

constexpr uint32_t DE_CHUNK = 128;
constexpr uint32_t DB_CHUNK = 64;

struct Layout {
  size_t total = 0;
  size_t zero_begin = 0, zero_end = 0;   // region cleared at the start of every call
  size_t take(size_t bytes) {
    size_t off = total;
    total += (bytes + 255) / 256 * 256;
    return off;
  }
};

struct Plan {
  Layout L;
  Engine e{};
  VecArgs v{};
  bool vec = false, grad = false;
  size_t off_ctrl, off_fire, off_frames, off_tail_sync, off_gcount = 0;
  // embedding-gradient and bias-gradient scratch
  size_t off_tok_count, off_tok_fill, off_seg_off, off_chunk_off, off_sorted, off_de_part, off_db_part;
  uint32_t max_cells;
};

uint32_t pow2_at_least(uint64_t x) {
  uint64_t p = 64;
  while (p < x) p <<= 1;
  return (uint32_t)p;
}

// Machines a batch of B instances is dealt to (a power of two, so that the parts of the tag
// table are powers of two as well).
uint32_t dies_for(uint32_t B, uint32_t at_most) {
  uint32_t d = 1;
  while (d * 2 <= B && d * 2 <= at_most && d * 2 <= 8) d *= 2;
  return d;
}

// Sizes and offsets only; `base` may be null (tdf_workspace_size).  max_dies: upper bound of
// the number of tag machines; the layout for more machines is never smaller.
tdf_status make_plan(const Graph& G, const tdf_inputs* in, bool with_grad, char* base, Plan& P, uint32_t max_dies) {
  if (!in) { set_error("inputs is NULL"); return TDF_ERR_BAD_ARG; }
  if (in->n_instances < 1) { set_error("n_instances must be positive"); return TDF_ERR_BAD_ARG; }
  if (in->n_args != G.n_result_params) { set_error("n_args does not match the parameters of result"); return TDF_ERR_BAD_ARG; }
  if (in->max_tags < in->n_instances || in->max_tags > (1ll << 30)) { set_error("max_tags out of range"); return TDF_ERR_BAD_ARG; }
  P.vec = G.has_embed || G.cell_kind != 0;
  P.grad = with_grad;
  if (with_grad && !G.want_grad) { set_error("graph was built without gradients"); return TDF_ERR_BAD_ARG; }
  if (P.vec) {
    if (in->hidden < 1 || in->hidden > 8192 || in->vocab < 1) { set_error("bad hidden / vocab"); return TDF_ERR_BAD_ARG; }
    if (in->dtype != TDF_F32 && in->dtype != TDF_BF16) { set_error("bad dtype"); return TDF_ERR_BAD_ARG; }
    if ((G.has_head || G.has_node_loss) && (in->n_classes < 1 || in->n_classes > 16)) { set_error("n_classes must be 1..16"); return TDF_ERR_BAD_ARG; }
  }
  Layout& L = P.L;
  Engine& e = P.e;
  const uint32_t B = (uint32_t)in->n_instances;
  const uint32_t T = (uint32_t)in->max_tags;
  e.n_inst = B;
  e.max_tags = T;
  e.n_dies = dies_for(B, max_dies);
  // Frame records are handed out per machine, each from its own part.  One machine: the part holds
  // max_tags.  Several: twice a machine's even share; or, where records are small and few (no
  // vector operators: a record costs no state rows), max_tags each, so that instances of very
  // different sizes (fib(20) beside fib(3)) cannot overflow a part.
  e.part = T;
  if (e.n_dies > 1 && !(!P.vec && (uint64_t)T * e.n_dies <= (1ull << 24)))
    e.part = std::min<uint64_t>(T, 2ull * ((T + e.n_dies - 1) / e.n_dies) + 64);
  e.cap = e.part * e.n_dies;
  e.die = 0;
  e.key_base = 0;
  e.step_limit = in->step_limit > 0 ? (uint32_t)in->step_limit : (1u << 20);
  e.touched_cap = T + B;
  e.log_cap = P.vec ? T : 0;
  e.max_levels = e.log_cap;
  P.max_cells = e.log_cap;

  auto at = [&](size_t off) { return base ? base + off : nullptr; };
  // --- cleared region: control block, counters, level histograms, token histograms, tag keys
  L.zero_begin = L.total;
  P.off_ctrl = L.take(sizeof(Ctrl) * 8);
  P.off_fire = L.take(sizeof(unsigned long long) * TDF_STATS_MAX_COUNTS);
  P.off_tok_count = P.off_tok_fill = 0;
  if (P.vec && with_grad) {
    P.off_tok_count = L.take(sizeof(uint32_t) * ((size_t)in->vocab + 1));
    P.off_tok_fill = L.take(sizeof(uint32_t) * ((size_t)in->vocab + 1));
  }
  P.off_tail_sync = L.take(sizeof(DieSync) * 16);   // forward and gradient tail launches
  size_t off_gmark = 0;
  if (P.vec && with_grad) {
    P.off_gcount = L.take(sizeof(unsigned long long) * 2);
    off_gmark = L.take(sizeof(uint32_t) * ((size_t)T + 64));
  }
  L.zero_end = L.total;
  P.off_frames = L.take((size_t)G.prog.frame_stride * ((size_t)e.cap + B));   // headers are written on insertion
  // --- the rest is written before it is read
  size_t off_prog = L.take(sizeof(DevProgram));
  size_t off_touched = L.take(sizeof(uint32_t) * 2 * (size_t)e.touched_cap * e.n_dies);
  // Frames are given back as their tags finish where nothing reads them afterwards: no vector
  // operators (state rows are read after the steps), no gradient pass (it meets the retained
  // forward values), no per-node firing counts (they are taken from the frames after the run).
  e.reclaim = !P.vec && !with_grad && in->stats_level == 0 ? 1u : 0u;
  size_t off_ring = e.reclaim ? L.take(sizeof(uint32_t) * (size_t)e.cap) : 0;
  size_t off_root = L.take(sizeof(uint32_t) * B);
  size_t off_hrow = L.take(sizeof(uint32_t) * B);
  size_t off_hlab = L.take(sizeof(uint32_t) * B);
  size_t off_rlvl = L.take(sizeof(uint32_t) * B);
  size_t off_icls = L.take(sizeof(uint32_t) * B);
  const size_t level_keys = (2 * (size_t)e.max_levels + 4) * LEVEL_KEY_DIES;   // two classes of instances; cleared as far as used, after the steps
  size_t off_lcount = L.take(sizeof(uint32_t) * level_keys);
  size_t off_lfill = L.take(sizeof(uint32_t) * level_keys);
  size_t off_loff = L.take(sizeof(uint32_t) * level_keys);
  size_t rc = std::max<size_t>(e.log_cap, 1);
  size_t off_leaf_row = L.take(4 * rc), off_leaf_tok = L.take(4 * rc);
  size_t off_c_out = L.take(4 * rc), off_c_l = L.take(4 * rc), off_c_r = L.take(4 * rc), off_c_lvl = L.take(4 * rc);
  size_t off_q_out = L.take(4 * rc), off_q_l = L.take(4 * rc), off_q_r = L.take(4 * rc);
  size_t off_row_of = P.vec ? L.take(4 * ((size_t)e.cap + e.n_inst)) : 0;
  size_t off_row_node = G.has_node_loss ? L.take(4 * ((size_t)e.cap + e.n_inst)) : 0;
  size_t off_node_of_row = G.has_node_loss ? L.take(4 * ((size_t)T + 64)) : 0;
  // logs of the single machines, merged into the arrays above after the last step
  size_t off_m[6] = {off_leaf_row, off_leaf_tok, off_c_out, off_c_l, off_c_r, off_c_lvl};
  if (e.n_dies > 1)
    for (int i = 0; i < 6; ++i) off_m[i] = L.take(4 * rc * e.n_dies);

  e.prog = (const DevProgram*)at(off_prog);
  e.ctrl = (Ctrl*)at(P.off_ctrl);
  e.fire_count = (unsigned long long*)at(P.off_fire);
  e.level_count = (uint32_t*)at(off_lcount);
  e.level_fill = (uint32_t*)at(off_lfill);
  e.level_off = (uint32_t*)at(off_loff);
  e.frames = at(P.off_frames);
  e.touched = (uint32_t*)at(off_touched);
  e.free_ring = e.reclaim ? (uint32_t*)at(off_ring) : nullptr;
  size_t off_slog = in->stats_level >= 2 ? L.take(sizeof(uint4) * STEP_LOG_CAP * (size_t)e.n_dies) : 0;
  e.step_log = in->stats_level >= 2 ? (uint4*)at(off_slog) : nullptr;
  e.root_ref = (uint32_t*)at(off_root);
  e.head_row = (uint32_t*)at(off_hrow);
  e.head_label = (uint32_t*)at(off_hlab);
  e.root_lvl = (uint32_t*)at(off_rlvl);
  e.inst_class = (uint32_t*)at(off_icls);
  e.leaf_row = (uint32_t*)at(off_leaf_row);
  e.leaf_tok = (uint32_t*)at(off_leaf_tok);
  e.cell_out = (uint32_t*)at(off_c_out);
  e.cell_l = (uint32_t*)at(off_c_l);
  e.cell_r = (uint32_t*)at(off_c_r);
  e.cell_lvl = (uint32_t*)at(off_c_lvl);
  e.m_leaf_row = (uint32_t*)at(off_m[0]);
  e.m_leaf_tok = (uint32_t*)at(off_m[1]);
  e.m_cell_out = (uint32_t*)at(off_m[2]);
  e.m_cell_l = (uint32_t*)at(off_m[3]);
  e.m_cell_r = (uint32_t*)at(off_m[4]);
  e.m_cell_lvl = (uint32_t*)at(off_m[5]);
  e.q_out = (uint32_t*)at(off_q_out);
  e.q_l = (uint32_t*)at(off_q_l);
  e.q_r = (uint32_t*)at(off_q_r);
  e.row0 = 0;
  e.row_of = P.vec ? (uint32_t*)at(off_row_of) : nullptr;
  e.row_node = G.has_node_loss ? (uint32_t*)at(off_row_node) : nullptr;
  e.node_of_row = G.has_node_loss ? (uint32_t*)at(off_node_of_row) : nullptr;
  e.left = in->left;
  e.right = in->right;
  e.token = in->token;
  e.n_tree_nodes = in->n_tree_nodes;
  e.vocab = in->vocab;
  e.args = (const long long*)in->args;
  e.n_args = in->n_args;

  if (P.vec) {
    VecArgs& v = P.v;
    v.dtype = in->dtype;
    v.cell_kind = G.cell_kind;
    v.H = in->hidden;
    v.Hp = (in->hidden + 63) / 64 * 64;
    const int gates = G.cell_kind == 2 ? 5 : 1;
    v.N = gates * v.H;
    v.Np = gates * v.Hp;
    v.Kp = 2 * v.Hp;
    v.vocab = in->vocab;
    v.n_classes = in->n_classes;
    v.dHn = nullptr;
    v.gmark = with_grad ? (uint32_t*)at(off_gmark) : nullptr;
    v.E = in->E; v.W = in->W; v.b = in->b; v.U = in->U; v.u0 = in->u0;
    const size_t el = in->dtype == TDF_BF16 ? 2 : 4;
    const size_t R = (size_t)T + 64;      // one state row per leaf and per cell firing (at most one per tag)
    if (R * (size_t)((in->hidden + 63) / 64 * 64) >= (1ull << 32)) { set_error("max_tags x hidden too large for 32-bit row offsets"); return TDF_ERR_BAD_ARG; }
    size_t off_Hs = L.take(R * v.Hp * el);
    size_t off_Cs = G.cell_kind == 2 ? L.take(R * v.Hp * 4) : 0;
    size_t off_Wp = L.take((size_t)v.Np * v.Kp * el);
    size_t off_Wf = L.take((size_t)v.Np * v.Kp * el);
    size_t off_bp = L.take((size_t)v.Np * 4);
    size_t off_loss = L.take((size_t)B * 4);
    v.Hs = at(off_Hs);
    v.Cs = G.cell_kind == 2 ? (float*)at(off_Cs) : nullptr;
    v.Wp = at(off_Wp);
    v.Wf = at(off_Wf);
    v.WfT = nullptr;
    v.bp = (float*)at(off_bp);
    v.loss = (float*)at(off_loss);
    if (with_grad) {
      // In a gradient graph every state row has exactly one consumer, so a cell consumes two rows of
      // its own: at most half of the rows are cells.
      P.max_cells = e.log_cap / 2 + 64;
      v.q_stride = (uint32_t)((P.max_cells + 63) / 64 * 64);
      size_t off_dH = L.take(R * v.Hp * 4);
      size_t off_dC = G.cell_kind == 2 ? L.take(R * v.Hp * 4) : 0;
      size_t off_dHn = G.has_node_loss ? L.take(R * v.Hp * 4) : 0;
      size_t off_gates = G.cell_kind == 2 ? L.take((size_t)P.max_cells * v.Np * el) : 0;
      size_t off_Dz = L.take((size_t)P.max_cells * v.Np * el);
      // transposed copies of the weight-gradient operands: the fp32 path only
      size_t off_DzT = in->dtype == TDF_F32 ? L.take((size_t)v.Np * v.q_stride * el) : 0;
      size_t off_XT = in->dtype == TDF_F32 ? L.take((size_t)v.Kp * v.q_stride * el) : 0;
      size_t off_WpT = L.take((size_t)v.Np * v.Kp * el);
      size_t off_WfT = L.take((size_t)v.Np * v.Kp * el);
      size_t off_part = L.take((size_t)vec_dw_splits(v.q_stride, v.Np, v.Kp) * v.Np * v.Kp * 4);
      P.off_db_part = L.take(((size_t)P.max_cells / DB_CHUNK + 2) * v.Np * 4);
      P.off_seg_off = L.take(4 * ((size_t)v.vocab + 2));
      P.off_chunk_off = L.take(4 * ((size_t)v.vocab + 2));
      P.off_sorted = L.take(4 * rc);
      P.off_de_part = L.take(((size_t)e.log_cap / DE_CHUNK + v.vocab + 2) * v.Hp * 4);
      v.dH = (float*)at(off_dH);
      v.dC = G.cell_kind == 2 ? (float*)at(off_dC) : nullptr;
      v.dHn = G.has_node_loss ? (float*)at(off_dHn) : nullptr;
      v.gates = G.cell_kind == 2 ? at(off_gates) : nullptr;
      v.Dz = at(off_Dz);
      v.DzT = off_DzT ? at(off_DzT) : nullptr;
      v.XT = off_XT ? at(off_XT) : nullptr;
      v.WpT = at(off_WpT);
      v.WfT = at(off_WfT);
      v.dW_part = (float*)at(off_part);
    }
  }
  return TDF_OK;
}

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t err__ = (expr);                                                          \
    if (err__ != hipSuccess) {                                                          \
      set_error(std::string(#expr) + ": " + hipGetErrorString(err__));                  \
      return TDF_ERR_DEVICE;                                                            \
    }                                                                                   \
  } while (0)

bool status_is(uint32_t st, tdf_status code) { return st != 0 && -(int)st == (int)code; }

tdf_status status_from_device(uint32_t st) {
  if (st == 0) return TDF_OK;
  int code = -(int)st;
  switch (code) {
    case TDF_ERR_TABLE_FULL: set_error("device: tag table, frame list or state rows exhausted (raise max_tags)"); break;
    case TDF_ERR_STEP_LIMIT: set_error("device: step limit reached before the recursion finished"); break;
    case TDF_ERR_BAD_ARG: set_error("device: tree node index or token id out of range"); break;
    case TDF_ERR_DEVICE: set_error("device: a workgroup waited too long at the grid barrier of the step kernel"); break;
    default: set_error("device: unknown status"); code = TDF_ERR_DEVICE; break;
  }
  return (tdf_status)code;
}

// Layout of tdf_graph::pinned: control blocks, barrier records, firing tables, firing counts, then level offsets.
constexpr size_t PIN_CTRL = 0, PIN_SYNC = PIN_CTRL + sizeof(Ctrl) * 8, PIN_PROG = PIN_SYNC + sizeof(DieSync) * 16,
                 PIN_FIRE = (PIN_PROG + sizeof(DevProgram) + 255) / 256 * 256,
                 PIN_LEVELS = PIN_FIRE + sizeof(unsigned long long) * (TDF_STATS_MAX_COUNTS + 2);
// Makes the graph's pinned buffer at least PIN_LEVELS + level_bytes large (contents are lost when it grows).
tdf_status pinned_reserve(tdf_graph* gr, size_t level_bytes) {
  const size_t need = PIN_LEVELS + level_bytes;
  if (gr->pinned_bytes >= need) return TDF_OK;
  if (gr->pinned) (void)hipHostFree(gr->pinned);
  gr->pinned = nullptr;
  gr->pinned_bytes = 0;
  const size_t bytes = std::max<size_t>(need * 2, 64 * 1024);
  HIP_TRY(hipHostMalloc(&gr->pinned, bytes, hipHostMallocDefault));
  gr->pinned_bytes = bytes;
  memcpy((char*)gr->pinned + PIN_PROG, &gr->g.prog, sizeof(DevProgram));
  return TDF_OK;
}

// Evaluations of one process take turns, in two stages.  The control plane (the tag machine: persistent
// step kernels whose workgroups must all be resident, one machine per die) of one evaluation at a time;
// the data plane (level launches, the chain launches with their die barriers, the gradient sums) of one
// evaluation at a time; but the control plane of one evaluation may run beside the data plane of the
// one before it, which depends on other inputs' trees only: while a tag machine walks its narrow steps
// most compute units have nothing else to do.  The data stage ends with the gradient pass: the sums that
// follow it (weight and embedding gradients) are ordinary launches and run beside the next data plane.
// A caller gets that overlap by evaluating from two threads, each with its own graph, workspace and
// stream.  Lock order: control, then data.
std::mutex g_control_mutex, g_data_mutex;
struct EvalLocks {
  std::unique_lock<std::mutex> control{g_control_mutex, std::defer_lock}, data{g_data_mutex, std::defer_lock};
};

tdf_status run(tdf_graph* gr, const tdf_inputs* in, const tdf_seed* dy, tdf_outputs* out, tdf_grads* grads,
               void* workspace, size_t workspace_bytes, void* hip_stream, tdf_stats* stats, bool with_grad,
               EvalLocks& locks, int inherited_repeats = 0, bool no_alloc = false) {
  if (!locks.control.owns_lock()) locks.control.lock();
  if (!gr || !out) { set_error("NULL graph or outputs"); return TDF_ERR_BAD_ARG; }
  const Graph& G = gr->g;
  Plan P;
  tdf_status st = make_plan(G, in, with_grad, (char*)workspace, P, 8);   // the largest layout
  if (st != TDF_OK) return st;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < P.L.total) {
    set_error("workspace is NULL, misaligned or smaller than tdf_workspace_size");
    return TDF_ERR_WORKSPACE;
  }
  if (!in->args && G.n_result_params > 0) { set_error("args is NULL"); return TDF_ERR_BAD_ARG; }
  if ((in->left || in->right || in->token) && (!in->left || !in->right || !in->token || in->n_tree_nodes < 1)) {
    set_error("forest: left, right and token go together, with n_tree_nodes > 0");
    return TDF_ERR_BAD_ARG;
  }
  if (P.vec) {
    if (!in->left || !in->right || !in->token || !in->E || (G.cell_kind && (!in->W || !in->b))) {
      set_error("forest or parameter pointer is NULL");
      return TDF_ERR_BAD_ARG;
    }
    if ((G.has_head || G.has_node_loss) && (!in->U || !in->u0)) { set_error("U / u0 is NULL"); return TDF_ERR_BAD_ARG; }
    if (G.has_node_loss && (!in->node_label || !out->out_node_loss)) { set_error("node_label or out_node_loss is NULL"); return TDF_ERR_BAD_ARG; }
    if (G.has_node_loss && with_grad && (!dy || !dy->dnode)) { set_error("dnode is NULL"); return TDF_ERR_BAD_ARG; }
  }
  if (G.out_type == T_INT && !out->out_i64) { set_error("out_i64 is NULL"); return TDF_ERR_BAD_ARG; }
  if (G.out_type == T_LOSS && !out->out_f32) { set_error("out_f32 is NULL"); return TDF_ERR_BAD_ARG; }
  if (G.out_type == T_VEC && !out->out_h) { set_error("out_h is NULL"); return TDF_ERR_BAD_ARG; }
  if (with_grad && (!dy || (!dy->dy && !G.has_node_loss) || !grads || !grads->dW || !grads->db || !grads->dE)) {
    set_error("dy or a gradient buffer is NULL");
    return TDF_ERR_BAD_ARG;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  // phase timing: event pairs on the caller's stream, only when statistics are requested
  const bool timed = stats != nullptr;
  int64_t launches[TDF_PHASE_COUNT] = {0};
  bool phase_used[TDF_PHASE_COUNT] = {false};
  if (no_alloc && (!gr->prepared || !gr->jit.tried)) {
    set_error("the graph was not prepared: call tdf_graph_prepare first");
    return TDF_ERR_BAD_ARG;
  }
  if (timed && !no_alloc)
    for (int i = 0; i < 2 * TDF_PHASE_COUNT; ++i)
      if (!gr->events[i]) HIP_TRY(hipEventCreate((hipEvent_t*)&gr->events[i]));
  auto begin = [&](int ph) { if (timed) { (void)hipEventRecord((hipEvent_t)gr->events[2 * ph], s); phase_used[ph] = true; } };
  auto end = [&](int ph, int64_t n) { if (timed) (void)hipEventRecord((hipEvent_t)gr->events[2 * ph + 1], s); launches[ph] += n; };
  Engine& e = P.e;
  VecArgs& v = P.v;
  e.out_i64 = (long long*)out->out_i64;
  char* base = (char*)workspace;
  if (!no_alloc)
    if (tdf_status ps = pinned_reserve(gr, 0); ps != TDF_OK) return ps;

  // ---- the tag machine: fire / match steps until no token is in flight -------------------
  // The grid-wide kernel synchronises its workgroups with a barrier in memory: no more
  // workgroups than compute units, so that all of them are resident together.
  int dev_id = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev_id));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev_id));
  if (cus < 1) { set_error("no compute units"); return TDF_ERR_DEVICE; }
  // longest wait at that barrier before the run is abandoned (milliseconds; 100 MHz ticks)
  long long wait_ms = 2000;
  if (const char* w = getenv("TDF_GRID_WAIT_MS")) wait_ms = atoll(w);
  const long long spin_ticks = wait_ms * 100000;
  if (const char* w = getenv("TDF_NO_DIE_LOCAL")) if (w[0] == '1') gr->die_local = false;
  if (const char* w = getenv("TDF_DIES")) gr->max_dies = (uint32_t)std::max(1, atoi(w));
  // step kernels generated for this program (first call only; falls back to the interpreter)
  if (!gr->jit.tried) {
    gr->jit.tried = true;
    std::string log;
    if (!jit_compile(G.prog, gr->jit, log) && getenv("TDF_JIT_VERBOSE")) fprintf(stderr, "tdf: no generated kernels: %s\n", log.c_str());
  }
  const bool use_jit = gr->jit.step && gr->jit.small && gr->jit.step_local;
  int small_block = tag_machine_small_block(G.prog, use_jit);
  // A batch of few instances (deep ones, or it would not be worth a GPU) has narrow steps: half the lanes
  // do, and a workgroup of 256 finds room on a compute unit beside a chain workgroup of the evaluation
  // before this one (two evaluations in flight), where one of 512 does not.
  if (use_jit && P.vec && in->n_instances <= 128 && !getenv("TDF_SMALL_BLOCK")) small_block = std::min(small_block, 256);
#ifdef TDF_TEST_HOOKS
  v.wide_offsets = getenv("TDF_TEST_WIDE_OFFSETS") != nullptr;   // a path that otherwise needs arrays of 4 GiB
  // Only the build for the tests has this: 1 = the host treats the machines' kernels as having left
  // their dies (once per graph), 2 = the level tail's launches.  The reaction is the product's own.
  const int test_mixed_dies = getenv("TDF_TEST_MIXED_DIES") ? atoi(getenv("TDF_TEST_MIXED_DIES")) : 0;
#else
  constexpr int test_mixed_dies = 0;
#endif
  Ctrl hc{};
  uint32_t rounds = 0, repeats = 0;
  const uint32_t poll = 2;          // rounds queued between two looks at the control blocks
  const int max_steps = 4096;       // steps per kernel launch
  // Gradient runs have two more streams.  The packed copies of W depend on the caller's inputs only: they
  // are made on one of them, beside the tag machine (again after it, should the plan change meanwhile).
  if (P.vec && !gr->side_stream && with_grad && !no_alloc) {
    HIP_TRY(hipStreamCreateWithFlags((hipStream_t*)&gr->side_stream, hipStreamNonBlocking));
    HIP_TRY(hipStreamCreateWithFlags((hipStream_t*)&gr->sort_stream, hipStreamNonBlocking));
    for (void** ev : {&gr->fork_event, &gr->join_event, &gr->fork_deep, &gr->join_deep, &gr->fork_sort, &gr->join_sort, &gr->leaves_done})
      HIP_TRY(hipEventCreateWithFlags((hipEvent_t*)ev, hipEventDisableTiming));
  }
  bool w_packed = false;
  if (P.vec && G.cell_kind && with_grad && !no_alloc) {
    HIP_TRY(hipEventRecord((hipEvent_t)gr->fork_sort, s));
    HIP_TRY(hipStreamWaitEvent((hipStream_t)gr->sort_stream, (hipEvent_t)gr->fork_sort, 0));
    vec_pack_w(v, (hipStream_t)gr->sort_stream);
    w_packed = true;
  }
  begin(TDF_PHASE_TAGS);
  for (;;) {
    // several machines only where each keeps to its own die; the device-scope kernel runs one
    const uint32_t want_dies = gr->die_local ? gr->max_dies : 1;
    if (dies_for(e.n_inst, want_dies) != e.n_dies) {
      P = Plan();
      st = make_plan(G, in, with_grad, (char*)workspace, P, want_dies);
      if (st != TDF_OK) return st;
      w_packed = false;   // (the packed weights lie elsewhere now)
      e.out_i64 = (long long*)out->out_i64;
    }
    e.small_limit = (uint32_t)small_block;   // one pass of the single workgroup
    if (const char* w = getenv("TDF_SMALL_LIMIT")) e.small_limit = (uint32_t)std::max(1, atoi(w));
    // Fewer machines than dies (few instances, or the one machine of a batch that overflowed a
    // part of the table): steps with more frames than one die's lanes take in two passes run on
    // the whole GPU, at device scope.
    e.wide_limit = gr->die_local && e.n_dies < XCDS ? 16384u : 0u;
    if (const char* w = getenv("TDF_WIDE_LIMIT")) e.wide_limit = gr->die_local && e.n_dies < XCDS ? (uint32_t)std::max(0, atoi(w)) : 0u;
    e.follow_limit = e.small_limit;
    if (const char* w = getenv("TDF_FOLLOW_LIMIT")) e.follow_limit = (uint32_t)std::max(0, atoi(w));
    HIP_TRY(hipMemsetAsync(base + P.L.zero_begin, 0, P.L.zero_end - P.L.zero_begin, s));
    if (e.row_node) HIP_TRY(hipMemsetAsync(e.row_node, 0xFF, sizeof(uint32_t) * ((size_t)e.cap + e.n_inst), s));
    HIP_TRY(hipMemcpyAsync((void*)e.prog, (char*)gr->pinned + PIN_PROG, sizeof(DevProgram), hipMemcpyHostToDevice, s));
    launch_seed(G.prog, e, s);
    const Ctrl* hcs = (const Ctrl*)((char*)gr->pinned + PIN_CTRL);
    for (;;) {
      for (uint32_t i = 0; i < poll; ++i, ++rounds) {
        tdf_status lr = launch_round(G.prog, e, cus, gr->die_local, small_block, max_steps, spin_ticks, gr->jit, s);
        if (lr != TDF_OK) return lr;
      }
      HIP_TRY(hipMemcpyAsync((void*)hcs, e.ctrl, sizeof(Ctrl) * e.n_dies, hipMemcpyDeviceToHost, s));
      HIP_TRY(hipStreamSynchronize(s));
      bool all_done = true, any_status = false;
      for (uint32_t d = 0; d < e.n_dies; ++d) {
        all_done = all_done && hcs[d].done;
        any_status = any_status || hcs[d].status;
      }
      if (all_done || any_status) break;
    }
    // totals over the machines
    hc = Ctrl{};
    bool mixed_dies = false;
    uint32_t leaf_off[9] = {0}, cell_off[9] = {0};
    for (uint32_t d = 0; d < e.n_dies; ++d) {
      const Ctrl& c = hcs[d];
      hc.n_leaf += c.n_leaf; hc.n_cell += c.n_cell; hc.n_head += c.n_head;
      hc.n_tags += c.n_tags; hc.n_tokens += c.n_tokens;
      hc.n_alloc += c.n_alloc;
      hc.step = std::max(hc.step, c.step);
      hc.max_depth = std::max(hc.max_depth, c.max_depth);
      hc.max_level = std::max(hc.max_level, c.max_level);
      if (!hc.status) hc.status = c.status;
      hc.done = 1;
      mixed_dies = mixed_dies || (c.xcc_mask & (c.xcc_mask - 1)) != 0;
      leaf_off[d + 1] = leaf_off[d] + c.n_leaf;
      cell_off[d + 1] = cell_off[d] + c.n_cell;
    }
    // A die-local machine relies on its workgroups sharing one L2.  If the GPU placed them on
    // several dies, the run is void: repeat it with the kernel that synchronises through memory.
    if (gr->die_local && (mixed_dies || test_mixed_dies == 1)) {
      gr->die_local = false;
      ++repeats;
      continue;
    }
    // A part of the tag table can fill up although the whole table would not (instances of very
    // different sizes): repeat with one machine, which owns the whole table.
    if (e.n_dies > 1 && status_is(hc.status, TDF_ERR_TABLE_FULL) && (e.reclaim || hc.n_tags <= (unsigned long long)e.max_tags)) {
      gr->max_dies = 1;
      ++repeats;
      continue;
    }
    if (!e.reclaim && hc.n_tags > (unsigned long long)e.max_tags && !hc.status) hc.status = (uint32_t)(-TDF_ERR_TABLE_FULL);
    if (!hc.status) launch_merge_logs(e, leaf_off, cell_off, s);
    break;
  }
  end(TDF_PHASE_TAGS, 2 + 2ll * rounds);
  if (!hc.status && P.vec && with_grad && hc.n_cell > P.max_cells) hc.status = (uint32_t)(-TDF_ERR_TABLE_FULL);
  tdf_status dev = status_from_device(hc.status);

  uint32_t tail_first = 0;
  bool use_tail = false;   // the narrow levels run in one launch per pass on the caller's stream
  bool deep = false;       // deep instances run apart from the others, all their levels in one launch per pass
  bool deep_beside = false;   // ... on the side stream, beside the others
  uint32_t sh_last = 0, deep_base = 0, q_deep0 = 0, n_wide_levels = 0;
  const uint32_t* level_off = nullptr;   // by sort key; in the pinned buffer
  bool gcount_fetched = false;
  auto lvl_begin = [&](uint32_t lvl) { return level_off[(size_t)lvl * LEVEL_KEY_DIES]; };
  if (dev == TDF_OK && P.vec) {
    // ---- vector operators: leaves at once, cells level by level --------------------------
    // From here on the next evaluation's tag machine may run (not beside an evaluation in the static
    // workspace, which has one user at a time).  The leaves' rows and the sorts of the schedule are
    // ordinary launches: they do not wait for the data stage, which begins with the first cell launch.
    if (no_alloc) locks.data.lock();
    else locks.control.unlock();
    auto enter_data_stage = [&]() { if (!locks.data.owns_lock()) locks.data.lock(); };
    e.row0 = hc.n_leaf;   // leaf i has row i, the cell at position q of the sorted log row n_leaf + q
    hipStream_t s2 = (hipStream_t)gr->side_stream, s3 = (hipStream_t)gr->sort_stream;
    auto begin2 = [&](int ph) { if (timed) { (void)hipEventRecord((hipEvent_t)gr->events[2 * ph], s2); phase_used[ph] = true; } };
    auto end2 = [&](int ph, int64_t n) { if (timed) (void)hipEventRecord((hipEvent_t)gr->events[2 * ph + 1], s2); launches[ph] += n; };
    begin(TDF_PHASE_LEAVES);
    if (G.cell_kind && !w_packed) vec_pack_w(v, s);   // (a program of EMBEDs alone has no W: the pointers may be NULL)
    if (!with_grad) vec_embed(v, e, hc.n_leaf, s);
    end(TDF_PHASE_LEAVES, 2);
    if (with_grad) {
      // Gradient runs have a third stream.  The leaves' rows do not wait for the level sort, nor it for
      // them: they are written there, beside the sort on the caller's stream, and so is the embedding
      // gradient's token sort, which needs the leaf log only and has until the gradient pass's end.
      HIP_TRY(hipEventRecord((hipEvent_t)gr->fork_sort, s));
      HIP_TRY(hipStreamWaitEvent(s3, (hipEvent_t)gr->fork_sort, 0));
      vec_embed(v, e, hc.n_leaf, s3);
      HIP_TRY(hipEventRecord((hipEvent_t)gr->leaves_done, s3));
    }
    // (the token sort is put on its stream only after the level sort is on the caller's: the host's time
    // for its launches is not in the way of the first cell launch then)
    auto token_sort = [&]() -> tdf_status {
      if (!with_grad) return TDF_OK;
      vec_embed_sort(v, e, hc.n_leaf, (uint32_t*)(base + P.off_tok_count), (uint32_t*)(base + P.off_seg_off),
                     (uint32_t*)(base + P.off_chunk_off), (uint32_t*)(base + P.off_tok_fill),
                     (uint32_t*)(base + P.off_sorted), DE_CHUNK, s3);
      HIP_TRY(hipEventRecord((hipEvent_t)gr->join_sort, s3));
      return TDF_OK;
    };
    // Instances never exchange values, so instances whose recursion is deep (long chains: many
    // levels of a few cells each, bound by latency) can run beside the others (few levels of many
    // cells each, bound by throughput) instead of after them.  An instance is deep if its root's
    // level is at least deep_level; its cells get sort keys behind all keys of the shallow ones.
    uint32_t deep_level = 32;
    if (const char* w = getenv("TDF_DEEP_LEVEL")) deep_level = (uint32_t)std::max(0, atoi(w));
    const bool want_deep = with_grad && s2 && gr->die_local && !G.has_node_loss && deep_level > 0 && hc.max_level >= deep_level &&
                           hc.n_cell > 0;
    const int deep_wgs = getenv("TDF_DEEP_WGS") ? std::max(1, atoi(getenv("TDF_DEEP_WGS"))) : 16;   // workgroups per die
    if (hc.n_cell) {
      begin(TDF_PHASE_LEVELS);
      deep_base = want_deep ? deep_level * LEVEL_KEY_DIES : 0;
      const uint32_t n_keys = deep_base + (hc.max_level + 2) * LEVEL_KEY_DIES;
      if (want_deep) launch_class_keys(G.prog, e, hc.n_cell, deep_level, deep_base, s);
      launch_levels(e, hc.n_cell, n_keys, s);
      vec_number_rows(e, hc.n_leaf, hc.n_cell, G.has_head, G.out_type == T_VEC, s);
      const size_t level_bytes = (size_t)n_keys * sizeof(uint32_t);
      if (no_alloc && gr->pinned_bytes < PIN_LEVELS + level_bytes) {
        set_error("more dependency levels than the prepared graph's host buffer holds");
        return TDF_ERR_WORKSPACE;
      }
      if (!no_alloc)
        if (tdf_status ps = pinned_reserve(gr, level_bytes); ps != TDF_OK) return ps;
      level_off = (const uint32_t*)((char*)gr->pinned + PIN_LEVELS);
      HIP_TRY(hipMemcpyAsync((void*)level_off, e.level_off, level_bytes, hipMemcpyDeviceToHost, s));
      end(TDF_PHASE_LEVELS, 6);
      if (tdf_status ts_ = token_sort(); ts_ != TDF_OK) return ts_;
      HIP_TRY(hipStreamSynchronize(s));
      enter_data_stage();
      if (with_grad) HIP_TRY(hipStreamWaitEvent(s, (hipEvent_t)gr->leaves_done, 0));   // the cells read the leaves' rows
      sh_last = want_deep ? std::min(hc.max_level, deep_level - 1) : hc.max_level;
      q_deep0 = want_deep ? level_off[deep_base] : hc.n_cell;   // the shallow instances' cells come first
      deep = want_deep && q_deep0 < hc.n_cell;
      // Side by side only where the shallow instances' levels are worth about as much time as the deep
      // ones' chain (a level of the chain costs some microseconds whatever it holds, a wide level
      // costs its arithmetic); else the deep instances follow on the caller's stream with every
      // compute unit.  TDF_DEEP_BESIDE=0/1 forces either.
      bool beside = false;
      if (deep) {
        const double t_wide = 3.0 * 2.0 * (double)q_deep0 * v.N * (2.0 * v.H) / 4.5e14;
        const double t_chain = 16e-6 * hc.max_level;
        beside = t_wide >= 0.4 * t_chain;
        if (const char* w = getenv("TDF_DEEP_BESIDE")) beside = w[0] == '1';
      }
      hipStream_t sd = beside ? s2 : s;   // the deep instances' stream
      const int deep_per_die = beside ? deep_wgs : cus / (int)XCDS;
      auto begin_d = [&](int ph) { if (beside) begin2(ph); else begin(ph); };
      auto end_d = [&](int ph, int64_t n) { if (beside) end2(ph, n); else end(ph, n); };
      deep_beside = deep && beside;
      if (deep && beside) {
        // ---- the deep instances: forward, head and gradient pass in one chain on the side stream
        HIP_TRY(hipEventRecord((hipEvent_t)gr->fork_deep, s));
        HIP_TRY(hipStreamWaitEvent(s2, (hipEvent_t)gr->fork_deep, 0));
      }
      auto deep_chain = [&]() -> tdf_status {
        begin_d(TDF_PHASE_TAIL_FWD);
        vec_tail_fwd(v, e, e.level_off + deep_base, 1, hc.max_level, e.n_dies, base + P.off_tail_sync, spin_ticks, deep_per_die,
                     with_grad, sd);
        end_d(TDF_PHASE_TAIL_FWD, 1);
        if (G.has_head) vec_head(v, e, dy->dy, 1, 1, sd);
        begin_d(TDF_PHASE_TAIL_BWD);
        vec_tail_bwd(v, e, e.level_off + deep_base, 1, hc.max_level, e.n_dies, base + P.off_tail_sync + 8 * sizeof(DieSync),
                     spin_ticks, deep_per_die, q_deep0, G.has_head ? e.head_row : e.root_ref, sd);
        end_d(TDF_PHASE_TAIL_BWD, 2);
        if (beside) HIP_TRY(hipEventRecord((hipEvent_t)gr->join_deep, s2));
        return TDF_OK;
      };
      if (deep && G.out_type == T_VEC && !G.has_head) vec_seed_dy(v, e, dy->dy, s);   // (root rows of both classes)
      if (deep)
        if (tdf_status ds = deep_chain(); ds != TDF_OK) return ds;   // beside: on the side stream; else first, on the caller's
      // ---- the (other) instances on the caller's stream: wide levels one launch each; the narrow
      // levels behind them in one launch in which every die walks its own cells (unless the side
      // stream already runs such a launch)
      tail_first = sh_last + 1;
      while (tail_first > 1 && lvl_begin(tail_first) - lvl_begin(tail_first - 1) <= vec_small_level()) --tail_first;
      use_tail = !deep && gr->die_local && sh_last + 1 - tail_first >= 4;
      if (!use_tail) tail_first = sh_last + 1;
      n_wide_levels = tail_first - 1;
      begin(TDF_PHASE_CELLS_FWD);
      for (uint32_t lvl = 1; lvl < tail_first; ++lvl)
        vec_cell_fwd(v, e, lvl_begin(lvl), lvl_begin(lvl + 1) - lvl_begin(lvl), with_grad, s);
      end(TDF_PHASE_CELLS_FWD, tail_first - 1);
      if (use_tail) {
        begin(TDF_PHASE_TAIL_FWD);
        vec_tail_fwd(v, e, e.level_off, tail_first, sh_last, e.n_dies, base + P.off_tail_sync, spin_ticks, cus / (int)XCDS,
                     with_grad, s);
        end(TDF_PHASE_TAIL_FWD, 1);
      }
    }
    if (!hc.n_cell) {   // leaves only
      if (tdf_status ts_ = token_sort(); ts_ != TDF_OK) return ts_;
      enter_data_stage();
      vec_number_rows(e, hc.n_leaf, 0, G.has_head, G.out_type == T_VEC, s);
      if (with_grad) HIP_TRY(hipStreamWaitEvent(s, (hipEvent_t)gr->leaves_done, 0));
    }
    begin(TDF_PHASE_HEAD);
    if (G.has_head) {
      vec_head(v, e, with_grad ? dy->dy : nullptr, with_grad, deep ? 0 : -1, s);
    } else if (G.out_type == T_VEC) {
      if (G.has_node_loss) {
        // every state row that has a loss term: the term, and (gradient runs) its gradient with
        // respect to the row, which joins the row's dh where that is read
        HIP_TRY(hipMemsetAsync(out->out_node_loss, 0, sizeof(float) * (size_t)in->n_tree_nodes, s));
        vec_node_loss(v, e, hc.n_leaf, hc.n_cell, in->node_label, out->out_node_loss, with_grad ? dy->dnode : nullptr,
                      with_grad, s);
      }
      if (with_grad && !deep) vec_seed_dy(v, e, dy->dy, s);
    }
    end(TDF_PHASE_HEAD, G.has_node_loss ? 4 : 2);
    if (with_grad) {
      // ---- gradient pass: the level schedule walked backwards -----------------------------
      if (use_tail && hc.n_cell) {
        begin(TDF_PHASE_TAIL_BWD);
        vec_tail_bwd(v, e, e.level_off, tail_first, sh_last, e.n_dies, base + P.off_tail_sync + 8 * sizeof(DieSync),
                     spin_ticks, cus / (int)XCDS, lvl_begin(tail_first), G.has_head ? e.head_row : e.root_ref, s);
        end(TDF_PHASE_TAIL_BWD, 2);
      }
      begin(TDF_PHASE_CELLS_BWD);
      for (uint32_t lvl = tail_first - 1; lvl >= 1 && hc.n_cell; --lvl)
        vec_cell_bwd(v, e, lvl_begin(lvl), lvl_begin(lvl + 1) - lvl_begin(lvl), s);
      end(TDF_PHASE_CELLS_BWD, 2ll * (tail_first - 1));
      if (deep_beside) HIP_TRY(hipStreamWaitEvent(s, (hipEvent_t)gr->join_deep, 0));   // both classes' gradients are complete
    }
    // results of `result`, once every instance's root exists
    if (G.has_head) HIP_TRY(hipMemcpyAsync(out->out_f32, v.loss, sizeof(float) * e.n_inst, hipMemcpyDeviceToDevice, s));
    else if (G.out_type == T_VEC) vec_out_rows(v, e, out->out_h, out->out_c, s);
    if (with_grad) {
      // The embedding gradient and the weight gradients depend on the gradient pass only, not on
      // each other: the former runs on a second stream beside the latter.
      HIP_TRY(hipEventRecord((hipEvent_t)gr->fork_event, s));
      HIP_TRY(hipStreamWaitEvent(s2, (hipEvent_t)gr->fork_event, 0));
      HIP_TRY(hipStreamWaitEvent(s2, (hipEvent_t)gr->join_sort, 0));   // the leaves are in token order
      if (timed) { (void)hipEventRecord((hipEvent_t)gr->events[2 * TDF_PHASE_EMBED_GRAD], s2); phase_used[TDF_PHASE_EMBED_GRAD] = true; }
      vec_embed_sums(v, hc.n_leaf, (const uint32_t*)(base + P.off_seg_off), (const uint32_t*)(base + P.off_chunk_off),
                     (const uint32_t*)(base + P.off_sorted), (float*)(base + P.off_de_part), grads->dE, DE_CHUNK, s2);
      if (timed) (void)hipEventRecord((hipEvent_t)gr->events[2 * TDF_PHASE_EMBED_GRAD + 1], s2);
      launches[TDF_PHASE_EMBED_GRAD] += 5;
      // how often each tag's gradient body fired, as the kernels marked it (the cells' marks are complete
      // since the gradient pass, the leaves' since the sums just above)
      vec_count_grad(v, e, hc.n_leaf, hc.n_cell, (unsigned long long*)(base + P.off_gcount), s2);
      HIP_TRY(hipEventRecord((hipEvent_t)gr->join_event, s2));
      begin(TDF_PHASE_WEIGHT_GRAD);
      if (hc.n_cell) {
        v.q_stride = (hc.n_cell + 63) / 64 * 64;   // only the cells that fired
        vec_weight_grads(v, e, hc.n_cell, grads->dW, grads->db, (float*)(base + P.off_db_part), s);
      } else {
        HIP_TRY(hipMemsetAsync(grads->dW, 0, sizeof(float) * (size_t)v.N * 2 * v.H, s));
        HIP_TRY(hipMemsetAsync(grads->db, 0, sizeof(float) * (size_t)v.N, s));
      }
      end(TDF_PHASE_WEIGHT_GRAD, 7);
      HIP_TRY(hipStreamWaitEvent(s, (hipEvent_t)gr->join_event, 0));
    }
    HIP_TRY(hipGetLastError());
    const DieSync* ts = (const DieSync*)((char*)gr->pinned + PIN_SYNC);
    if (use_tail || deep) HIP_TRY(hipMemcpyAsync((void*)ts, base + P.off_tail_sync, sizeof(DieSync) * 16, hipMemcpyDeviceToHost, s));
    if (stats && with_grad) {   // (with the same synchronisation: how often the gradient bodies fired)
      HIP_TRY(hipMemcpyAsync((char*)gr->pinned + PIN_FIRE, base + P.off_gcount, sizeof(unsigned long long) * 2, hipMemcpyDeviceToHost, s));
      gcount_fetched = true;
    }
    if (with_grad && !no_alloc && locks.data.owns_lock()) {
      // Once the gradient pass is through (the event that the embedding gradient was forked at), what is
      // left of this evaluation are the weight and embedding sums: ordinary launches, no workgroups that
      // wait for each other.  The next evaluation's data plane may start beside them.
      HIP_TRY(hipEventSynchronize((hipEvent_t)gr->fork_event));
      locks.data.unlock();
    }
    HIP_TRY(hipStreamSynchronize(s));
    if (use_tail || deep) {
      bool mixed = false, gave_up = false;
      for (int k = 0; k < 16; ++k) {
        const DieSync& d = ts[k];
        mixed = mixed || (d.xcc_mask & (d.xcc_mask - 1)) != 0;
        gave_up = gave_up || d.abort != 0;
      }
      mixed = mixed || test_mixed_dies == 2;
      if (gave_up && !mixed) {
        set_error("device: a workgroup waited too long at a die barrier of the level tail");
        return TDF_ERR_DEVICE;
      }
      if (mixed) {   // the die-private launches did not keep to their dies: the results are void
        gr->die_local = false;
        if (locks.data.owns_lock()) locks.data.unlock();   // (control before data: start over in order)
        return run(gr, in, dy, out, grads, workspace, workspace_bytes, hip_stream, stats, with_grad, locks,
                   inherited_repeats + (int)repeats + 1, no_alloc);
      }
    }
  }
  HIP_TRY(hipGetLastError());

  if (stats) {
    HIP_TRY(hipStreamSynchronize(s));   // the last phase event may still be pending
    memset(stats, 0, sizeof(*stats));
    stats->n_tags = (int64_t)hc.n_tags;
    stats->n_steps = (int64_t)hc.step;
    stats->n_tokens = (int64_t)hc.n_tokens;
    stats->n_leaf_rows = hc.n_leaf;
    stats->n_cell_rows = hc.n_cell;
    stats->n_waves = hc.max_level;
    stats->n_wide_waves = hc.n_cell ? n_wide_levels : 0;
    stats->n_wide_cells = hc.n_cell && tail_first ? lvl_begin(tail_first) : 0;
    stats->deep_cells = deep ? (int64_t)(hc.n_cell - q_deep0) : 0;
    unsigned long long* pin_counts = (unsigned long long*)((char*)gr->pinned + PIN_FIRE);
    if (with_grad && dev == TDF_OK && P.vec) {
      if (!gcount_fetched) {
        HIP_TRY(hipMemcpyAsync(pin_counts, base + P.off_gcount, sizeof(unsigned long long) * 2, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
      }
      stats->n_grad_firings = (int64_t)pin_counts[0];
      stats->n_grad_not_once = (int64_t)pin_counts[1];
    }
    stats->n_machines = (int32_t)e.n_dies;
    stats->die_local = gr->die_local ? 1 : 0;
    stats->generated = use_jit ? 1 : 0;
    stats->repeats = (int32_t)repeats + inherited_repeats;
    stats->tail_used = use_tail || deep ? 1 : 0;
    stats->deep_split = deep ? (deep_beside ? 2 : 1) : 0;
    stats->max_tag_depth = hc.max_depth;
    stats->table_capacity = e.cap;
    stats->peak_frames = (int64_t)hc.n_alloc;
    stats->frames_reclaimed = e.reclaim ? 1 : 0;
    stats->max_probe = hc.n_tags > e.n_inst ? 1 : 0;   // the match table is addressed without collisions
    for (int ph = 0; ph < TDF_PHASE_COUNT; ++ph) {
      float ms = 0.f;
      if (phase_used[ph] && hipEventElapsedTime(&ms, (hipEvent_t)gr->events[2 * ph], (hipEvent_t)gr->events[2 * ph + 1]) == hipSuccess)
        stats->phase_ms[ph] = ms;
      stats->phase_launches[ph] = launches[ph];
    }
    if (phase_used[TDF_PHASE_CELLS_FWD]) {   // forward cell kernels on both streams: first launch to last end
      float a = 0.f, b = 0.f;
      (void)hipEventElapsedTime(&a, (hipEvent_t)gr->events[2 * TDF_PHASE_CELLS_FWD], (hipEvent_t)gr->events[2 * TDF_PHASE_CELLS_FWD + 1]);
      if (phase_used[TDF_PHASE_TAIL_FWD] &&
          hipEventElapsedTime(&b, (hipEvent_t)gr->events[2 * TDF_PHASE_CELLS_FWD], (hipEvent_t)gr->events[2 * TDF_PHASE_TAIL_FWD + 1]) != hipSuccess)
        b = 0.f;
      stats->fwd_cells_span_ms = std::max(a, b);
    }
    if (e.step_log && !no_alloc && dev == TDF_OK) {
      // the widest steps of the tag machines: frames, frames created, duration
      std::vector<uint4> log((size_t)STEP_LOG_CAP * e.n_dies);
      HIP_TRY(hipMemcpy(log.data(), e.step_log, log.size() * sizeof(uint4), hipMemcpyDeviceToHost));
      struct Rec { uint32_t frames, created; double us; };
      std::vector<Rec> recs;
      const Ctrl* hcs2 = (const Ctrl*)((char*)gr->pinned + PIN_CTRL);
      for (uint32_t d = 0; d < e.n_dies; ++d) {
        const uint32_t n_steps = std::min<uint32_t>(hcs2[d].step, STEP_LOG_CAP);
        for (uint32_t k = 1; k < n_steps; ++k) {
          const uint4 &a = log[(size_t)d * STEP_LOG_CAP + k - 1], &b = log[(size_t)d * STEP_LOG_CAP + k];
          recs.push_back(Rec{b.x, b.y - a.y, (double)(uint32_t)(b.z - a.z) / 100.0});
        }
      }
      std::sort(recs.begin(), recs.end(), [](const Rec& x, const Rec& y) { return x.frames > y.frames; });
      for (size_t k = 0; k < recs.size() && k < 8; ++k) {
        stats->wide_step_frames[k] = recs[k].frames;
        stats->wide_step_created[k] = recs[k].created;
        stats->wide_step_us[k] = recs[k].us;
      }
    }
    stats->device_status = -(int32_t)hc.status;
    stats->n_counts = (int32_t)G.snodes.size();
    if (in->stats_level >= 1) {   // (below that level the counts are not taken: fire_count stays zero, no read-back)
      launch_count_fired(G.prog, e, s);
      HIP_TRY(hipMemcpyAsync(pin_counts, e.fire_count, sizeof(unsigned long long) * TDF_STATS_MAX_COUNTS, hipMemcpyDeviceToHost, s));
      HIP_TRY(hipStreamSynchronize(s));
      for (int i = 0; i < TDF_STATS_MAX_COUNTS; ++i) stats->fire_count[i] = (int64_t)pin_counts[i];
    }
  }
  return dev;
}

}  // namespace
}  // namespace tdf

using namespace tdf;

tdf_graph::~tdf_graph() {
  jit_release(jit);
  for (void* ev : events)
    if (ev) (void)hipEventDestroy((hipEvent_t)ev);
  for (void* st : {side_stream, sort_stream})
    if (st) {
      (void)hipStreamSynchronize((hipStream_t)st);
      (void)hipStreamDestroy((hipStream_t)st);
    }
  for (void* ev : {fork_event, join_event, fork_deep, join_deep, fork_sort, join_sort, leaves_done})
    if (ev) (void)hipEventDestroy((hipEvent_t)ev);
  if (pinned) (void)hipHostFree(pinned);
}


extern "C" tdf_status tdf_workspace_size(const tdf_graph* g, const tdf_inputs* in, int with_grad, size_t* bytes) {
  if (!g || !bytes) {
    set_error("tdf_workspace_size: NULL argument");
    return TDF_ERR_BAD_ARG;
  }
  Plan P;
  tdf_status st = make_plan(g->g, in, with_grad != 0, nullptr, P, 8);
  if (st != TDF_OK) return st;
  *bytes = P.L.total;
  return TDF_OK;
}

// The step kernels and the chain launches are persistent: their workgroups wait for each other at
// barriers, so all of them must be on the GPU together.  Two tag machines, or two data planes, in
// flight on different streams could each hold a part of the compute units and wait for the rest (the
// bounded waits would end that with TDF_ERR_DEVICE, not a hang): evaluations of one process take
// turns, stage by stage (EvalLocks).

extern "C" tdf_status tdf_eval(tdf_graph* g, const tdf_inputs* in, tdf_outputs* out, void* workspace,
                               size_t workspace_bytes, void* hip_stream, tdf_stats* stats) {
  if (!g) { set_error("NULL graph"); return TDF_ERR_BAD_ARG; }
  std::lock_guard<std::mutex> own(g->busy);   // (before the stage locks: graph, control, data)
  EvalLocks locks;
  return run(g, in, nullptr, out, nullptr, workspace, workspace_bytes, hip_stream, stats, false, locks);
}

extern "C" tdf_status tdf_eval_grad(tdf_graph* g, const tdf_inputs* in, const tdf_seed* dy, tdf_outputs* out,
                                    tdf_grads* grads, void* workspace, size_t workspace_bytes,
                                    void* hip_stream, tdf_stats* stats) {
  if (!g) { set_error("NULL graph"); return TDF_ERR_BAD_ARG; }
  std::lock_guard<std::mutex> own(g->busy);
  EvalLocks locks;
  return run(g, in, dy, out, grads, workspace, workspace_bytes, hip_stream, stats, true, locks);
}

// ---- evaluation without any allocation ------------------------------------------------------------
// For callers that cannot allocate (code under stream capture, tight serving loops, harnesses that
// forbid it): the workspace is a file-scope device array, one copy per GPU, that lives as long as the
// process.  Host code never passes the array's name to the device: its address on a GPU is resolved
// once per device (hipGetSymbolAddress, by tdf_graph_prepare with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[TDF_STATIC_WORKSPACE_BYTES];
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {nullptr};   // by device ordinal
// levels of cell firings whose offsets the prepared host buffer can take (vector programs)
static constexpr size_t PREPARED_LEVEL_BYTES = (size_t)(8192 + 2) * LEVEL_KEY_DIES * sizeof(uint32_t);

extern "C" tdf_status tdf_graph_prepare(tdf_graph* g) {
  if (!g) {
    set_error("tdf_graph_prepare: NULL graph");
    return TDF_ERR_BAD_ARG;
  }
  std::lock_guard<std::mutex> own(g->busy);
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) {
    set_error("tdf_graph_prepare: device ordinal out of range");
    return TDF_ERR_UNSUPPORTED;
  }
  {
    std::lock_guard<std::mutex> l2(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void* ptr = nullptr;
      HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));   // this device's copy of the array
      if (!ptr || ((uintptr_t)ptr & 255)) {
        set_error("tdf_graph_prepare: the static workspace has no usable address on this device");
        return TDF_ERR_DEVICE;
      }
      g_scratch_ptr[dev] = ptr;
    }
  }
  for (int i = 0; i < 2 * TDF_PHASE_COUNT; ++i)
    if (!g->events[i]) HIP_TRY(hipEventCreate((hipEvent_t*)&g->events[i]));
  if (tdf_status ps = pinned_reserve(g, PREPARED_LEVEL_BYTES); ps != TDF_OK) return ps;
  if (!g->jit.tried) {
    g->jit.tried = true;
    std::string log;
    (void)jit_compile(g->g.prog, g->jit, log);   // without the run-time compiler the table interpreter runs
  }
  g->prepared = true;
  g->prepared_device = dev;
  return TDF_OK;
}

extern "C" tdf_status tdf_eval_static(tdf_graph* g, const tdf_inputs* in, tdf_outputs* out, void* hip_stream, tdf_stats* stats) {
  if (!g) {
    set_error("tdf_eval_static: NULL graph");
    return TDF_ERR_BAD_ARG;
  }
  std::lock_guard<std::mutex> own(g->busy);
  EvalLocks locks;
  locks.control.lock();
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  void* ptr = nullptr;
  if (dev >= 0 && dev < 64) {
    std::lock_guard<std::mutex> l2(g_scratch_mutex);
    ptr = g_scratch_ptr[dev];
  }
  if (!g->prepared || g->prepared_device != dev || !ptr) {
    set_error("tdf_eval_static: call tdf_graph_prepare on this device first");
    return TDF_ERR_BAD_ARG;
  }
  Plan P;
  tdf_status st = make_plan(g->g, in, false, nullptr, P, 8);
  if (st != TDF_OK) return st;
  if (P.L.total > TDF_STATIC_WORKSPACE_BYTES) {
    set_error("tdf_eval_static: these inputs need " + std::to_string(P.L.total) + " bytes of workspace, the static one has " +
              std::to_string((size_t)TDF_STATIC_WORKSPACE_BYTES) + " (lower max_tags, or use tdf_eval with a workspace of your own)");
    return TDF_ERR_WORKSPACE;
  }
  return run(g, in, nullptr, out, nullptr, ptr, TDF_STATIC_WORKSPACE_BYTES, hip_stream, stats, false, locks, 0, true);
}
