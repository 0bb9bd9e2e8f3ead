// Host side of tdf_graph_build: validation, the transformation of a set of function graphs
// into one static tagged graph (paper Section 3; while-loops: Section 2.3), the gradient half
// of the joint functions (Section 4), and the compilation of the per-function firing tables
// used on the device.
#include <string.h>

#include <map>
#include <sstream>

#include "tdf_internal.h"

namespace tdf {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }

namespace {

struct Bad {
  std::string msg;
};
[[noreturn]] void bad(const std::string& m) { throw Bad{m}; }

constexpr int T_UNKNOWN = 7;

int arity_of(int op, int n_in) {
  switch (op) {
    case TDF_OP_IN: case TDF_OP_CONST: return 0;
    case TDF_OP_OUT: case TDF_OP_ID: case TDF_OP_TREE_ISLEAF: case TDF_OP_TREE_LEFT:
    case TDF_OP_TREE_RIGHT: case TDF_OP_TREE_TOKEN: case TDF_OP_EMBED: return 1;
    case TDF_OP_ADD: case TDF_OP_SUB: case TDF_OP_MUL: case TDF_OP_EQ: case TDF_OP_LT:
    case TDF_OP_SWITCH: case TDF_OP_RNN_CELL: case TDF_OP_LSTM_CELL: case TDF_OP_CE_HEAD: case TDF_OP_CE_NODE: return 2;
    case TDF_OP_MERGE: case TDF_OP_CALLFN: case TDF_OP_LOOP: case TDF_OP_NEXT: return n_in;
  }
  return -1;
}

struct Builder {
  const tdf_program_desc* P;
  bool want_grad;
  Graph& G;
  std::vector<std::vector<int>> type;   // [fn][node] output type
  std::vector<int> ret_type;            // [fn]
  std::map<std::pair<int, int>, int> label_of;   // (fn, node) -> call label (LOOP nodes are numbered with the calls)
  std::vector<int> is_loop;             // [fn] the graph has a NEXT node: a loop graph

  Builder(const tdf_program_desc* p, bool wg, Graph& g) : P(p), want_grad(wg), G(g) {}

  const tdf_function_desc& F(int f) const { return P->functions[f]; }
  bool is_const(int f, tdf_ref r) const { return F(f).nodes[r.node].op == TDF_OP_CONST; }

  // ---- 1. validation --------------------------------------------------------------
  void validate() {
    if (!P || P->n_functions < 1 || !P->functions) bad("empty program");
    if (P->n_functions > MAX_FN) bad("too many functions");
    if (P->result_fn < 0 || P->result_fn >= P->n_functions) bad("result_fn out of range");
    is_loop.assign(P->n_functions, 0);
    std::vector<int> loop_users(P->n_functions, 0);
    for (int f = 0; f < P->n_functions; ++f) {
      const auto& fn = F(f);
      if (!fn.nodes || fn.n_nodes < 1) bad("function without nodes");
      for (int i = 0; i < fn.n_nodes; ++i) is_loop[f] += fn.nodes[i].op == TDF_OP_NEXT;
      if (is_loop[f] > 1) bad("a loop graph has exactly one NEXT");
    }
    if (is_loop[P->result_fn]) bad("result cannot be a loop graph");
    for (int f = 0; f < P->n_functions; ++f) {
      const auto& fn = F(f);
      if (fn.n_nodes > MAX_VALUES) bad("more than 64 nodes in a function");
      if (fn.n_params < 0 || fn.n_params > TDF_MAX_INPUTS) bad("a function has at most 4 parameters");
      int n_out = 0;
      std::vector<int> seen_param(fn.n_params, 0);
      for (int i = 0; i < fn.n_nodes; ++i) {
        const auto& nd = fn.nodes[i];
        if (nd.op < 0 || nd.op >= TDF_OP_COUNT) bad("unknown operator");
        if (nd.n_in < 0 || nd.n_in > TDF_MAX_INPUTS) bad("bad input count");
        int want = arity_of(nd.op, nd.n_in);
        if (want != nd.n_in) bad("wrong number of inputs for an operator");
        if (nd.op == TDF_OP_MERGE && nd.n_in < 2) bad("MERGE needs at least two inputs");
        int n_const = 0;
        for (int k = 0; k < nd.n_in; ++k) {
          tdf_ref r = nd.in[k];
          if (r.node < 0 || r.node >= i) bad("input refers to a later node (or itself)");
          int sop = fn.nodes[r.node].op;
          if (sop == TDF_OP_OUT || sop == TDF_OP_NEXT) bad("OUT and NEXT have no output");
          if (r.port != 0 && !(r.port == 1 && sop == TDF_OP_SWITCH)) bad("bad port");
          n_const += sop == TDF_OP_CONST;
        }
        if (nd.op == TDF_OP_OUT) ++n_out;
        if (nd.op == TDF_OP_IN) {
          if (nd.imm < 0 || nd.imm >= fn.n_params) bad("IN index out of range");
          if (seen_param[nd.imm]++) bad("parameter has two IN nodes");
        }
        if (nd.op == TDF_OP_CALLFN) {
          if (nd.imm < 0 || nd.imm >= P->n_functions) bad("call to undefined function");
          if (nd.imm == P->result_fn) bad("result cannot be called");
          if (nd.n_in != F((int)nd.imm).n_params) bad("arity mismatch in a call");
          if (nd.n_in < 1) bad("a called function needs at least one parameter");
          if (is_loop[nd.imm]) bad("a loop graph cannot be called");
        }
        if (nd.op == TDF_OP_LOOP) {
          if (nd.imm < 0 || nd.imm >= P->n_functions || !is_loop[nd.imm]) bad("LOOP over a graph without NEXT");
          if (nd.n_in != F((int)nd.imm).n_params) bad("LOOP needs one initial value per loop variable");
          if (want_grad) bad("gradient of a program with loops");
          ++loop_users[nd.imm];
        }
        if (nd.op == TDF_OP_NEXT && (nd.n_in != fn.n_params || nd.n_in < 1)) bad("NEXT needs one value per loop variable");
        if (nd.op == TDF_OP_MERGE && n_const) bad("MERGE of a constant");
        if (nd.op == TDF_OP_SWITCH && is_const(f, nd.in[0])) bad("SWITCH on a constant predicate");
        const bool per_input = nd.op == TDF_OP_CALLFN || nd.op == TDF_OP_LOOP || nd.op == TDF_OP_NEXT;   // one table entry per input
        if (n_const > 1 && !per_input) bad("operator with two constant inputs: fold it");
        if (nd.n_in > 0 && n_const == nd.n_in && f != P->result_fn)
          bad("operator fed by constants only outside result");
      }
      if (n_out != 1) bad("a function needs exactly one OUT");
    }
    for (int f = 0; f < P->n_functions; ++f)
      if (is_loop[f] && loop_users[f] != 1) bad("a loop graph belongs to exactly one LOOP node");
  }

  // ---- 2. types: int64 scalars, row references of vector operators, the head's loss ---
  void infer_types() {
    int nf = P->n_functions;
    type.assign(nf, {});
    ret_type.assign(nf, T_UNKNOWN);
    for (int f = 0; f < nf; ++f) type[f].assign(F(f).n_nodes, T_UNKNOWN);
    for (int iter = 0; iter < 4; ++iter) {
      for (int f = 0; f < nf; ++f) {
        const auto& fn = F(f);
        for (int i = 0; i < fn.n_nodes; ++i) {
          const auto& nd = fn.nodes[i];
          auto in_t = [&](int k) { return type[f][nd.in[k].node]; };
          int t = T_UNKNOWN;
          switch (nd.op) {
            case TDF_OP_IN: case TDF_OP_CONST: case TDF_OP_ADD: case TDF_OP_SUB: case TDF_OP_MUL:
            case TDF_OP_EQ: case TDF_OP_LT: case TDF_OP_TREE_ISLEAF: case TDF_OP_TREE_LEFT:
            case TDF_OP_TREE_RIGHT: case TDF_OP_TREE_TOKEN: t = T_INT; break;
            case TDF_OP_EMBED: case TDF_OP_RNN_CELL: case TDF_OP_LSTM_CELL: case TDF_OP_CE_NODE: t = T_VEC; break;
            case TDF_OP_CE_HEAD: t = T_LOSS; break;
            case TDF_OP_ID: case TDF_OP_OUT: t = in_t(0); break;
            case TDF_OP_SWITCH: t = in_t(1); break;
            case TDF_OP_MERGE:
              for (int k = 0; k < nd.n_in; ++k) if (in_t(k) != T_UNKNOWN) t = in_t(k);
              break;
            case TDF_OP_CALLFN: case TDF_OP_LOOP: t = ret_type[nd.imm]; break;
            case TDF_OP_NEXT: t = T_INT; break;   // no value; loop variables are integers
          }
          type[f][i] = t;
          if (nd.op == TDF_OP_OUT) ret_type[f] = t;
        }
      }
    }
    for (int f = 0; f < nf; ++f) {
      const auto& fn = F(f);
      for (int i = 0; i < fn.n_nodes; ++i) {
        const auto& nd = fn.nodes[i];
        if (type[f][i] == T_UNKNOWN) bad("cannot type a node (recursion without a base case?)");
        auto need = [&](int k, int t) { if (type[f][nd.in[k].node] != t) bad("operand type mismatch"); };
        switch (nd.op) {
          case TDF_OP_ADD: case TDF_OP_SUB: case TDF_OP_MUL: case TDF_OP_EQ: case TDF_OP_LT:
            need(0, T_INT); need(1, T_INT); break;
          case TDF_OP_TREE_ISLEAF: case TDF_OP_TREE_LEFT: case TDF_OP_TREE_RIGHT:
          case TDF_OP_TREE_TOKEN: case TDF_OP_EMBED: need(0, T_INT); break;
          case TDF_OP_RNN_CELL: case TDF_OP_LSTM_CELL: need(0, T_VEC); need(1, T_VEC); break;
          case TDF_OP_CE_HEAD: case TDF_OP_CE_NODE: need(0, T_VEC); need(1, T_INT); break;
          case TDF_OP_SWITCH: need(0, T_INT); break;
          case TDF_OP_MERGE: for (int k = 0; k < nd.n_in; ++k) need(k, type[f][i]); break;
          case TDF_OP_CALLFN: case TDF_OP_LOOP: case TDF_OP_NEXT:
            for (int k = 0; k < nd.n_in; ++k) need(k, T_INT);
            break;
          default: break;
        }
        if (nd.op == TDF_OP_RNN_CELL || nd.op == TDF_OP_LSTM_CELL) {
          int kind = nd.op == TDF_OP_RNN_CELL ? 1 : 2;
          if (G.cell_kind && G.cell_kind != kind) bad("RNN and LSTM cells in one program");
          G.cell_kind = kind;
        }
        if (nd.op == TDF_OP_EMBED) G.has_embed = true;
        if (nd.op == TDF_OP_CE_HEAD) {
          if (f != P->result_fn) bad("CE_HEAD is only allowed in result");
          G.has_head = true;
        }
        if (nd.op == TDF_OP_CE_NODE) G.has_node_loss = true;
        if (type[f][i] == T_LOSS && f != P->result_fn) bad("loss values are only allowed in result");
      }
    }
    if (G.has_head && G.has_node_loss) bad("CE_HEAD and CE_NODE in one program");
    // A vector value is named by the frame (the tag) that produced it, so a tag may produce one: two
    // operators that make state rows must lie on opposite sides of a Switch.  side[t][i]: the switches
    // whose true (t = 0) / false (t = 1) output node i cannot be live without; a Merge is live with
    // any one of its inputs and keeps only what all of them share.
    for (int f = 0; f < nf; ++f) {
      const auto& fn = F(f);
      std::vector<uint64_t> side[2] = {std::vector<uint64_t>(fn.n_nodes, 0), std::vector<uint64_t>(fn.n_nodes, 0)};
      std::vector<int> makers;
      for (int i = 0; i < fn.n_nodes; ++i) {
        const auto& nd = fn.nodes[i];
        for (int t = 0; t < 2; ++t) {
          uint64_t m = nd.op == TDF_OP_MERGE ? ~0ull : 0ull;
          for (int k = 0; k < nd.n_in; ++k) {
            const auto& r = nd.in[k];
            uint64_t from = side[t][r.node];
            if (fn.nodes[r.node].op == TDF_OP_SWITCH && r.port == t) from |= 1ull << r.node;
            m = nd.op == TDF_OP_MERGE ? (m & from) : (m | from);
          }
          side[t][i] = nd.n_in ? m : 0ull;
        }
        if (nd.op == TDF_OP_EMBED || nd.op == TDF_OP_RNN_CELL || nd.op == TDF_OP_LSTM_CELL) makers.push_back(i);
      }
      for (size_t a = 0; a < makers.size(); ++a)
        for (size_t b = a + 1; b < makers.size(); ++b) {
          const int i = makers[a], j = makers[b];
          if (((side[0][i] & side[1][j]) | (side[1][i] & side[0][j])) == 0)
            bad("two operators that make a vector value can fire under one tag: put each in a function of its own");
        }
    }
    G.out_type = ret_type[P->result_fn];
    G.n_result_params = F(P->result_fn).n_params;
    if (want_grad && G.out_type == T_INT) bad("gradient of an integer program");
  }

  // ---- 3. call labels: result's calls first, then the other functions ----------------
  std::vector<int> fn_order() const {
    std::vector<int> o{P->result_fn};
    for (int f = 0; f < P->n_functions; ++f) if (f != P->result_fn) o.push_back(f);
    return o;
  }
  void number_calls() {
    for (int f : fn_order())
      for (int i = 0; i < F(f).n_nodes; ++i)
        if (F(f).nodes[i].op == TDF_OP_CALLFN || F(f).nodes[i].op == TDF_OP_LOOP) {
          int lab = (int)label_of.size();
          label_of[{f, i}] = lab;
        }
    G.n_labels = (int)label_of.size();
    if (G.n_labels > MAX_LABELS) bad("too many call sites");
  }

  // ---- 4. the static graph (Section 3) ----------------------------------------------
  // smap: (fn, node, port) -> static node producing that value
  std::map<std::tuple<int, int, int>, int> smap;
  std::map<std::pair<int, int>, int> entry;        // (fn, param) -> entry Merge
  std::map<int, int> grad_entry;                   // fn -> gradient entry Merge / gin
  std::map<std::pair<int, int>, std::vector<int>> call_snodes;   // (fn,node) -> Call_i per param

  int add_snode(int kind, int fn, int label, int param, int is_grad, int64_t imm) {
    G.snodes.push_back(tdf_snode{kind, fn, label, param, is_grad, imm});
    return (int)G.snodes.size() - 1;
  }
  void add_edge(int src, int port, int dst, int slot, int ctl) {
    G.sedges.push_back(tdf_sedge{src, port, dst, slot, ctl});
  }

  void build_static_graph() {
    auto order = fn_order();
    // ordinary nodes; input nodes of callees become Merge nodes; call nodes vanish
    for (int f : order)
      for (int i = 0; i < F(f).n_nodes; ++i) {
        const auto& nd = F(f).nodes[i];
        if (nd.op == TDF_OP_CALLFN || nd.op == TDF_OP_LOOP || nd.op == TDF_OP_NEXT) continue;
        if (nd.op == TDF_OP_OUT && f != P->result_fn) continue;   // absorbed by the Returns / the Exit
        int s;
        if (nd.op == TDF_OP_IN && f != P->result_fn) {
          s = add_snode(TDF_SNODE_MERGE_ENTRY, f, -1, (int)nd.imm, 0, 0);
          entry[{f, (int)nd.imm}] = s;
        } else {
          s = add_snode(nd.op, f, -1, nd.op == TDF_OP_IN ? (int)nd.imm : -1, 0,
                        nd.op == TDF_OP_CONST ? nd.imm : 0);
        }
        smap[{f, i, 0}] = s;
        if (nd.op == TDF_OP_SWITCH) smap[{f, i, 1}] = s;
      }
    // Call_i (one per formal parameter) and Return_i; control edge Call_i -> Return_i
    for (int f : order)
      for (int i = 0; i < F(f).n_nodes; ++i) {
        const auto& nd = F(f).nodes[i];
        std::vector<int> cs;
        if (nd.op == TDF_OP_NEXT) {   // Section 2.3: one Next per loop variable, feeding its Merge
          for (int k = 0; k < nd.n_in; ++k) cs.push_back(add_snode(TDF_SNODE_NEXT, f, -1, k, 0, 0));
          call_snodes[{f, i}] = cs;
          continue;
        }
        if (nd.op != TDF_OP_CALLFN && nd.op != TDF_OP_LOOP) continue;
        const bool loop = nd.op == TDF_OP_LOOP;   // Enter per loop variable and Exit, placed like Call_i and Return_i
        int lab = label_of[{f, i}], callee = (int)nd.imm;
        for (int k = 0; k < nd.n_in; ++k)
          cs.push_back(add_snode(loop ? TDF_SNODE_ENTER : TDF_SNODE_CALL, f, lab, k, 0, callee));
        int r = add_snode(loop ? TDF_SNODE_EXIT : TDF_SNODE_RETURN, f, lab, -1, 0, callee);
        call_snodes[{f, i}] = cs;
        smap[{f, i, 0}] = r;
      }
    // edges
    for (int f : order)
      for (int i = 0; i < F(f).n_nodes; ++i) {
        const auto& nd = F(f).nodes[i];
        if (nd.op == TDF_OP_NEXT) {
          const auto& cs = call_snodes[{f, i}];
          for (int k = 0; k < nd.n_in; ++k) {
            add_edge(smap[{f, nd.in[k].node, 0}], nd.in[k].port, cs[k], 0, 0);
            auto it = entry.find({f, k});   // the Merge's slot after those of the labels
            if (it != entry.end()) add_edge(cs[k], 0, it->second, G.n_labels, 0);
          }
        } else if (nd.op == TDF_OP_CALLFN || nd.op == TDF_OP_LOOP) {
          int lab = label_of[{f, i}], callee = (int)nd.imm;
          const auto& cs = call_snodes[{f, i}];
          int r = smap[{f, i, 0}];
          for (int k = 0; k < nd.n_in; ++k) {
            add_edge(smap[{f, nd.in[k].node, 0}], nd.in[k].port, cs[k], 0, 0);
            auto it = entry.find({callee, k});
            if (it != entry.end()) add_edge(cs[k], 0, it->second, lab, 0);
            add_edge(cs[k], 0, r, k, 1);
          }
          // Return_i hangs on the value that fed the callee's OUT
          const auto& cf = F(callee);
          for (int j = 0; j < cf.n_nodes; ++j)
            if (cf.nodes[j].op == TDF_OP_OUT)
              add_edge(smap[{callee, cf.nodes[j].in[0].node, 0}], cf.nodes[j].in[0].port, r, 0, 0);
        } else if (!(nd.op == TDF_OP_OUT && f != P->result_fn)) {
          int s = smap[{f, i, 0}];
          for (int k = 0; k < nd.n_in; ++k)
            add_edge(smap[{f, nd.in[k].node, 0}], nd.in[k].port, s, k, 0);
        }
      }
  }

  // ---- 5. gradient half of the joint functions (Section 4) -----------------------------
  // Only row references (and the head's loss) are differentiable; integer values carry no
  // gradient.  Every differentiable value must have a single differentiable consumer, so
  // no summation node is needed.
  void build_gradient_graph() {
    auto order = fn_order();
    for (int f : order) {
      if (ret_type[f] == T_INT) continue;
      grad_entry[f] = f == P->result_fn ? add_snode(TDF_OP_IN, f, -1, 0, 1, 0)
                                        : add_snode(TDF_SNODE_MERGE_ENTRY, f, -1, 0, 1, 0);
    }
    for (int f : order) {
      if (ret_type[f] == T_INT) continue;
      const auto& fn = F(f);
      std::map<std::pair<int, int>, std::pair<int, int>> dval;   // (node,port) -> (snode, port)
      auto push = [&](tdf_ref r, int s, int port) {
        if (type[f][r.node] == T_INT || fn.nodes[r.node].op == TDF_OP_CONST) return;
        if (dval.count({r.node, r.port})) bad("a vector value has two differentiable consumers");
        dval[{r.node, r.port}] = {s, port};
      };
      for (int i = fn.n_nodes - 1; i >= 0; --i) {
        const auto& nd = fn.nodes[i];
        if (nd.op == TDF_OP_OUT) {
          push(nd.in[0], grad_entry[f], 0);
          continue;
        }
        if (nd.op == TDF_OP_SWITCH) {
          auto t = dval.find({i, 0}), e = dval.find({i, 1});
          if (t == dval.end() && e == dval.end()) continue;
          if (t != dval.end() && e != dval.end()) {
            int m = add_snode(TDF_OP_SWITCH, f, -1, -1, 1, 0);   // Switch^grad: merge of the two sides
            add_edge(t->second.first, t->second.second, m, 0, 0);
            add_edge(e->second.first, e->second.second, m, 1, 0);
            push(nd.in[1], m, 0);
          } else {
            auto one = t != dval.end() ? t->second : e->second;
            push(nd.in[1], one.first, one.second);
          }
          continue;
        }
        auto it = dval.find({i, 0});
        if (it == dval.end()) {
          // A state row nobody differentiates would still fire and be walked by the gradient pass,
          // which would then read a gradient row that no operator wrote.
          if (nd.op == TDF_OP_EMBED || nd.op == TDF_OP_RNN_CELL || nd.op == TDF_OP_LSTM_CELL || nd.op == TDF_OP_CE_NODE)
            bad("a vector value without a consumer on the differentiable path");
          continue;
        }
        int dy = it->second.first, dyp = it->second.second;
        auto fwd = [&](int k) { return smap[{f, nd.in[k].node, 0}]; };
        switch (nd.op) {
          case TDF_OP_ID: push(nd.in[0], dy, dyp); break;
          case TDF_OP_MERGE:
            for (int k = 0; k < nd.n_in; ++k) {   // dx_k = dy where x_k was live, else dead
              int s = add_snode(TDF_OP_MERGE, f, -1, k, 1, 0);
              add_edge(fwd(k), nd.in[k].port, s, 0, 0);
              add_edge(dy, dyp, s, 1, 0);
              push(nd.in[k], s, 0);
            }
            break;
          case TDF_OP_CALLFN: {   // Call_i^grad with the label of the forward call
            int lab = label_of[{f, i}], callee = (int)nd.imm;
            int c = add_snode(TDF_SNODE_CALL, f, lab, 0, 1, callee);
            add_edge(dy, dyp, c, 0, 0);
            add_edge(c, 0, grad_entry[callee], lab, 0);
            break;
          }
          case TDF_OP_EMBED: {
            int s = add_snode(TDF_OP_EMBED, f, -1, -1, 1, 0);   // sink: dE[token] += dy
            add_edge(fwd(0), nd.in[0].port, s, 0, 0);
            add_edge(dy, dyp, s, 1, 0);
            break;
          }
          case TDF_OP_RNN_CELL: case TDF_OP_LSTM_CELL: {
            int s = add_snode(nd.op, f, -1, -1, 1, 0);   // (x_l, x_r, dy) -> (dx_l, dx_r)
            add_edge(fwd(0), nd.in[0].port, s, 0, 0);
            add_edge(fwd(1), nd.in[1].port, s, 1, 0);
            add_edge(dy, dyp, s, 2, 0);
            push(nd.in[0], s, 0);
            push(nd.in[1], s, 1);
            break;
          }
          case TDF_OP_CE_HEAD: {
            int s = add_snode(TDF_OP_CE_HEAD, f, -1, -1, 1, 0);   // (h, label, dloss) -> dh
            add_edge(fwd(0), nd.in[0].port, s, 0, 0);
            add_edge(fwd(1), nd.in[1].port, s, 1, 0);
            add_edge(dy, dyp, s, 2, 0);
            push(nd.in[0], s, 0);
            break;
          }
          case TDF_OP_CE_NODE: {
            int s = add_snode(TDF_OP_CE_NODE, f, -1, -1, 1, 0);   // (row, node, drow) -> drow plus the term's gradient
            add_edge(fwd(0), nd.in[0].port, s, 0, 0);
            add_edge(fwd(1), nd.in[1].port, s, 1, 0);
            add_edge(dy, dyp, s, 2, 0);
            push(nd.in[0], s, 0);
            break;
          }
          default: bad("no gradient operator for a node on the differentiable path");
        }
      }
    }
  }

  // ---- 6. device firing tables --------------------------------------------------------
  void compile_device_tables() {
    DevProgram& D = G.prog;
    memset(&D, 0, sizeof(D));
    D.n_fn = P->n_functions;
    D.result_fn = P->result_fn;
    D.n_labels = G.n_labels;
    int n_instr = 0, max_stored = 0, max_sites = 0;
    for (int f = 0; f < P->n_functions; ++f) {
      const auto& fn = F(f);
      std::map<std::pair<int, int>, int> val;   // (node, port) -> value id
      int n_val = 0, n_stored = fn.n_params;
      int first = n_instr;
      auto emit = [&](Instr I, int snode) {
        if (n_instr >= MAX_INSTR) bad("program too large for the device tables");
        if (n_instr - first >= 64) bad("more than 64 firing-table entries in a function");
        D.stat_idx[n_instr] = (uint16_t)snode;
        D.instr[n_instr++] = I;
      };
      auto new_val = [&]() {
        if (n_val >= MAX_VALUES) bad("too many values in a function");
        return n_val++;
      };
      for (int i = 0; i < fn.n_nodes; ++i) {
        const auto& nd = fn.nodes[i];
        if (nd.op == TDF_OP_CONST) continue;
        Instr I;
        memset(&I, 0, sizeof(I));
        for (int k = 0; k < 4; ++k) I.src[k] = SRC_NONE;
        auto set_src = [&](int slot, tdf_ref r) {
          if (is_const(f, r)) {
            I.src[slot] = SRC_IMM;
            I.imm = fn.nodes[r.node].imm;
          } else {
            I.src[slot] = (uint8_t)val.at({r.node, r.port});
          }
        };
        if (nd.op == TDF_OP_NEXT) {
          const auto& cs = call_snodes[{f, i}];
          for (int k = 0; k < nd.n_in; ++k) {
            Instr C = I;
            C.op = D_NEXT;
            C.dst = (uint8_t)new_val();
            C.aux2 = (uint8_t)k;
            if (is_const(f, nd.in[k])) {
              C.src[0] = SRC_IMM;
              C.imm = fn.nodes[nd.in[k].node].imm;
            } else {
              C.src[0] = (uint8_t)val.at({nd.in[k].node, nd.in[k].port});
            }
            emit(C, cs[k]);
          }
          continue;
        }
        const bool is_call = nd.op == TDF_OP_CALLFN || nd.op == TDF_OP_LOOP;
        int sn = is_call || (nd.op == TDF_OP_OUT && f != P->result_fn) ? -1 : smap.at({f, i, 0});
        if (is_call) {
          int lab = label_of[{f, i}];
          const auto& cs = call_snodes[{f, i}];
          for (int k = 0; k < nd.n_in; ++k) {
            Instr C = I;
            C.op = D_CALL;
            C.dst = (uint8_t)new_val();
            C.aux = (uint8_t)lab;
            C.aux2 = (uint8_t)k;
            if (is_const(f, nd.in[k])) {
              C.src[0] = SRC_IMM;
              C.imm = fn.nodes[nd.in[k].node].imm;
            } else {
              C.src[0] = (uint8_t)val.at({nd.in[k].node, nd.in[k].port});
            }
            emit(C, cs[k]);
          }
          Instr R = I;
          R.op = D_RET;
          R.dst = (uint8_t)new_val();
          if (n_stored >= MAX_STORED) bad("too many stored values in a function");
          R.aux = (uint8_t)n_stored++;
          R.aux2 = (uint8_t)lab;
          for (int k = 0; k < nd.n_in; ++k)
            R.src[k] = is_const(f, nd.in[k]) ? SRC_NONE : (uint8_t)val.at({nd.in[k].node, nd.in[k].port});
          val[{i, 0}] = R.dst;
          D.label_callee[lab] = (uint8_t)nd.imm;
          D.label_ret_slot[lab] = R.aux;
          emit(R, smap.at({f, i, 0}));
          continue;
        }
        for (int k = 0; k < nd.n_in; ++k) set_src(k, nd.in[k]);
        switch (nd.op) {
          case TDF_OP_IN: I.op = D_IN; I.aux = (uint8_t)nd.imm; break;
          case TDF_OP_OUT: I.op = D_OUT; I.aux = (uint8_t)type[f][i]; break;
          case TDF_OP_ADD: I.op = D_ADD; break;
          case TDF_OP_SUB: I.op = D_SUB; break;
          case TDF_OP_MUL: I.op = D_MUL; break;
          case TDF_OP_EQ: I.op = D_EQ; break;
          case TDF_OP_LT: I.op = D_LT; break;
          case TDF_OP_ID: I.op = D_ID; break;
          case TDF_OP_SWITCH: I.op = D_SWITCH; break;
          case TDF_OP_MERGE: I.op = D_MERGE; break;
          case TDF_OP_TREE_ISLEAF: I.op = D_ISLEAF; break;
          case TDF_OP_TREE_LEFT: I.op = D_LEFT; break;
          case TDF_OP_TREE_RIGHT: I.op = D_RIGHT; break;
          case TDF_OP_TREE_TOKEN: I.op = D_TOKEN; break;
          case TDF_OP_EMBED: I.op = D_EMBED; break;
          case TDF_OP_RNN_CELL: case TDF_OP_LSTM_CELL: I.op = D_CELL; break;
          case TDF_OP_CE_HEAD: I.op = D_HEAD; break;
          case TDF_OP_CE_NODE: I.op = D_CE_NODE; break;
        }
        if (I.op == D_EMBED || I.op == D_CELL || I.op == D_HEAD) {
          if (n_stored >= MAX_STORED) bad("too many stored values in a function");
          I.aux = (uint8_t)n_stored++;
        }
        if (nd.op != TDF_OP_OUT) {
          I.dst = (uint8_t)new_val();
          val[{i, 0}] = I.dst;
          if (nd.op == TDF_OP_SWITCH) val[{i, 1}] = new_val();
        }
        emit(I, sn < 0 ? 0xFFFF : sn);
      }
      D.fn[f].first = (uint16_t)first;
      D.fn[f].count = (uint16_t)(n_instr - first);
      D.fn[f].n_values = (uint8_t)n_val;
      D.fn[f].n_stored = (uint8_t)n_stored;
      D.fn[f].out_type = (uint8_t)ret_type[f];
      D.fn[f].n_params = (uint8_t)fn.n_params;
      int n_emit = 0;
      for (int q = first; q < n_instr; ++q)
        n_emit += D.instr[q].op == D_CALL || D.instr[q].op == D_OUT || D.instr[q].op == D_NEXT;
      D.fn[f].n_emit = (uint8_t)n_emit;
      // the scopes a frame of f opens (one child link each): its call / loop sites in table order,
      // then the next iteration of a loop graph
      int n_sites = 0;
      bool has_next = false;
      for (int q = first; q < n_instr; ++q) {
        if (D.instr[q].op == D_CALL && D.instr[q].aux2 == 0) D.label_site[D.instr[q].aux] = (uint8_t)n_sites++;
        has_next = has_next || D.instr[q].op == D_NEXT;
      }
      D.fn[f].next_site = (uint8_t)n_sites;
      if (has_next) ++n_sites;
      if (n_sites > MAX_SITES) bad("more than 8 call and loop sites in a function");
      D.fn[f].n_sites = (uint8_t)n_sites;
      if (n_sites > max_sites) max_sites = n_sites;
      if (n_stored > max_stored) max_stored = n_stored;
    }
    // frame record: 32-byte header, the stored values, the child links; records are handed out in
    // creation order, so neighbours are created and completed together
    D.links_off = 32 + 8 * max_stored;
    D.n_links = max_sites;
    // programs with vector operators also keep the instance (the root of the tag) in every frame:
    // the data plane schedules deep instances apart from the others
    const bool vec = G.has_embed || G.cell_kind != 0;
    D.inst_off = vec ? D.links_off + 4 * max_sites : 0;
    D.frame_stride = (D.links_off + 4 * max_sites + (vec ? 4 : 0) + 31) / 32 * 32;
    if ((int)G.snodes.size() > TDF_STATS_MAX_COUNTS) bad("static graph too large for tdf_stats");
  }
};

}  // namespace
}  // namespace tdf

using namespace tdf;

extern "C" tdf_status tdf_graph_build(const tdf_program_desc* prog, int want_grad, tdf_graph** out) {
  if (!out) {
    set_error("tdf_graph_build: out is NULL");
    return TDF_ERR_BAD_ARG;
  }
  *out = nullptr;
  if (!prog) {
    set_error("tdf_graph_build: prog is NULL");
    return TDF_ERR_BAD_ARG;
  }
  tdf_graph* g = new tdf_graph();
  g->g.want_grad = want_grad != 0;
  try {
    Builder b(prog, want_grad != 0, g->g);
    b.validate();
    b.infer_types();
    b.number_calls();
    b.build_static_graph();
    if (want_grad) b.build_gradient_graph();
    b.compile_device_tables();
  } catch (const Bad& e) {
    set_error(std::string("tdf_graph_build: ") + e.msg);
    delete g;
    return TDF_ERR_BAD_PROGRAM;
  } catch (const std::exception& e) {
    set_error(std::string("tdf_graph_build: ") + e.what());
    delete g;
    return TDF_ERR_BAD_PROGRAM;
  }
  *out = g;
  return TDF_OK;
}

extern "C" void tdf_graph_destroy(tdf_graph* g) { delete g; }   // ~tdf_graph is in eval.hip

extern "C" tdf_status tdf_graph_info(const tdf_graph* g, tdf_graph_info_t* out) {
  if (!g || !out) {
    set_error("tdf_graph_info: NULL argument");
    return TDF_ERR_BAD_ARG;
  }
  out->n_nodes = (int32_t)g->g.snodes.size();
  out->n_edges = (int32_t)g->g.sedges.size();
  out->n_labels = g->g.n_labels;
  out->nodes = g->g.snodes.data();
  out->edges = g->g.sedges.data();
  return TDF_OK;
}

extern "C" const char* tdf_last_error(void) { return tdf::g_last_error.c_str(); }
