// Host-only driver for the sanitizer build of the graph compiler (graph_build.cpp): reads program
// descriptions from a text file, builds each through the C ABI, walks the static graph that
// tdf_graph_info returns, destroys the graph, and prints one status line per program.  Compiled by
// tests/test_host_sanitizers.py with -fsanitize=address,undefined; no GPU code is linked.
//
// File format, one program after the other:
//   program <name> <want_grad> <result_fn> <n_functions>
//   function <name> <n_params> <n_nodes>
//   node <op> <imm> <n_in> (<node> <port>)*
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "tdf_internal.h"

tdf_graph::~tdf_graph() {}   // (the library's destructor also releases GPU objects; none exist here)

int main(int argc, char** argv) {
  if (argc < 2) return 2;
  FILE* f = fopen(argv[1], "r");
  if (!f) return 2;
  char word[64], name[128];
  while (fscanf(f, "%63s", word) == 1) {
    if (strcmp(word, "program") != 0) return 3;
    int want_grad = 0, result_fn = 0, n_fn = 0;
    if (fscanf(f, "%127s %d %d %d", name, &want_grad, &result_fn, &n_fn) != 4) return 3;
    std::vector<std::vector<tdf_node_desc>> nodes(n_fn);
    std::vector<std::string> names(n_fn);
    std::vector<tdf_function_desc> fns(n_fn);
    for (int i = 0; i < n_fn; ++i) {
      char fname[128];
      int n_params = 0, n_nodes = 0;
      if (fscanf(f, "%63s %127s %d %d", word, fname, &n_params, &n_nodes) != 4 || strcmp(word, "function") != 0) return 3;
      names[i] = fname;
      nodes[i].resize(n_nodes > 0 ? n_nodes : 0);
      for (int j = 0; j < n_nodes; ++j) {
        tdf_node_desc& nd = nodes[i][j];
        memset(&nd, 0, sizeof(nd));
        long long imm = 0;
        int op = 0, n_in = 0;
        if (fscanf(f, "%63s %d %lld %d", word, &op, &imm, &n_in) != 4 || strcmp(word, "node") != 0) return 3;
        nd.op = op;
        nd.imm = imm;
        nd.n_in = n_in;
        for (int k = 0; k < n_in; ++k) {
          int a = 0, b = 0;
          if (fscanf(f, "%d %d", &a, &b) != 2) return 3;
          if (k < TDF_MAX_INPUTS) { nd.in[k].node = a; nd.in[k].port = b; }
        }
      }
      fns[i].name = names[i].c_str();
      fns[i].n_params = n_params;
      fns[i].n_nodes = n_nodes;
      fns[i].nodes = nodes[i].empty() ? nullptr : nodes[i].data();
    }
    tdf_program_desc prog{n_fn, fns.data(), result_fn};
    tdf_graph* g = nullptr;
    const tdf_status st = tdf_graph_build(&prog, want_grad, &g);
    long long checksum = 0;
    if (st == TDF_OK) {
      tdf_graph_info_t info;
      if (tdf_graph_info(g, &info) != TDF_OK) return 4;
      for (int i = 0; i < info.n_nodes; ++i) checksum += info.nodes[i].kind + info.nodes[i].label + info.nodes[i].imm;
      for (int i = 0; i < info.n_edges; ++i) {
        if (info.edges[i].src < 0 || info.edges[i].src >= info.n_nodes || info.edges[i].dst < 0 || info.edges[i].dst >= info.n_nodes) return 5;
        checksum += info.edges[i].src * 3 + info.edges[i].dst;
      }
      // the firing tables the device would run: every entry inside its function's range
      const tdf::DevProgram& P = g->g.prog;
      for (int fi = 0; fi < P.n_fn; ++fi)
        for (int q = P.fn[fi].first; q < P.fn[fi].first + P.fn[fi].count; ++q) checksum += P.instr[q].op + P.stat_idx[q];
      printf("%s %d nodes %d edges %d labels %d stride %d checksum %lld\n", name, (int)st, info.n_nodes, info.n_edges, info.n_labels,
             P.frame_stride, checksum);
      tdf_graph_destroy(g);
    } else {
      printf("%s %d %s\n", name, (int)st, tdf_last_error());
    }
  }
  fclose(f);
  // NULL arguments are errors, not crashes
  tdf_graph* g = nullptr;
  if (tdf_graph_build(nullptr, 0, &g) != TDF_ERR_BAD_ARG || tdf_graph_build(nullptr, 0, nullptr) != TDF_ERR_BAD_ARG) return 6;
  if (tdf_graph_info(nullptr, nullptr) != TDF_ERR_BAD_ARG) return 6;
  tdf_graph_destroy(nullptr);
  return 0;
}
