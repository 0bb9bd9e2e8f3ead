// Firing tables shared by the host compiler (graph_build.cpp), the device engine and the
// run-time generated sweeps.  No standard-library includes: this header is also compiled by
// the run-time compiler.
#pragma once
#include <stdint.h>

#include "tdf.h"

namespace tdf {

// ---- device firing tables -------------------------------------------------------------
// Every function graph is compiled into a straight-line table of instructions in
// topological order.  One lane evaluates the table for one frame (= one call-context tag):
// an instruction fires when all its source values are present under that tag (the firing
// rule of Section 2.2).  Values that arrive from other tags (arguments pushed by Call_i,
// results popped by Return_i) and row references of vector operators are kept in the frame
// record; everything else is recomputed from them on each sweep.
enum DevOp : uint8_t {
  D_IN = 0,   // aux = stored slot (= parameter index)
  D_RET,      // Return_i seen from the caller: aux = stored slot, aux2 = label,
              // src[] = argument values of the call (dead arguments => dead result)
  D_ADD, D_SUB, D_MUL, D_EQ, D_LT, D_ID,
  D_SWITCH,   // dst = true side, dst+1 = false side; src[0] = predicate, src[1] = data
  D_MERGE,
  D_CALL,     // Call_i for one parameter: src[0] = argument, aux = label, aux2 = parameter
              // (also the Enter of one loop variable: it pushes iteration counter 0)
  D_OUT,      // function output: emits the Return token (or writes the program output)
  D_ISLEAF, D_LEFT, D_RIGHT, D_TOKEN,
  D_EMBED,    // aux = stored slot of the row reference
  D_CELL,     // aux = stored slot
  D_HEAD,     // aux = stored slot
  D_NEXT,     // Next of one loop variable: src[0] = value, aux2 = variable
  D_CE_NODE,  // src[0] = row reference (handed on), src[1] = tree node whose loss term the row gets
};

constexpr uint8_t SRC_IMM = 0xFF;   // source is the instruction's immediate
constexpr uint8_t SRC_NONE = 0xFE;

struct Instr {
  uint8_t op, dst, aux, aux2;
  uint8_t src[4];
  int64_t imm;
};
static_assert(sizeof(Instr) == 16, "Instr must be 16 bytes");

constexpr int MAX_FN = 8;
constexpr int MAX_INSTR = 176;
constexpr int MAX_LABELS = 32;
constexpr int MAX_VALUES = 64;   // per function
constexpr int MAX_STORED = 24;   // per function
constexpr int MAX_SITES = 8;     // per function: call sites, loop sites, next iteration

enum ValueType : uint8_t { T_INT = 0, T_VEC = 1, T_LOSS = 2 };

struct DevFn {
  uint16_t first, count;   // instruction range
  uint8_t n_values, n_stored, out_type, n_params;
  uint8_t n_emit;          // entries that emit a token (Call_i per parameter, function output)
  uint8_t n_sites;         // scopes a frame of this function can open: its call and loop sites, plus
                           // the next iteration if it is a loop graph (at most MAX_SITES)
  uint8_t next_site;       // loop graphs: the site of the next iteration (= number of call sites)
  uint8_t pad[5];
};

// Lives in the workspace; every workgroup of a step kernel copies it into LDS.
struct DevProgram {
  int32_t n_fn, result_fn, n_labels, frame_stride;   // frame_stride in bytes
  int32_t links_off, n_links;           // frame record: byte offset and number of the child links (program-wide)
  int32_t inst_off, pad0;               // frame record: byte offset of the instance index the tag belongs to
                                        // (programs with vector operators; 0: not kept)
  DevFn fn[MAX_FN];
  uint8_t label_callee[MAX_LABELS];     // function entered by Call_i
  uint8_t label_ret_slot[MAX_LABELS];   // stored slot of Return_i's value in the caller's frame
  uint8_t label_site[MAX_LABELS];       // which of the caller's child links belongs to the scope opened by Call_i
  uint16_t stat_idx[MAX_INSTR];         // static-graph node counted when the instruction fires live
  Instr instr[MAX_INSTR];
};
static_assert(sizeof(DevProgram) <= 4096, "DevProgram is copied into LDS by every workgroup");

}  // namespace tdf
