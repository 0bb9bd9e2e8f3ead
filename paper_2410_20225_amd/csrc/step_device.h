// Device side of the tag machine: one step = one pass over the frames that received a token.
//
//   fire    one lane per frame (= per call-context tag) evaluates the firing table of the
//           frame's function; an entry fires when its sources are present under that tag
//           (Section 2.2: all inputs hold tokens with the same tag).  Dead values (hiatons)
//           propagate; Switch, Merge and dead calls follow the paper's equations.
//   match   the tokens a sweep emits are delivered right after it:
//           Call_i  <t,d> -> <i:t,d>: find-or-insert the entry (frame of t, i) of the match
//                   table, which is the child link of call site i in the frame of t (Section 3;
//                   Section 5.1: a new frame that stores the label i), and write the argument
//                   into that frame;
//           Return_i <i:t,d> -> <t,d>: the frame's own key names its label i and the frame of
//                   t, which is the label check of Section 5.1 (only the Return_i of the call
//                   that created the frame produces output); the value goes to the caller's
//                   frame.
//   compact the first token that reaches a frame in a step puts it on the next step's list;
//           list and log entries are staged in LDS (wave ballot + prefix sum) and the
//           workgroup reserves its range of each global list with one atomic per pass.
//
// A frame that is being swept may receive a token in the same step from another lane.  Such
// a token sets a bit in the frame's arrival word of the *next* step and puts the frame on the
// next list; the running sweep neither sees the bit nor reads the value.  Only the key and
// the arrival words are written concurrently, with atomics.
//
// The sweep itself is a policy: the table interpreter below, or straight-line code generated
// from the firing tables by the run-time compiler (jit.cpp).  Both use the same helpers.
#pragma once
#include "die_sync.h"
#include "engine.h"

namespace tdf {

__device__ __forceinline__ void raise(Ctrl* c, int status) {
  atomicCAS(&c->status, 0u, (uint32_t)(-status));
}

template <typename T> __device__ __forceinline__ T ld(const T* p) { return __atomic_load_n(p, __ATOMIC_RELAXED); }
template <typename T> __device__ __forceinline__ void st(T* p, T v) { __atomic_store_n(p, v, __ATOMIC_RELAXED); }

// Atomics on frame words at the scope of the running kernel: device scope when the whole grid
// works on a step, workgroup scope when a single workgroup does (its atomics then stay in the
// local L2; kernel boundaries make them visible to whoever runs the next step).
template <int SCOPE> __device__ __forceinline__ uint32_t a_or(uint32_t* p, uint32_t v) {
  return __hip_atomic_fetch_or(p, v, __ATOMIC_RELAXED, SCOPE);
}
template <int SCOPE> __device__ __forceinline__ uint32_t a_exch(uint32_t* p, uint32_t v) {
  return __hip_atomic_exchange(p, v, __ATOMIC_RELAXED, SCOPE);
}
// Reads of data that another compute unit of the same die may have rewritten since this one
// last read it (frame records, which are swept again and again, and the touched lists, whose
// storage is reused every other step).  COHERENT: a device-scope load, which goes past this
// CU's L1 to the die's L2, where the other CU's store is.  An L1 invalidation per step would do
// too, but its workgroup-scope form does not drop these lines and its device-scope form also
// drops the L2's.
template <bool COHERENT, typename T> __device__ __forceinline__ T ld_shared(const T* p) {
  if (COHERENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return *p;
}

template <int SCOPE> __device__ __forceinline__ unsigned long long a_ld(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, SCOPE);
}
template <int SCOPE> __device__ __forceinline__ unsigned long long a_cas(unsigned long long* p, unsigned long long expect,
                                                                        unsigned long long v) {
  __hip_atomic_compare_exchange_strong(p, &expect, v, __ATOMIC_RELAXED, __ATOMIC_RELAXED, SCOPE);
  return expect;
}

// Per-workgroup staging of one pass.
struct Stage {
  uint32_t n_touched, n_leaf, n_cell, n_head, n_tags, n_tokens;
  uint32_t max_depth, max_level;
  uint32_t base_touched, base_leaf, base_cell;
};

struct Sizes {
  int max_values, max_stored, max_emit;
};
__host__ __device__ inline Sizes sizes_of(const DevProgram& P) {
  Sizes z{1, 1, 1};
  for (int f = 0; f < P.n_fn; ++f) {
    z.max_values = z.max_values > P.fn[f].n_values ? z.max_values : P.fn[f].n_values;
    z.max_stored = z.max_stored > P.fn[f].n_stored ? z.max_stored : P.fn[f].n_stored;
    z.max_emit = z.max_emit > P.fn[f].n_emit ? z.max_emit : P.fn[f].n_emit;
  }
  return z;
}
// Dynamic LDS of a step kernel with `rb` lanes: value file (LDS sweeps only), cell / leaf /
// touched staging, and the tokens a sweep has emitted but not yet delivered.
__host__ __device__ inline size_t step_lds_bytes(const Sizes& z, int rb, bool lds_values) {
  const size_t vals = lds_values ? (size_t)(z.max_values + z.max_stored) * 8 : 0;
  return (size_t)rb * (vals + (size_t)z.max_emit * (4 + 8 + 4) + 8 + 16) + sizeof(Stage);
}

// ---- what a sweep sees of its lane ------------------------------------------------------------
struct LaneCtx {
  const Engine* e;
  Ctrl* c;
  Stage* S;
  uint4* stg_cell;
  uint2* stg_leaf;
  long long* pend_val;     // [emission][lane]
  uint32_t* pend_meta;
  long long* lds_vals;     // LDS value file [value][lane] then [stored][lane] (LDS sweeps only)
  int lds_stored_base;     // first stored row in lds_vals
  int RB, tid;
  bool direct;             // single-workgroup run: list and log entries go straight to the global arrays
  bool active;
  uint32_t frame;
  int myfn, result_fn;
  long long* slots;        // stored values of the frame (global memory)
  unsigned long long fired;
  uint32_t present;
  int n_pend;
  long long sv[8];         // the first eight stored values, loaded before the sweep
  uint32_t links[MAX_SITES];   // the frame's child links (frame id + 1, 0 = scope not opened), loaded before the sweep
  uint32_t inst;           // instance the tag belongs to (programs with vector operators)
  bool complete;           // set by the sweep: every value that reaches this tag from another tag (parameters,
                           // results of its calls and loops) has arrived or is known never to come, so
                           // everything in the body has fired and no token can reach the frame any more
  uint32_t mx_level;       // largest cell level this lane produced in the pass
  long long tc_v;          // forest entries of the last node looked at
  int tc_left, tc_right, tc_token;
};

// ---- helpers shared by the interpreter and by generated sweeps ----------------------------------
// The token emitted by a Call_i entry (meta = 0x80000000 | label | param << 8), by a Next entry
// (meta = 0xC0000000 | variable << 8) or by the function output (meta = 0: the Return token, or
// the Exit token of a loop graph); delivered after the sweep.
__device__ __forceinline__ void sw_emit(LaneCtx& x, bool go, uint32_t meta, long long v) {
  if (go) {
    x.pend_val[x.n_pend * x.RB + x.tid] = v;
    x.pend_meta[x.n_pend * x.RB + x.tid] = meta;
    ++x.n_pend;
  }
}
// output of `result`
__device__ __forceinline__ void sw_result(LaneCtx& x, bool go, int type, long long v) {
  if (go) {
    const uint32_t b = x.frame - x.e->cap;
    if (type == T_INT) { if (x.e->out_i64) x.e->out_i64[b] = v; }
    else if (type == T_VEC) {
      x.e->root_ref[b] = (uint32_t)v;
      x.e->root_lvl[b] = (uint32_t)(v >> 32);
    }
  }
}
// forest accessors at node index v: which = 0 isleaf, 1 left, 2 right, 3 token; sets `dead` and
// raises an error for an index outside the forest
__device__ __forceinline__ long long sw_tree(LaneCtx& x, long long v, int which, bool& dead) {
  const Engine& e = *x.e;
  if (v < 0 || v >= e.n_tree_nodes || e.left == nullptr) {
    raise(x.c, TDF_ERR_BAD_ARG);
    dead = true;
    return 0;
  }
  if (x.tc_v != v) {   // one round trip serves isleaf / left / right / token of the same node
    x.tc_left = e.left[v];
    x.tc_right = e.right[v];
    x.tc_token = e.token[v];
    x.tc_v = v;
  }
  return which == 0 ? (long long)(x.tc_left < 0) : which == 1 ? x.tc_left : which == 2 ? x.tc_right : x.tc_token;
}
// CE_NODE: the row (= frame that produced the state) is marked with the tree node whose loss term
// it gets; the row reference goes on unchanged.  Repeated by later sweeps of the frame with the
// same values.
__device__ __forceinline__ void sw_ce_node(LaneCtx& x, long long row, long long v, bool& dead) {
  const Engine& e = *x.e;
  if (v < 0 || v >= e.n_tree_nodes || e.row_node == nullptr) {
    raise(x.c, TDF_ERR_BAD_ARG);
    dead = true;
    return;
  }
  e.row_node[(uint32_t)row] = (uint32_t)v;
}
// EMBED: the leaf's state row is the row of this frame, level 0.  Whole wave must call.
__device__ __forceinline__ void sw_embed(LaneCtx& x, bool on, int slot, long long stored, bool ap, bool ad, long long av,
                                         long long& v, bool& p, bool& live) {
  const bool had = on && ((x.present >> slot) & 1);
  const bool go = on && ap && !ad && !had;
  const bool ok = go && av >= 0 && av < (long long)x.e->vocab;
  if (go && !ok) raise(x.c, TDF_ERR_BAD_ARG);   // token id outside the embedding table
  const uint32_t pos = wave_alloc(ok, x.direct ? &x.c->n_leaf : &x.S->n_leaf);
  if (ok) {
    if (!x.direct) {
      x.stg_leaf[pos] = make_uint2(x.frame, (uint32_t)av);
    } else if (pos < x.e->log_cap) {
      x.e->leaf_row[pos] = x.frame;
      x.e->leaf_tok[pos] = (uint32_t)av;
    } else {
      raise(x.c, TDF_ERR_TABLE_FULL);
    }
    x.slots[slot] = (long long)x.frame;
    x.present |= 1u << slot;
  }
  v = had ? stored : (long long)x.frame;
  p = had || ok;
  live = p;
}
// RNN / LSTM cell: appended to the schedule log with its dependency level.  Whole wave must call.
__device__ __forceinline__ void sw_cell(LaneCtx& x, bool on, int slot, long long stored, bool ap, bool ad, long long av,
                                        bool bp, bool bd, long long bv, long long& v, bool& p, bool& live) {
  const bool had = on && ((x.present >> slot) & 1);
  const bool go = on && ap && bp && !ad && !bd && !had;
  const uint32_t pos = wave_alloc(go, x.direct ? &x.c->n_cell : &x.S->n_cell);
  long long r = stored;
  if (go) {
    const uint32_t la = (uint32_t)(av >> 32), lb = (uint32_t)(bv >> 32);
    const uint32_t lvl = 1 + (la > lb ? la : lb);
    if (!x.direct) {
      x.stg_cell[pos] = make_uint4(x.frame, (uint32_t)av, (uint32_t)bv, lvl * LEVEL_KEY_DIES + x.e->die);
    } else if (pos < x.e->log_cap) {
      x.e->cell_out[pos] = x.frame;
      x.e->cell_l[pos] = (uint32_t)av;
      x.e->cell_r[pos] = (uint32_t)bv;
      x.e->cell_lvl[pos] = lvl * LEVEL_KEY_DIES + x.e->die;
    } else {
      raise(x.c, TDF_ERR_TABLE_FULL);
    }
    r = (long long)x.frame | ((long long)lvl << 32);
    x.slots[slot] = r;
    x.present |= 1u << slot;
    x.mx_level = lvl > x.mx_level ? lvl : x.mx_level;
  }
  v = r;
  p = had || go;
  live = p;
}
// CE_HEAD of `result`
__device__ __forceinline__ void sw_head(LaneCtx& x, bool on, int slot, bool ap, bool ad, long long av, bool bp, bool bd,
                                        long long bv, long long& v, bool& p, bool& live) {
  const bool had = on && ((x.present >> slot) & 1);
  const bool go = on && ap && bp && !ad && !bd && !had && x.myfn == x.result_fn;
  if (go) {
    const uint32_t inst = x.frame - x.e->cap;
    x.e->head_row[inst] = (uint32_t)av;
    x.e->root_lvl[inst] = (uint32_t)(av >> 32);
    x.e->head_label[inst] = (uint32_t)bv;
    x.slots[slot] = inst;
    x.present |= 1u << slot;
  }
  wave_count32(go, x.direct ? &x.c->n_head : &x.S->n_head);
  v = (long long)(x.frame - x.e->cap);
  p = had || go;
  live = p;
}

// ---- the table interpreter -------------------------------------------------------------------
// NV > 0: the value file of a sweep (at most NV values, 8 stored values) lives in registers,
// indexed with the wave-uniform value ids of the firing table; NV == 0: it lives in LDS.
__device__ __forceinline__ uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ Instr fetch(const DevProgram& P, int idx) {
  union { Instr i; uint32_t w[4]; } u;
  u.i = P.instr[idx];
#pragma unroll
  for (int k = 0; k < 4; ++k) u.w[k] = uni(u.w[k]);
  return u.i;
}

struct Src {
  long long v;
  bool p, d;   // present, dead
};

template <int NV>
struct InterpSweep {
  static constexpr bool kLdsValues = NV == 0;
  static __device__ void run(LaneCtx& x, const DevProgram& P) {
    const int RB = x.RB, tid = x.tid;
    long long rloc[NV > 0 ? NV : 1];
    auto rd = [&](int idx) -> long long {
      if constexpr (NV > 0) return rloc[idx]; else return x.lds_vals[idx * RB + tid];
    };
    auto wr = [&](int idx, long long v) {
      if constexpr (NV > 0) rloc[idx] = v; else x.lds_vals[idx * RB + tid] = v;
    };
    auto rd_st = [&](int idx) -> long long {
      if constexpr (NV > 0) return x.sv[idx]; else return x.lds_vals[(x.lds_stored_base + idx) * RB + tid];
    };
    const int n_fn = (int)uni((uint32_t)P.n_fn);
    for (int f = 0; f < n_fn; ++f) {
      const bool on = x.myfn == f;
      if (__ballot(on) == 0) continue;
      const int first_i = (int)uni(P.fn[f].first), count = (int)uni(P.fn[f].count);
      const bool is_result = f == x.result_fn;
      unsigned long long pres = 0, dead = 0;   // over value ids
      bool all_in = true;                       // every D_IN / D_RET entry is resolved
      Instr I_next = fetch(P, first_i);
      for (int ip = 0; ip < count; ++ip) {
        const Instr I = I_next;
        if (ip + 1 < count) I_next = fetch(P, first_i + ip + 1);   // fetched while this entry runs
        const unsigned long long ibit = 1ull << ip;
        auto src = [&](int k) -> Src {
          const uint8_t s = I.src[k];
          if (s == SRC_IMM) return Src{I.imm, true, false};
          return Src{rd(s), ((pres >> s) & 1) != 0, ((dead >> s) & 1) != 0};
        };
        auto put = [&](int dst, long long v, bool p, bool d) {
          wr(dst, v);
          if (p) pres |= 1ull << dst;
          if (d) dead |= 1ull << dst;
        };
        bool live = false;   // this entry holds a live value under this tag
        switch (I.op) {
          case D_IN: {
            const bool p = on && ((x.present >> I.aux) & 1);
            put(I.dst, rd_st(I.aux), p, false);
            live = p;
            all_in = all_in && p;
            break;
          }
          case D_RET: {
            const bool p = on && ((x.present >> I.aux) & 1);
            bool all_p = true, any_d = false, any_arg = false;
            for (int k = 0; k < 4; ++k) {
              if (I.src[k] == SRC_NONE) continue;
              any_arg = true;
              all_p = all_p && ((pres >> I.src[k]) & 1);
              any_d = any_d || ((dead >> I.src[k]) & 1);
            }
            const bool is_dead = on && !p && any_arg && all_p && any_d;   // the call never happened
            put(I.dst, rd_st(I.aux), p || is_dead, is_dead);
            live = p;
            all_in = all_in && (p || is_dead);
            break;
          }
          case D_ADD: case D_SUB: case D_MUL: case D_EQ: case D_LT: {
            const Src a = src(0), b = src(1);
            const bool p = on && a.p && b.p, d = a.d || b.d;
            const unsigned long long ua = (unsigned long long)a.v, ub = (unsigned long long)b.v;
            long long r = 0;
            if (I.op == D_ADD) r = (long long)(ua + ub);
            else if (I.op == D_SUB) r = (long long)(ua - ub);
            else if (I.op == D_MUL) r = (long long)(ua * ub);
            else if (I.op == D_EQ) r = a.v == b.v;
            else r = a.v < b.v;
            put(I.dst, r, p, p && d);
            live = p && !d;
            break;
          }
          case D_ID: {
            const Src a = src(0);
            put(I.dst, a.v, on && a.p, on && a.p && a.d);
            live = on && a.p && !a.d;
            break;
          }
          case D_ISLEAF: case D_LEFT: case D_RIGHT: case D_TOKEN: {
            const Src a = src(0);
            const bool p = on && a.p;
            bool d = a.d;
            long long r = 0;
            if (p && !d) r = sw_tree(x, a.v, I.op - D_ISLEAF, d);
            put(I.dst, r, p, p && d);
            live = p && !d;
            break;
          }
          case D_CE_NODE: {
            const Src a = src(0), b = src(1);
            const bool p = on && a.p && b.p;
            bool d = a.d || b.d;
            if (p && !d) sw_ce_node(x, a.v, b.v, d);
            put(I.dst, a.v, p, p && d);
            live = p && !d;
            break;
          }
          case D_SWITCH: {
            const Src pr = src(0), da = src(1);
            const bool p = on && pr.p && da.p, d = pr.d || da.d;
            const bool t = pr.v != 0;
            put(I.dst, da.v, p, p && (d || !t));
            put(I.dst + 1, da.v, p, p && (d || t));
            live = p && !d;
            break;
          }
          case D_MERGE: {
            bool any_live = false, all_p = true;
            long long r = 0;
            for (int k = 0; k < 4; ++k) {
              if (I.src[k] == SRC_NONE) continue;
              const Src a = src(k);
              if (a.p && !a.d && !any_live) {
                any_live = true;
                r = a.v;
              }
              all_p = all_p && a.p;
            }
            const bool p = on && (any_live || all_p);
            put(I.dst, r, p, p && !any_live);
            live = on && any_live;
            break;
          }
          case D_CALL: {
            const Src a = src(0);
            sw_emit(x, on && a.p && !a.d && !(x.fired & ibit), 0x80000000u | I.aux | ((uint32_t)I.aux2 << 8), a.v);
            live = on && a.p && !a.d;
            break;
          }
          case D_NEXT: {
            const Src a = src(0);
            sw_emit(x, on && a.p && !a.d && !(x.fired & ibit), 0xC0000000u | ((uint32_t)I.aux2 << 8), a.v);
            live = on && a.p && !a.d;
            break;
          }
          case D_OUT: {
            const Src a = src(0);
            const bool go = on && a.p && !a.d && !(x.fired & ibit);
            if (is_result) sw_result(x, go, I.aux, a.v);
            else sw_emit(x, go, 0u, a.v);
            live = on && a.p && !a.d;
            break;
          }
          case D_EMBED: {
            const Src a = src(0);
            long long v;
            bool p;
            sw_embed(x, on, I.aux, rd_st(I.aux), a.p, a.d, a.v, v, p, live);
            put(I.dst, v, p, false);
            break;
          }
          case D_CELL: {
            const Src a = src(0), b = src(1);
            long long v;
            bool p;
            sw_cell(x, on, I.aux, rd_st(I.aux), a.p, a.d, a.v, b.p, b.d, b.v, v, p, live);
            put(I.dst, v, p, false);
            break;
          }
          case D_HEAD: {
            const Src a = src(0), b = src(1);
            long long v;
            bool p;
            sw_head(x, on, I.aux, a.p, a.d, a.v, b.p, b.d, b.v, v, p, live);
            put(I.dst, v, p, false);
            break;
          }
          default: break;
        }
        if (live) x.fired |= ibit;   // counted after the run, from the fired masks
      }
      if (on) x.complete = all_in;
    }
  }
};

// A token emitted by a sweep, while it is being delivered.
struct Emission {
  bool has, is_call;   // is_call: the token opens or finds a scope (Call_i, Enter, Next)
  uint32_t target, slot, bits, callee, depth, site, res;
  unsigned long long ckey;
  long long val;
};

__device__ __forceinline__ void load_program(DevProgram* dst, const DevProgram* src) {
  const uint32_t* s = reinterpret_cast<const uint32_t*>(src);
  uint32_t* d = reinterpret_cast<uint32_t*>(dst);
  for (int i = threadIdx.x; i < (int)(sizeof(DevProgram) / 4); i += blockDim.x) d[i] = s[i];
  __syncthreads();
}

// One pass over the touched frames [0, n) of the current list; lane `first + tid` takes frames
// i, i + lane_stride, ...  `c` is the control block the pass counts in: the global one, or a
// workgroup's LDS copy.  The loop over passes is uniform for the workgroup.
template <int SCOPE, bool kDirect, class SW>
__device__ void step_pass(const DevProgram& P, const Engine& e, Ctrl* c, uint32_t step, uint32_t n,
                          uint32_t first, uint32_t lane_stride, char* lds) {
  const int tid = threadIdx.x;
  const int RB = blockDim.x;
  Sizes z = sizes_of(P);
  const int n_st = z.max_stored;
  if (!SW::kLdsValues) z.max_values = z.max_stored = 0;   // no LDS value file
  long long* lds_vals = reinterpret_cast<long long*>(lds);
  uint4* stg_cell = reinterpret_cast<uint4*>(lds_vals + (size_t)(z.max_values + z.max_stored) * RB);
  uint2* stg_leaf = reinterpret_cast<uint2*>(stg_cell + RB);
  long long* pend_val = reinterpret_cast<long long*>(stg_leaf + RB);   // [max_emit][lane]
  uint32_t* pend_meta = reinterpret_cast<uint32_t*>(pend_val + (size_t)z.max_emit * RB);
  uint32_t* stg_touched = pend_meta + (size_t)z.max_emit * RB;         // [max_emit * RB]
  Stage* S = reinterpret_cast<Stage*>(stg_touched + (size_t)z.max_emit * RB);
  const int stride = (int)uni((uint32_t)P.frame_stride);
  const int links_off = (int)uni((uint32_t)P.links_off), n_links = (int)uni((uint32_t)P.n_links);
  const int inst_off = (int)uni((uint32_t)P.inst_off);
  const uint32_t* cur_list = e.touched + (size_t)(step & 1) * e.touched_cap;
  uint32_t* next_list = e.touched + (size_t)((step & 1) ^ 1) * e.touched_cap;
  uint32_t* next_count = &c->touched_count[(step & 1) ^ 1];
  const uint32_t word = step & 1;    // arrival word of the next step (this step reads word ^ 1)

  // kDirect: one workgroup alone (its control block `c` is in LDS): positions in the global lists
  // come straight from the counters in `c`, without staging and without barriers between passes.
  // several compute units of one die on one machine: see ld_shared
  constexpr bool kCoherent = SCOPE == __HIP_MEMORY_SCOPE_WORKGROUP && !kDirect;
  uint32_t cnt_tags = 0, cnt_tokens = 0;   // per wave, wave-uniform

  for (uint32_t base = first; base < n; base += lane_stride) {
    if (!kDirect) {
      if (tid == 0) *S = Stage{};
      __syncthreads();
    }
    LaneCtx x;
    x.direct = kDirect;
    x.e = &e; x.c = c; x.S = S;
    x.stg_cell = stg_cell; x.stg_leaf = stg_leaf; x.pend_val = pend_val; x.pend_meta = pend_meta;
    x.lds_vals = lds_vals; x.lds_stored_base = z.max_values;
    x.RB = RB; x.tid = tid;
    const uint32_t i = base + tid;
    x.active = i < n;
    x.frame = x.active ? ld_shared<kCoherent>(&cur_list[i]) : 0;
    if (x.frame >= e.cap + e.n_inst) {   // never true for a list this engine wrote
      raise(c, TDF_ERR_DEVICE);
      x.active = false;
      x.frame = 0;
    }
    x.result_fn = (int)uni((uint32_t)P.result_fn);
    FrameHdr* h = frame_at(e, stride, x.frame);
    x.slots = frame_slots(h);
    x.fired = 0; x.present = 0; x.myfn = -1; x.n_pend = 0; x.tc_v = -1; x.mx_level = 0;
    uint32_t mx_depth = 0;
    x.tc_left = x.tc_right = x.tc_token = 0;
    unsigned long long key = 0;
    uint32_t depth = 0, pf_in = 0;
    if (x.active) {
      // tokens that arrived for this step; the word of the other parity belongs to the next
      const uint32_t arr = a_exch<SCOPE>(&h->arrived[word ^ 1], 0u);
      pf_in = ld_shared<kCoherent>(&h->present_fn);
      key = ld_shared<kCoherent>(&h->key);
      x.fired = ld_shared<kCoherent>(&h->fired);
      const uint32_t pf = pf_in | arr;
      depth = ld_shared<kCoherent>(&h->depth);
      x.present = pf & 0xFFFFFFu;
      x.myfn = (int)(pf >> 24);
    }
    unsigned long long fired_in = x.fired;
#pragma unroll
    for (int k = 0; k < MAX_SITES; ++k)
      x.links[k] = (x.active && k < n_links) ? ld_shared<kCoherent>(&frame_links(h, links_off)[k]) : 0u;
    x.inst = (x.active && inst_off) ? ld_shared<kCoherent>(frame_links(h, inst_off)) : 0u;
    // stored values (meaningful where the present bit is set), all loads in flight at once
#pragma unroll
    for (int k = 0; k < 8; ++k) x.sv[k] = (x.active && k < n_st) ? ld_shared<kCoherent>(&x.slots[k]) : 0;
    if (SW::kLdsValues) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k < n_st) lds_vals[(z.max_values + k) * RB + tid] = x.sv[k];
      for (int k = 8; k < n_st; ++k) lds_vals[(z.max_values + k) * RB + tid] = x.active ? ld_shared<kCoherent>(&x.slots[k]) : 0;
    }

    // A lane that creates the frame of a one-parameter call goes on with that frame in the same
    // step instead of putting it on the next list (kDirect only): nobody else can reach a fresh
    // frame, its only argument is at hand, so its first sweep needs no loads of the header.  A
    // chain of such calls is descended by one lane at two round trips per call instead of one
    // step per call.  Of several calls of one sweep the lane follows the first and lists the
    // others, so the descent that gets shorter is the one along first calls (f(n-1) of fib, the
    // left spine of a tree).  While the machine's steps still grow, all descents advance together
    // one call per step anyway and a long sweep would only hold the others up: lanes follow only
    // in a step with exactly as many frames as the two steps before (chains descending side by
    // side) or with fewer, once the steps are down to a quarter of the machine's largest (the tail
    // of a batch, where the deep stragglers decide the number of steps).  Bounded, so that a
    // recursion without a base case still meets the step limit.
    constexpr int FOLLOW_DEPTH = 256;
    const bool may_follow = kDirect && n <= e.follow_limit &&
                            ((n == c->prev_count && c->same_steps >= 1u) || (n < c->prev_count && n * 4u <= c->peak_count));
    for (int follow = 0;; ++follow) {
    bool has_next = false;
    uint32_t nx_frame = 0, nx_bits = 0, nx_slot = 0, nx_depth = 0;
    unsigned long long nx_key = 0;
    long long nx_val = 0;

    x.complete = false;
    SW::run(x, P);   // ---- fire

    // ---- match: deliver the emitted tokens, two at a time so that their atomics overlap ------
    for (int e0 = 0; __ballot(x.active && e0 < x.n_pend) != 0; e0 += 2) {
      Emission em[2];
      bool fresh[2];   // the token opens its scope: a new frame record is taken
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        Emission& m = em[q];
        m = Emission{};
        fresh[q] = false;
        m.has = x.active && e0 + q < x.n_pend;
        if (m.has) {
          const uint32_t meta = pend_meta[(e0 + q) * RB + tid];
          m.val = pend_val[(e0 + q) * RB + tid];
          m.is_call = (meta >> 31) != 0;
          if (m.is_call) {
            const uint32_t label = meta & 0xFFu, param = (meta >> 8) & 0xFFu;
            if ((meta >> 30) & 1u) {   // Next <n:t,d> = <(n+1):t,d>: same scope, same parent, counter + 1
              m.callee = (uint32_t)x.myfn;
              m.ckey = key + 0x100ull;
              m.depth = depth;
              m.site = P.fn[x.myfn].next_site;
              if (((key >> 8) & 0xFFFFFFull) == 0xFFFFFFull) {   // the counter has 24 bits
                raise(c, TDF_ERR_STEP_LIMIT);
                m.has = false;
              }
            } else {                   // Call_i <t,d> = <i:t,d>, Enter <t,d> = <0:t,d>
              m.callee = P.label_callee[label];
              m.ckey = ((unsigned long long)(x.frame + 1u) << 32) | (label + 1u);
              m.depth = depth + 1u;
              m.site = P.label_site[label];
            }
            m.slot = param;
            m.bits = (1u << param) | (m.callee << 24);
            // the match: the entry for (frame of t, i) is this frame's link of the site
            uint32_t link = 0;
#pragma unroll
            for (int k = 0; k < MAX_SITES; ++k) link = (uint32_t)k == m.site ? x.links[k] : link;
            m.target = link - 1u;
            fresh[q] = m.has && link == 0u;
          } else {
            m.target = (uint32_t)(key >> 32) - 1u;
            m.slot = P.label_ret_slot[(((uint32_t)key & 0xFFu) - 1u) & (MAX_LABELS - 1)];
            m.bits = 1u << m.slot;
            if (m.target >= e.cap + e.n_inst) {   // never true for a key this engine wrote
              raise(c, TDF_ERR_DEVICE);
              m.has = false;
            }
          }
        }
      }
      // two parameters of one call: the second token follows the first into its frame
      const bool same_call = em[0].has && em[1].has && em[0].is_call && em[1].is_call && em[0].ckey == em[1].ckey;
      if (same_call) fresh[1] = false;
      // new scopes take the machine's next free records: one counter bump per wave
      {
        uint32_t pos[2];
        wave_take_frames<kDirect ? __HIP_MEMORY_SCOPE_WORKGROUP : SCOPE>(fresh[0], fresh[1], &c->n_alloc, &c->free_head, &c->free_limit,
                                                                         e.reclaim ? e.free_ring : nullptr, e.part, pos[0], pos[1]);
#pragma unroll
        for (int q = 0; q < 2; ++q)
          if (fresh[q]) {
            if (pos[q] < e.part) {
              em[q].target = e.key_base + pos[q];
#pragma unroll
              for (int k = 0; k < MAX_SITES; ++k)
                if ((uint32_t)k == em[q].site) x.links[k] = em[q].target + 1u;
              frame_links(h, links_off)[em[q].site] = em[q].target + 1u;   // read again by later sweeps of this frame
            } else {
              raise(c, TDF_ERR_TABLE_FULL);
              em[q].has = false;
              fresh[q] = false;
            }
          }
        if (same_call) {
          em[1].has = em[0].has;       // em[0] failed only if the machine's part is full
          em[1].target = em[0].target;
        }
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {   // values and arrival bits, both tokens' atomics in flight
        Emission& m = em[q];
        if (m.has) {
          FrameHdr* th = frame_at(e, stride, m.target);
          frame_slots(th)[m.slot] = m.val;                    // read in a later step only
          if (!m.is_call) m.res = a_or<SCOPE>(&th->arrived[word], m.bits);
        }
      }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        Emission& m = em[q];
        bool first_tok = false;
        if (m.has && m.is_call) {
          FrameHdr* th = frame_at(e, stride, m.target);
          const bool inserted = fresh[q];
          if (inserted) {
            uint32_t* tl = frame_links(th, links_off);
            for (int k = 0; k < n_links; ++k) tl[k] = 0u;     // no scope opened from the new frame yet
            if (inst_off) *frame_links(th, inst_off) = x.inst;   // same instance as the scope that opens it
          }
          if (inserted && may_follow && !has_next && follow + 1 < FOLLOW_DEPTH && P.fn[m.callee].n_params == 1) {
            // the frame this lane goes on with: complete header, nothing pending, not listed
            th->key = m.ckey;
            th->fired = 0;
            th->present_fn = m.bits;
            th->depth = m.depth;
            th->arrived[0] = 0;
            th->arrived[1] = 0;
            has_next = true;
            nx_frame = m.target; nx_bits = m.bits; nx_slot = m.slot; nx_key = m.ckey; nx_val = m.val; nx_depth = m.depth;
          } else if (inserted) {
            // a fresh frame: nobody else can reach it in this step, so its creator writes the header
            th->key = m.ckey;
            th->fired = 0;
            th->present_fn = 0;
            th->depth = m.depth;
            th->arrived[word ^ 1] = 0;
            // an atomic, not a store: further parameters of the same call follow with atomics on
            // this word in this very step, and only atomics on one address keep their order
            (void)a_exch<SCOPE>(&th->arrived[word], m.bits);
            first_tok = true;
          } else {
            first_tok = a_or<SCOPE>(&th->arrived[word], m.bits) == 0;
          }
        } else if (m.has) {
          first_tok = m.res == 0;   // the arrival word was empty: first token for that frame in this step
        }
        const uint32_t pos = wave_alloc(first_tok, kDirect ? next_count : &S->n_touched);
        if (first_tok) {
          if (!kDirect) stg_touched[pos] = m.target;
          else if (pos < e.touched_cap) next_list[pos] = m.target;
          else raise(c, TDF_ERR_TABLE_FULL);
        }
        cnt_tags += (uint32_t)__popcll(__ballot(fresh[q]));
        cnt_tokens += (uint32_t)__popcll(__ballot(m.has));
        if (fresh[q]) mx_depth = em[q].depth > mx_depth ? em[q].depth : mx_depth;
      }
    }
    if (x.active) {
      if (x.fired != fired_in) h->fired = x.fired;
      const uint32_t pf_out = x.present | ((uint32_t)x.myfn << 24);
      if (pf_out != pf_in) h->present_fn = pf_out;
    }
    if (e.reclaim) {
      // Section 5.1: Return_i deallocates the frame.  A tag whose sweep found everything resolved has
      // fired all it ever will (its Return token left above) and can receive nothing more: its frame
      // goes back to the machine, for scopes opened from the next step on.  (Root records stay.)
      const bool give = x.active && x.complete && x.frame < e.cap;
      const uint32_t pos = wave_alloc_scoped<kDirect ? __HIP_MEMORY_SCOPE_WORKGROUP : SCOPE>(give, &c->free_tail);
      if (give) e.free_ring[pos % e.part] = x.frame - e.key_base;
    }
    if (!kDirect || __ballot(has_next) == 0) break;
    // go on with the frame just created
    x.active = has_next;
    x.frame = has_next ? nx_frame : 0;
    h = frame_at(e, stride, x.frame);
    x.slots = frame_slots(h);
    x.fired = 0;
    fired_in = 0;
    pf_in = nx_bits;
    x.present = nx_bits & 0xFFFFFFu;
    x.myfn = has_next ? (int)(nx_bits >> 24) : -1;
    key = nx_key;
    depth = nx_depth;
    x.n_pend = 0;
    x.tc_v = -1;
#pragma unroll
    for (int k = 0; k < MAX_SITES; ++k) x.links[k] = 0u;
#pragma unroll
    for (int k = 0; k < 8; ++k) x.sv[k] = (has_next && (uint32_t)k == nx_slot) ? nx_val : 0;
    if (SW::kLdsValues) {
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (k < n_st) lds_vals[(z.max_values + k) * RB + tid] = x.sv[k];
      for (int k = 8; k < n_st; ++k) lds_vals[(z.max_values + k) * RB + tid] = 0;
    }
    }   // follow
    {   // per-wave maxima of the pass
      const uint32_t wl = wave_umax(x.mx_level), wd = wave_umax(mx_depth);
      if ((tid & 63) == 0) {
        if (wl) atomicMax(kDirect ? &c->max_level : &S->max_level, wl);
        if (wd) atomicMax(kDirect ? &c->max_depth : &S->max_depth, wd);
        if (!kDirect) {
          if (cnt_tags) atomicAdd(&S->n_tags, cnt_tags);
          if (cnt_tokens) atomicAdd(&S->n_tokens, cnt_tokens);
          cnt_tags = cnt_tokens = 0;
        }
      }
    }
    if (kDirect) continue;
    // ---- the workgroup reserves its ranges of the global lists and copies the entries out ---
    __syncthreads();
    if (tid == 0) {
      S->base_touched = S->n_touched ? atomicAdd(next_count, S->n_touched) : 0;
      S->base_leaf = S->n_leaf ? atomicAdd(&c->n_leaf, S->n_leaf) : 0;
      S->base_cell = S->n_cell ? atomicAdd(&c->n_cell, S->n_cell) : 0;
      if (S->n_head) atomicAdd(&c->n_head, S->n_head);
      if (S->n_tags) atomicAdd(&c->n_tags, (unsigned long long)S->n_tags);
      if (S->n_tokens) atomicAdd(&c->n_tokens, (unsigned long long)S->n_tokens);
      if (S->max_depth > c->max_depth) atomicMax(&c->max_depth, S->max_depth);
      if (S->max_level > c->max_level) atomicMax(&c->max_level, S->max_level);
      if (S->base_touched + S->n_touched > e.touched_cap || S->base_leaf + S->n_leaf > e.log_cap ||
          S->base_cell + S->n_cell > e.log_cap)
        raise(c, TDF_ERR_TABLE_FULL);
    }
    __syncthreads();
    for (uint32_t k = tid; k < S->n_touched; k += RB)
      if (S->base_touched + k < e.touched_cap) next_list[S->base_touched + k] = stg_touched[k];
    for (uint32_t k = tid; k < S->n_leaf; k += RB) {
      const uint32_t j = S->base_leaf + k;
      if (j < e.log_cap) {
        e.leaf_row[j] = stg_leaf[k].x;
        e.leaf_tok[j] = stg_leaf[k].y;
      }
    }
    for (uint32_t k = tid; k < S->n_cell; k += RB) {
      const uint32_t j = S->base_cell + k;
      if (j < e.log_cap) {
        const uint4 v = stg_cell[k];
        e.cell_out[j] = v.x;
        e.cell_l[j] = v.y;
        e.cell_r[j] = v.z;
        e.cell_lvl[j] = v.w;
      }
    }
    __syncthreads();
  }
  if (kDirect) {
    if ((tid & 63) == 0) {
      if (cnt_tags) atomicAdd(&c->n_tags, (unsigned long long)cnt_tags);
      if (cnt_tokens) atomicAdd(&c->n_tokens, (unsigned long long)cnt_tokens);
    }
    __syncthreads();
  }
}

// ---- step bookkeeping: reset the consumed list, count the step, detect the end ---------------
__device__ inline void advance(const Engine& e, Ctrl* c, uint32_t step) {
  const int parity = (int)(step & 1);
  const uint32_t next = ld(&c->touched_count[parity ^ 1]);
  uint32_t status = ld(&c->status);
  {
    const uint32_t n = ld(&c->touched_count[parity]);
    st(&c->same_steps, n == ld(&c->prev_count) ? ld(&c->same_steps) + 1u : 0u);
    st(&c->prev_count, n);
    if (n > ld(&c->peak_count)) st(&c->peak_count, n);
  }
  if (e.step_log && step < STEP_LOG_CAP)
    e.step_log[step] = make_uint4(ld(&c->touched_count[parity]), ld(&c->n_alloc), (uint32_t)wall_clock64(), 0u);
  st(&c->touched_count[parity], 0u);
  st(&c->step, step + 1);
  if (e.reclaim) {
    // what this step gave back may be taken from the next step on; a head that ran past the limit
    // (takers found the ring empty) goes back to it
    const uint32_t limit = ld(&c->free_limit);
    if ((int)(ld(&c->free_head) - limit) > 0) st(&c->free_head, limit);
    st(&c->free_limit, ld(&c->free_tail));
  }
  // (with frames given back, max_tags bounds the tags alive at once: the part overflows instead)
  if (!e.reclaim && ld(&c->n_tags) > e.max_tags && status == 0) status = (uint32_t)(-TDF_ERR_TABLE_FULL);
  if (step + 1 >= e.step_limit && next != 0 && status == 0) status = (uint32_t)(-TDF_ERR_STEP_LIMIT);
  if (status != 0) {
    st(&c->status, status);
    st(&c->touched_count[parity ^ 1], 0u);   // drain: nothing more fires
    st(&c->done, 1u);
  } else if (next == 0) {
    st(&c->done, 1u);
  }
}

// A step is "small" when its frames fit two passes of one workgroup; small steps run in the
// single-workgroup kernel, the others in the grid-wide kernel.
__device__ __forceinline__ bool step_is_small(const Engine& e, uint32_t n) { return n <= e.small_limit; }
// Which of the two grid-wide kernels takes a step that is not small: with wide_limit set, the
// die-local one up to that many frames and the device-wide one beyond; else whichever is launched.
template <bool LOCAL> __device__ __forceinline__ bool step_is_other_grids(const Engine& e, uint32_t n) {
  return e.wide_limit != 0 && (LOCAL ? n > e.wide_limit : n <= e.wide_limit);
}

constexpr int STEP_BLOCK = 256;    // lanes per workgroup of the grid-wide kernel
constexpr int LOCAL_BLOCK = 512;   // ... and of its variant that keeps to one accelerator die
constexpr int GEN_SMALL_BLOCK = 512, GEN_LOCAL_BLOCK = 512;   // launch bounds of the generated kernels

// Grid-wide steps: the workgroups of one launch (all resident at once: the host launches no
// more than the GPU holds) run step after step; each takes a slice of the touched list, and a
// grid barrier closes the step.  The last workgroup to arrive does the step bookkeeping and
// releases the others.  A workgroup that waits longer than `spin_ticks` (100 MHz ticks) raises
// an error and ends the run, so every wave leaves the kernel in any case.  Returns when the
// recursion is finished, when the next step is small, or after max_steps steps.
//
// LOCAL: workgroups are handed to the eight accelerator dies (XCDs) in turn, so workgroups
// i, i + 8, i + 16, ... of a launch run on one die and share its L2; they serve machine i % 8
// (machines beyond n_dies have none: their workgroups return at once).  The frame atomics of a
// machine then execute in that L2 (workgroup scope) instead of in memory, and a step boundary
// needs no L2 write-back or invalidation, only an invalidation of the per-CU L1.  The dies a
// machine ran on are recorded in its Ctrl::xcc_mask; the host discards the run if any machine
// saw more than one.  Not LOCAL: device scope, the workgroups dealt evenly to the machines
// (one machine when the whole evaluation runs this way).
// Orders this thread's accesses to the control block, which are all atomic loads, stores and
// read-modify-writes performed in memory.  Die-local runs must not use a device-scope fence
// for this: it would also write back and invalidate the L2 that the step kernel relies on.
template <bool LOCAL> __device__ __forceinline__ void ctrl_fence() {
  if (LOCAL) __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
  else __threadfence();
}

template <bool LOCAL, class SW>
__device__ void steps_grid(Engine e, int max_steps, long long spin_ticks, char* lds, DevProgram* P_lds, uint32_t* sh) {
  constexpr int SCOPE = LOCAL ? __HIP_MEMORY_SCOPE_WORKGROUP : __HIP_MEMORY_SCOPE_AGENT;
  __builtin_amdgcn_s_setprio(3);   // (as in steps_small)
  uint32_t G = gridDim.x, rank = blockIdx.x, die = 0;
  if (LOCAL) {   // workgroup i runs on die i % 8 and serves machine i % 8
    die = blockIdx.x % XCDS;
    if (die >= e.n_dies) return;
    G = gridDim.x / XCDS;
    rank = blockIdx.x / XCDS;
  } else {       // (the host launches a multiple of n_dies workgroups)
    die = blockIdx.x % e.n_dies;
    G = gridDim.x / e.n_dies;
    rank = blockIdx.x / e.n_dies;
  }
  e = die_view(e, die);
  Ctrl* c = e.ctrl;
  uint32_t* const bar_count = LOCAL ? &c->bar_count : &c->wbar_count;
  uint32_t* const bar_gen = LOCAL ? &c->bar_gen : &c->wbar_gen;
  // Nothing changes these before the first barrier completes, and a workgroup reads them before
  // it arrives there: all workgroups see the same values and take the same way.
  uint32_t gen = ld(bar_gen);
  uint32_t step = ld(&c->step);
  uint32_t n = ld(&c->touched_count[step & 1]);
  if (ld(&c->done) || n == 0 || step_is_small(e, n) || step_is_other_grids<LOCAL>(e, n)) return;
  if (LOCAL && threadIdx.x == 0)
    atomicOr(&c->xcc_mask, 1u << xcc_id());
  load_program(P_lds, e.prog);
  for (int it = 0; it < max_steps; ++it) {
    if (rank * blockDim.x < n)
      step_pass<SCOPE, false, SW>(*P_lds, e, c, step, n, rank * blockDim.x, G * blockDim.x, lds);
    // release of this step's writes, before the arrival below.  LOCAL: each wave waits until the
    // die's L2 has acknowledged its stores (vmcnt counts stores here; the barrier alone does not wait)
    if (!LOCAL) __threadfence();
    else __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t arrived = atomicAdd(bar_count, 1u);   // monotone: G per barrier
      if (arrived == (gen + 1u) * G - 1u) {
        ctrl_fence<LOCAL>();
        advance(e, c, step);
        ctrl_fence<LOCAL>();
        st(bar_gen, gen + 1u);
      } else {
        const long long t0 = wall_clock64();
        while (ld(bar_gen) == gen) {
          __builtin_amdgcn_s_sleep(1);
          if (wall_clock64() - t0 > spin_ticks) {   // a workgroup is missing: give up
            raise(c, TDF_ERR_DEVICE);
            st(&c->done, 1u);
            break;
          }
        }
      }
      ctrl_fence<LOCAL>();
      const uint32_t s1 = ld(&c->step);
      sh[0] = s1;
      sh[1] = ld(&c->touched_count[s1 & 1]);
      sh[2] = ld(&c->done);
    }
    __syncthreads();
    // the other workgroups' writes, before the next step reads them
    if (!LOCAL) __threadfence();   // (LOCAL: the next step reads them past the L1, see ld_shared)
    ++gen;
    step = sh[0];
    n = sh[1];
    const bool stop = sh[2] != 0 || n == 0 || step_is_small(e, n) || step_is_other_grids<LOCAL>(e, n);
    __syncthreads();   // sh is written again in the next round
    if (stop) break;
  }
}

// Small steps: one workgroup runs step after step with workgroup barriers only and keeps the
// control block (all list and log counters) in LDS.  Returns when the recursion is finished,
// when a step is too large for one workgroup, or after max_steps steps.
template <class SW>
__device__ void steps_small(Engine e, int max_steps, char* lds, DevProgram* P_lds, Ctrl* lc_) {
  e = die_view(e, blockIdx.x);   // one workgroup per machine
  // A step is a chain of dependent round trips; another evaluation's data plane may share the compute
  // unit (two evaluations in flight): issue before its waves.
  __builtin_amdgcn_s_setprio(3);
  Ctrl& lc = *lc_;
  Ctrl* g = e.ctrl;
  {
    const uint32_t n0 = ld(&g->touched_count[g->step & 1]);
    if (g->done || n0 == 0 || !step_is_small(e, n0)) return;   // nothing to do for this kernel
  }
  load_program(P_lds, e.prog);
  if (threadIdx.x == 0) {
    lc.touched_count[0] = ld(&g->touched_count[0]);
    lc.touched_count[1] = ld(&g->touched_count[1]);
    lc.step = g->step;
    lc.prev_count = ld(&g->prev_count);
    lc.peak_count = ld(&g->peak_count);
    lc.same_steps = ld(&g->same_steps);
    lc.n_leaf = ld(&g->n_leaf);
    lc.n_cell = ld(&g->n_cell);
    lc.n_head = ld(&g->n_head);
    lc.status = ld(&g->status);
    lc.done = g->done;
    lc.n_alloc = ld(&g->n_alloc);
    lc.free_head = ld(&g->free_head);
    lc.free_tail = ld(&g->free_tail);
    lc.free_limit = ld(&g->free_limit);
    lc.max_depth = ld(&g->max_depth);
    lc.max_level = ld(&g->max_level);
    lc.bar_count = lc.bar_gen = 0;
    lc.n_tags = ld(&g->n_tags);
    lc.n_tokens = ld(&g->n_tokens);
  }
  __syncthreads();
  for (int it = 0; it < max_steps; ++it) {
    const uint32_t step = lc.step;
    const uint32_t n = lc.touched_count[step & 1];
    if (lc.done || n == 0 || !step_is_small(e, n)) break;   // uniform: lc changes only between barriers
    step_pass<__HIP_MEMORY_SCOPE_WORKGROUP, true, SW>(*P_lds, e, &lc, step, n, 0, blockDim.x, lds);
    if (threadIdx.x == 0) advance(e, &lc, step);
    __syncthreads();
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    st(&g->touched_count[0], lc.touched_count[0]);
    st(&g->touched_count[1], lc.touched_count[1]);
    g->step = lc.step;
    st(&g->prev_count, lc.prev_count);
    st(&g->peak_count, lc.peak_count);
    st(&g->same_steps, lc.same_steps);
    st(&g->n_leaf, lc.n_leaf);
    st(&g->n_cell, lc.n_cell);
    st(&g->n_head, lc.n_head);
    st(&g->status, lc.status);
    g->done = lc.done;
    st(&g->n_alloc, lc.n_alloc);
    st(&g->free_head, lc.free_head);
    st(&g->free_tail, lc.free_tail);
    st(&g->free_limit, lc.free_limit);
    st(&g->max_depth, lc.max_depth);
    st(&g->max_level, lc.max_level);
    st(&g->n_tags, lc.n_tags);
    st(&g->n_tokens, lc.n_tokens);
  }
}

}  // namespace tdf
