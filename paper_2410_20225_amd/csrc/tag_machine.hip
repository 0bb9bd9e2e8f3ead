// The tag machine: tokens are matched by call-context tag, the frames that received a token
// are compacted into a list, and the node bodies of every listed frame fire at once.
//
// One step = one pass over the touched list, one lane per frame (= per tag):
//   fire    the lane walks the firing table of the frame's function; an entry fires when its
//           sources are present under that tag (Section 2.2: all inputs hold tokens with the
//           same tag).  Dead values (hiatons) propagate; Switch, Merge and dead calls follow
//           the paper's equations.
//   match   every token the sweep emits is delivered on the spot:
//           Call_i  <t,d> -> <i:t,d>: find-or-insert the key (frame of t, i) in the tag-hash
//                   table (Section 3; Section 5.1: a new frame that stores the label i), write
//                   the argument into that frame;
//           Return_i <i:t,d> -> <t,d>: the frame's own key names its label i and the frame of
//                   t, which is the label check of Section 5.1 (only the Return_i of the call
//                   that created the frame produces output); the value goes to the caller's
//                   frame.
//   compact the first token that reaches a frame in a step appends it to the next step's list
//           (wave ballot + prefix sum, one counter bump per wave).
//
// A frame that is being swept may receive a token in the same step from another lane.  Such
// a token sets a bit in the frame's arrival word of the *next* step and puts the frame on the
// next list; the running sweep neither sees the bit nor reads the value.  Only the key, the
// step stamp and the arrival words are written concurrently, with device-scope atomics.
#include "engine.h"

namespace tdf {

namespace {

constexpr int FIRE_BLOCK = 128;   // grid-wide kernel

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
template <int SCOPE> __device__ __forceinline__ unsigned long long a_cas(unsigned long long* p, unsigned long long expect,
                                                                        unsigned long long v) {
  __hip_atomic_compare_exchange_strong(p, &expect, v, __ATOMIC_RELAXED, __ATOMIC_RELAXED, SCOPE);
  return expect;
}
template <int SCOPE> __device__ __forceinline__ unsigned long long a_ld(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, SCOPE);
}

// fmix64 of MurmurHash3 (Appleby, public domain).
__device__ __forceinline__ unsigned long long mix64(unsigned long long x) {
  x ^= x >> 33;
  x *= 0xff51afd7ed558ccdULL;
  x ^= x >> 33;
  x *= 0xc4ceb9fe1a85ec53ULL;
  x ^= x >> 33;
  return x;
}

// ---- seed: one root frame per instance, holding the arguments of `result` ---------------
__global__ void k_seed(DevProgram P, Engine e) {
  uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= e.n_inst) return;
  uint32_t f = e.cap + b;
  FrameHdr* h = frame_at(e, P.frame_stride, f);
  long long* s = frame_slots(h);
  int np = P.fn[P.result_fn].n_params;
  for (int k = 0; k < np; ++k) s[k] = e.args[(size_t)b * e.n_args + k];
  h->key = 0;
  h->fired = 0;
  h->present_fn = ((1u << np) - 1u) | ((uint32_t)P.result_fn << 24);
  h->arrived[0] = h->arrived[1] = 0;
  e.touched[b] = f;
  if (b == 0) e.ctrl->touched_count[0] = e.n_inst;
}

struct Src {
  long long v;
  bool p, d;   // present, dead
};

// The firing tables are copied into LDS by every workgroup; a table entry read from there is
// the same in all lanes and is moved to scalar registers, so that the dispatch on it and the
// indexing of the register value file stay wave-uniform.
__device__ __forceinline__ uint32_t uni(uint32_t x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ Instr fetch(const DevProgram& P, int idx) {
  union { Instr i; uint32_t w[4]; } u;
  u.i = P.instr[idx];
#pragma unroll
  for (int k = 0; k < 4; ++k) u.w[k] = uni(u.w[k]);
  return u.i;
}
__device__ __forceinline__ void load_program(DevProgram* dst, const DevProgram* src) {
  const uint32_t* s = reinterpret_cast<const uint32_t*>(src);
  uint32_t* d = reinterpret_cast<uint32_t*>(dst);
  for (int i = threadIdx.x; i < (int)(sizeof(DevProgram) / 4); i += blockDim.x) d[i] = s[i];
  __syncthreads();
}

// Per-workgroup staging of one pass.  Lanes take positions in these LDS lists with wave ballots;
// the workgroup reserves its ranges of the global lists with one atomic per list when the pass
// ends and copies the entries out.
struct Stage {
  uint32_t n_touched, n_leaf, n_cell, n_head, n_tags, n_tokens;
  uint32_t max_probe, max_depth, max_level;
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
// dynamic LDS of a step kernel with `rb` lanes
__host__ __device__ inline size_t step_lds_bytes(const Sizes& z, int rb) {
  return (size_t)rb * ((size_t)(z.max_values + z.max_stored) * 8 + (size_t)z.max_emit * 4 + 8 + 16) + sizeof(Stage);
}

// Deliver one value to slot `slot` of frame `target`, and stage the frame for the next list if
// this is the first token to reach it in this step.  `exclusive`: the frame was created by this
// lane and no other token can reach it before its first sweep (single-parameter callee), so
// plain stores do.  Must be reached by the whole wave.
template <int SCOPE>
__device__ __forceinline__ void deliver(const Engine& e, int stride, bool go, uint32_t target, uint32_t slot,
                                        long long value, uint32_t or_bits, uint32_t word, bool exclusive,
                                        Stage* S, uint32_t* stg_touched) {
  bool first = false;
  if (go) {
    FrameHdr* h = frame_at(e, stride, target);
    frame_slots(h)[slot] = value;                     // read in a later step only
    if (exclusive) {
      h->arrived[word] = or_bits;
      first = true;
    } else {
      first = a_or<SCOPE>(&h->arrived[word], or_bits) == 0;
    }
  }
  const uint32_t pos = wave_alloc(first, &S->n_touched);
  if (first) stg_touched[pos] = target;
}

// One pass over the touched frames [0, n) of the current list; lane `first + tid` takes frames
// i, i + lane_stride, ...  `c` is the control block the pass counts in: the global one, or a
// workgroup's LDS copy.  The loop over passes is uniform for the workgroup.
// NV > 0: the value file of a sweep (at most NV values, 8 stored values) lives in registers,
// indexed with the wave-uniform value ids of the firing table; NV == 0: it lives in LDS.
template <int SCOPE, int NV>
__device__ void step_pass(const DevProgram& P, const Engine& e, Ctrl* c, uint32_t step, uint32_t n,
                          uint32_t first, uint32_t lane_stride, char* lds) {
  const int tid = threadIdx.x;
  const int RB = blockDim.x;
  Sizes z = sizes_of(P);
  if (NV > 0) z.max_values = z.max_stored = 0;   // no LDS value file
  long long rloc[NV > 0 ? NV : 1], sloc[NV > 0 ? 8 : 1];
  auto rd = [&](int idx) -> long long {
    if constexpr (NV > 0) return rloc[idx]; else return reinterpret_cast<long long*>(lds)[idx * RB + tid];
  };
  auto wr = [&](int idx, long long v) {
    if constexpr (NV > 0) rloc[idx] = v; else reinterpret_cast<long long*>(lds)[idx * RB + tid] = v;
  };
  auto rd_st = [&](int idx) -> long long {
    if constexpr (NV > 0) return sloc[idx];
    else return reinterpret_cast<long long*>(lds)[(z.max_values + idx) * RB + tid];
  };
  long long* regs = reinterpret_cast<long long*>(lds);                 // [value][lane]
  long long* stv = regs + (size_t)z.max_values * RB;                   // [stored slot][lane]
  uint4* stg_cell = reinterpret_cast<uint4*>(stv + (size_t)z.max_stored * RB);
  uint2* stg_leaf = reinterpret_cast<uint2*>(stg_cell + RB);
  uint32_t* stg_touched = reinterpret_cast<uint32_t*>(stg_leaf + RB);  // [max_emit * RB]
  Stage* S = reinterpret_cast<Stage*>(stg_touched + (size_t)z.max_emit * RB);
  const int stride = (int)uni((uint32_t)P.frame_stride);
  const uint32_t* cur_list = e.touched + (size_t)(step & 1) * e.touched_cap;
  uint32_t* next_list = e.touched + (size_t)((step & 1) ^ 1) * e.touched_cap;
  uint32_t* next_count = &c->touched_count[(step & 1) ^ 1];
  const uint32_t word = step & 1;    // arrival word of the next step (this step reads word ^ 1)
  const int n_st = sizes_of(P).max_stored;

  for (uint32_t base = first; base < n; base += lane_stride) {
    if (tid == 0) *S = Stage{};
    __syncthreads();
    const uint32_t i = base + tid;
    const bool active = i < n;
    const uint32_t frame = active ? cur_list[i] : 0;
    FrameHdr* h = frame_at(e, stride, frame);
    long long* slots = frame_slots(h);
    unsigned long long fired = 0, key = 0;
    uint32_t present = 0, depth = 0, pf_in = 0;
    int myfn = -1;
    if (active) {
      // tokens that arrived for this step; the word of the other parity belongs to the next
      const uint32_t arr = a_exch<SCOPE>(&h->arrived[word ^ 1], 0u);
      pf_in = h->present_fn;
      key = h->key;
      fired = h->fired;
      const uint32_t pf = pf_in | arr;
      depth = (uint32_t)(key >> 8) & 0xFFFFFFu;
      present = pf & 0xFFFFFFu;
      myfn = (int)(pf >> 24);
    }
    const unsigned long long fired_in = fired;
    // stored values (meaningful where the present bit is set), all loads in flight at once
    if constexpr (NV > 0) {
#pragma unroll
      for (int k = 0; k < 8; ++k) sloc[k] = (active && k < n_st) ? slots[k] : 0;
    } else {
      for (int k0 = 0; k0 < n_st; k0 += 8) {
        long long sv[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) sv[k] = (active && k0 + k < n_st) ? slots[k0 + k] : 0;
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (k0 + k < n_st) stv[(k0 + k) * RB + tid] = sv[k];
      }
    }
    // Warm the lines this sweep may write to: the frames of the calls it can make (their keys
    // depend only on this frame and the label) on a first sweep, the caller's frame otherwise.
    // The loaded words are only folded into `warm`, which is never acted on.
    unsigned long long warm = 0;
    if (active && myfn >= 0) {
      if (fired == 0) {
        const int ncl = P.fn[myfn].n_call_labels;
        for (int k = 0; k < ncl; ++k) {
          const unsigned long long ckey = ((unsigned long long)(frame + 1u) << 32) |
                                          ((unsigned long long)(depth + 1u) << 8) | (P.fn[myfn].call_labels[k] + 1u);
          warm += frame_at(e, stride, (uint32_t)mix64(ckey) & e.cap_mask)->fired;
        }
      }
      if (key != 0) warm += frame_at(e, stride, (uint32_t)(key >> 32) - 1u)->fired;
    }
    // forest entries of the last node looked at: one round trip serves isleaf/left/right/token
    long long tc_v = -1;
    int tc_left = 0, tc_right = 0, tc_token = 0;

    const int n_fn = (int)uni((uint32_t)P.n_fn);
    for (int f = 0; f < n_fn; ++f) {
      const bool on = myfn == f;
      if (__ballot(on) == 0) continue;
      const int first_i = (int)uni(P.fn[f].first), count = (int)uni(P.fn[f].count);
      const bool is_result = f == (int)uni((uint32_t)P.result_fn);
      unsigned long long pres = 0, dead = 0;   // over value ids

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
            const bool p = on && ((present >> I.aux) & 1);
            put(I.dst, rd_st(I.aux), p, false);
            live = p;
            break;
          }
          case D_RET: {
            const bool p = on && ((present >> I.aux) & 1);
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
            if (p && !d) {
              if (a.v < 0 || a.v >= e.n_tree_nodes || e.left == nullptr) {
                raise(c, TDF_ERR_BAD_ARG);
                d = true;
              } else {
                if (tc_v != a.v) {
                  tc_left = e.left[a.v];
                  tc_right = e.right[a.v];
                  tc_token = e.token[a.v];
                  tc_v = a.v;
                }
                if (I.op == D_ISLEAF) r = tc_left < 0;
                else if (I.op == D_LEFT) r = tc_left;
                else if (I.op == D_RIGHT) r = tc_right;
                else r = tc_token;
              }
            }
            put(I.dst, r, p, p && d);
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
            // Call_i: <t,d> -> <i:t,d>.  The tag i:t is the key (this frame, tag length, i).
            const Src a = src(0);
            const bool go = on && a.p && !a.d && !(fired & ibit);
            const uint32_t label = I.aux, param = I.aux2;
            uint32_t child = 0, probes = 0;
            bool found = false, inserted = false;
            if (go) {
              const unsigned long long ckey =
                  ((unsigned long long)(frame + 1u) << 32) | ((unsigned long long)(depth + 1u) << 8) | (label + 1u);
              uint32_t s = (uint32_t)mix64(ckey) & e.cap_mask;
              const uint32_t probe_limit = e.cap < 8192u ? e.cap : 8192u;
              for (probes = 1; probes <= probe_limit; ++probes) {
                FrameHdr* ch = frame_at(e, stride, s);
                const unsigned long long cur = a_cas<SCOPE>(&ch->key, 0ull, ckey);
                if (cur == 0) {
                  inserted = found = true;
                  break;
                }
                if (cur == ckey) {
                  found = true;
                  break;
                }
                s = (s + 1) & e.cap_mask;
              }
              child = s;
              if (!found) raise(c, TDF_ERR_TABLE_FULL);
            }
            const uint32_t callee = P.label_callee[label];
            deliver<SCOPE>(e, stride, go && found, child, param, a.v, (1u << param) | (callee << 24), word,
                           inserted && P.fn[callee].n_params == 1, S, stg_touched);
            (void)wave_alloc(inserted, &S->n_tags);
            (void)wave_alloc(go && found, &S->n_tokens);
            if (__ballot(inserted)) {
              wave_max(inserted ? probes : 0, &S->max_probe);
              wave_max(inserted ? depth + 1 : 0, &S->max_depth);
            }
            live = on && a.p && !a.d;
            break;
          }
          case D_OUT: {
            const Src a = src(0);
            const bool go = on && a.p && !a.d && !(fired & ibit);
            if (is_result) {
              if (go) {
                const uint32_t b = frame - e.cap;
                if (I.aux == T_INT) { if (e.out_i64) e.out_i64[b] = a.v; }
                else if (I.aux == T_VEC) e.root_ref[b] = (uint32_t)a.v;
              }
            } else {
              // Return_i: <i:t,d> -> <t,d>; i and the frame of t are in this frame's key
              const uint32_t parent = (uint32_t)(key >> 32) - 1u, label = ((uint32_t)key & 0xFFu) - 1u;
              const uint32_t slot = go ? P.label_ret_slot[label] : 0;
              deliver<SCOPE>(e, stride, go, parent, slot, a.v, 1u << slot, word, false, S, stg_touched);
              (void)wave_alloc(go, &S->n_tokens);
            }
            live = on && a.p && !a.d;
            break;
          }
          case D_EMBED: {
            // the leaf's state row is the row of this frame; level 0
            const Src a = src(0);
            const bool had = on && ((present >> I.aux) & 1);
            const bool go = on && a.p && !a.d && !had;
            const bool ok = go && a.v >= 0;
            if (go && !ok) raise(c, TDF_ERR_BAD_ARG);
            const uint32_t pos = wave_alloc(ok, &S->n_leaf);
            if (ok) {
              stg_leaf[pos] = make_uint2(frame, (uint32_t)a.v);
              slots[I.aux] = (long long)frame;
              present |= 1u << I.aux;
            }
            put(I.dst, had ? rd_st(I.aux) : (long long)frame, had || ok, false);
            live = had || ok;
            break;
          }
          case D_CELL: {
            const Src a = src(0), b = src(1);
            const bool had = on && ((present >> I.aux) & 1);
            const bool go = on && a.p && b.p && !a.d && !b.d && !had;
            const uint32_t pos = wave_alloc(go, &S->n_cell);
            long long r = rd_st(I.aux);
            uint32_t lvl = 0;
            if (go) {
              const uint32_t la = (uint32_t)(a.v >> 32), lb = (uint32_t)(b.v >> 32);
              lvl = 1 + (la > lb ? la : lb);
              stg_cell[pos] = make_uint4(frame, (uint32_t)a.v, (uint32_t)b.v, lvl);
              r = (long long)frame | ((long long)lvl << 32);
              slots[I.aux] = r;
              present |= 1u << I.aux;
            }
            if (__ballot(go)) wave_max(lvl, &S->max_level);
            put(I.dst, r, had || go, false);
            live = had || go;
            break;
          }
          case D_HEAD: {
            const Src a = src(0), b = src(1);
            const bool had = on && ((present >> I.aux) & 1);
            const bool go = on && a.p && b.p && !a.d && !b.d && !had && is_result;
            if (go) {
              const uint32_t inst = frame - e.cap;
              e.head_row[inst] = (uint32_t)a.v;
              e.head_label[inst] = (uint32_t)b.v;
              slots[I.aux] = inst;
              present |= 1u << I.aux;
            }
            (void)wave_alloc(go, &S->n_head);
            put(I.dst, (long long)(frame - e.cap), had || go, false);
            live = had || go;
            break;
          }
          default: break;
        }
        if (live) fired |= ibit;   // counted after the run, from the fired masks
      }
    }
    if (warm == 0xFEEDFACECAFEBEEFull) raise(c, TDF_ERR_DEVICE);   // keeps the warming loads alive
    if (active) {
      if (fired != fired_in) h->fired = fired;
      const uint32_t pf_out = present | ((uint32_t)myfn << 24);
      if (pf_out != pf_in) h->present_fn = pf_out;
    }

    // ---- the workgroup reserves its ranges of the global lists and copies the entries out ---
    __syncthreads();
    if (tid == 0) {
      S->base_touched = S->n_touched ? atomicAdd(next_count, S->n_touched) : 0;
      S->base_leaf = S->n_leaf ? atomicAdd(&c->n_leaf, S->n_leaf) : 0;
      S->base_cell = S->n_cell ? atomicAdd(&c->n_cell, S->n_cell) : 0;
      if (S->n_head) atomicAdd(&c->n_head, S->n_head);
      if (S->n_tags) atomicAdd(&c->n_tags, (unsigned long long)S->n_tags);
      if (S->n_tokens) atomicAdd(&c->n_tokens, (unsigned long long)S->n_tokens);
      if (S->max_probe > c->max_probe) atomicMax(&c->max_probe, S->max_probe);
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
        const uint4 x = stg_cell[k];
        e.cell_out[j] = x.x;
        e.cell_l[j] = x.y;
        e.cell_r[j] = x.z;
        e.cell_lvl[j] = x.w;
      }
    }
    __syncthreads();
  }
}

// ---- step bookkeeping: reset the consumed list, count the step, detect the end ---------------
__device__ void advance(const Engine& e, Ctrl* c, uint32_t step) {
  const int parity = (int)(step & 1);
  const uint32_t next = ld(&c->touched_count[parity ^ 1]);
  uint32_t status = ld(&c->status);
  st(&c->touched_count[parity], 0u);
  c->step = step + 1;
  if (ld(&c->n_tags) > e.max_tags && status == 0) status = (uint32_t)(-TDF_ERR_TABLE_FULL);
  if (step + 1 >= e.step_limit && next != 0 && status == 0) status = (uint32_t)(-TDF_ERR_STEP_LIMIT);
  if (status != 0) {
    st(&c->status, status);
    st(&c->touched_count[parity ^ 1], 0u);   // drain: nothing more fires
    c->done = 1;
  } else if (next == 0) {
    c->done = 1;
  }
}

// A step is "small" when its frames fit two passes of one workgroup; small steps run in
// k_steps_small, the others in the grid-wide k_step.
__device__ __forceinline__ bool step_is_small(const Engine& e, uint32_t n) { return n <= e.small_limit; }

template <int NV>
__global__ void __launch_bounds__(FIRE_BLOCK) k_step(Engine e) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ DevProgram P;
  Ctrl* c = e.ctrl;
  const uint32_t step = c->step;
  const uint32_t n = ld(&c->touched_count[step & 1]);
  if (c->done || n == 0 || step_is_small(e, n)) return;
  if (blockIdx.x * blockDim.x < n) {   // workgroups without frames only take part in closing the step
    load_program(&P, e.prog);
    step_pass<__HIP_MEMORY_SCOPE_AGENT, NV>(P, e, c, step, n, blockIdx.x * blockDim.x, gridDim.x * blockDim.x, lds);
  }
  // the last workgroup to finish closes the step
  __shared__ bool last;
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    last = atomicAdd(&c->blocks_done, 1u) == gridDim.x - 1;
  }
  __syncthreads();
  if (last && threadIdx.x == 0) {
    __threadfence();
    st(&c->blocks_done, 0u);
    advance(e, c, step);
  }
}

// Small steps: one workgroup runs step after step with workgroup barriers only and keeps the
// control block (all list and log counters) in LDS.  Returns when the recursion is finished,
// when a step is too large for one workgroup, or after max_steps steps.
template <int NV>
__global__ void __launch_bounds__(512) k_steps_small(Engine e, int max_steps) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ DevProgram P;
  __shared__ Ctrl lc;
  Ctrl* g = e.ctrl;
  {
    const uint32_t n0 = ld(&g->touched_count[g->step & 1]);
    if (g->done || n0 == 0 || !step_is_small(e, n0)) return;   // nothing to do for this kernel
  }
  load_program(&P, e.prog);
  if (threadIdx.x == 0) {
    lc.touched_count[0] = ld(&g->touched_count[0]);
    lc.touched_count[1] = ld(&g->touched_count[1]);
    lc.step = g->step;
    lc.n_leaf = ld(&g->n_leaf);
    lc.n_cell = ld(&g->n_cell);
    lc.n_head = ld(&g->n_head);
    lc.status = ld(&g->status);
    lc.done = g->done;
    lc.max_probe = ld(&g->max_probe);
    lc.max_depth = ld(&g->max_depth);
    lc.max_level = ld(&g->max_level);
    lc.blocks_done = 0;
    lc.n_tags = ld(&g->n_tags);
    lc.n_tokens = ld(&g->n_tokens);
  }
  __syncthreads();
  for (int it = 0; it < max_steps; ++it) {
    const uint32_t step = lc.step;
    const uint32_t n = lc.touched_count[step & 1];
    if (lc.done || n == 0 || !step_is_small(e, n)) break;   // uniform: lc changes only between barriers
    step_pass<__HIP_MEMORY_SCOPE_WORKGROUP, NV>(P, e, &lc, step, n, 0, blockDim.x, lds);
    if (threadIdx.x == 0) advance(e, &lc, step);
    __syncthreads();
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    st(&g->touched_count[0], lc.touched_count[0]);
    st(&g->touched_count[1], lc.touched_count[1]);
    g->step = lc.step;
    st(&g->n_leaf, lc.n_leaf);
    st(&g->n_cell, lc.n_cell);
    st(&g->n_head, lc.n_head);
    st(&g->status, lc.status);
    g->done = lc.done;
    st(&g->max_probe, lc.max_probe);
    st(&g->max_depth, lc.max_depth);
    st(&g->max_level, lc.max_level);
    st(&g->n_tags, lc.n_tags);
    st(&g->n_tokens, lc.n_tokens);
  }
}

// ---- statistics: live firings per static-graph node, counted from the fired masks -------------
__global__ void k_count_fired(DevProgram P, Engine e) {
  __shared__ uint32_t cnt[MAX_INSTR];
  for (int i = threadIdx.x; i < MAX_INSTR; i += blockDim.x) cnt[i] = 0;
  __syncthreads();
  const uint32_t total = e.cap + e.n_inst;
  for (uint32_t f = blockIdx.x * blockDim.x + threadIdx.x; f < total; f += gridDim.x * blockDim.x) {
    const FrameHdr* h = frame_at(e, P.frame_stride, f);
    unsigned long long fired = h->fired;
    if (fired == 0) continue;
    const int fn = (int)(h->present_fn >> 24);
    const int first = P.fn[fn].first;
    while (fired) {
      const int ip = __ffsll((long long)fired) - 1;
      fired &= fired - 1;
      atomicAdd(&cnt[first + ip], 1u);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < MAX_INSTR; i += blockDim.x) {
    const uint16_t st_idx = P.stat_idx[i];
    if (cnt[i] && st_idx != 0xFFFF) atomicAdd(&e.fire_count[st_idx], (unsigned long long)cnt[i]);
  }
}

// ---- cells by dependency level --------------------------------------------------------------
// A cell's level is 1 + the larger level of its two operands (leaves are level 0); cells of
// one level are independent of each other.  Counting sort of the firing log by level.
__global__ void k_level_hist(Engine e) {
  const uint32_t n = e.ctrl->n_cell;
  for (uint32_t base = blockIdx.x * blockDim.x; base < n; base += gridDim.x * blockDim.x) {
    const uint32_t j = base + threadIdx.x;
    (void)wave_alloc_keyed(j < n, j < n ? e.cell_lvl[j] : 0, e.level_count);
  }
}

__global__ void k_level_scan(Engine e) {
  // single block; levels 1..max_level
  __shared__ uint32_t carry;
  __shared__ uint32_t buf[1024];
  const uint32_t L = e.ctrl->max_level + 2;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (uint32_t base = 0; base < L; base += 1024) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t v = i < L ? e.level_count[i] : 0;
    buf[threadIdx.x] = v;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      uint32_t t = threadIdx.x >= (unsigned)off ? buf[threadIdx.x - off] : 0;
      __syncthreads();
      buf[threadIdx.x] += t;
      __syncthreads();
    }
    if (i < L) e.level_off[i] = carry + buf[threadIdx.x] - v;
    __syncthreads();
    if (threadIdx.x == 1023) carry += buf[1023];
    __syncthreads();
  }
}

__global__ void k_level_scatter(Engine e) {
  const uint32_t n = e.ctrl->n_cell;
  for (uint32_t base = blockIdx.x * blockDim.x; base < n; base += gridDim.x * blockDim.x) {
    const uint32_t j = base + threadIdx.x;
    const bool on = j < n;
    const uint32_t lvl = on ? e.cell_lvl[j] : 0;
    const uint32_t rank = wave_alloc_keyed(on, lvl, e.level_fill);
    if (on) {
      const uint32_t q = e.level_off[lvl] + rank;
      e.q_out[q] = e.cell_out[j];
      e.q_l[q] = e.cell_l[j];
      e.q_r[q] = e.cell_r[j];
    }
  }
}

}  // namespace

// ---- host launchers ----------------------------------------------------------------------
static int grid_for(uint32_t n, int block, int max_blocks) {
  long long g = ((long long)n + block - 1) / block;
  if (g < 1) g = 1;
  return (int)(g > max_blocks ? max_blocks : g);
}

void launch_seed(const DevProgram& P, const Engine& e, hipStream_t s) {
  hipLaunchKernelGGL(k_seed, dim3(grid_for(e.n_inst, 256, 1 << 20)), dim3(256), 0, s, P, e);
}

// Register value file when every function has at most 16 values and 8 stored values.
static bool fits_registers(const Sizes& z) { return z.max_values <= 16 && z.max_stored <= 8; }
static Sizes lds_sizes(const DevProgram& P) {
  Sizes z = sizes_of(P);
  if (fits_registers(z)) z.max_values = z.max_stored = 0;
  return z;
}

// Lanes of the single-workgroup kernel: as many as the per-lane LDS footprint allows.
int tag_machine_small_block(const DevProgram& P) {
  const Sizes z = lds_sizes(P);
  int rb = 512;
  while (rb > 64 && step_lds_bytes(z, rb) > 120 * 1024) rb >>= 1;
  return rb;
}

// One round of the tag machine: as many small steps as fit (one workgroup), then one
// grid-wide step if the next step is large.  Each kernel decides on the device whether the
// current step is its own.
void launch_round(const DevProgram& P, const Engine& e, int blocks, int small_block, int small_steps,
                  hipStream_t s) {
  const Sizes z = lds_sizes(P);
  const bool in_regs = fits_registers(sizes_of(P));
  const size_t small_lds = step_lds_bytes(z, small_block);
  if (small_lds > 48 * 1024)   // large value files need the LDS opt-in
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_steps_small<0>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_lds);
  if (in_regs) {
    hipLaunchKernelGGL(k_steps_small<16>, dim3(1), dim3(small_block), small_lds, s, e, small_steps);
    hipLaunchKernelGGL(k_step<16>, dim3(blocks), dim3(FIRE_BLOCK), step_lds_bytes(z, FIRE_BLOCK), s, e);
  } else {
    hipLaunchKernelGGL(k_steps_small<0>, dim3(1), dim3(small_block), small_lds, s, e, small_steps);
    hipLaunchKernelGGL(k_step<0>, dim3(blocks), dim3(FIRE_BLOCK), step_lds_bytes(z, FIRE_BLOCK), s, e);
  }
}

void launch_count_fired(const DevProgram& P, const Engine& e, hipStream_t s) {
  hipLaunchKernelGGL(k_count_fired, dim3(grid_for(e.cap + e.n_inst, 256, 1024)), dim3(256), 0, s, P, e);
}

void launch_levels(const Engine& e, uint32_t n_cell, hipStream_t s) {
  int g = grid_for(n_cell, 256, 2048);
  hipLaunchKernelGGL(k_level_hist, dim3(g), dim3(256), 0, s, e);
  hipLaunchKernelGGL(k_level_scan, dim3(1), dim3(1024), 0, s, e);
  hipLaunchKernelGGL(k_level_scatter, dim3(g), dim3(256), 0, s, e);
}

}  // namespace tdf
