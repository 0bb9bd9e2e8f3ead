// The tag machine: match tokens by call-context tag, compact the frames that received a
// token, and fire the node bodies of every such frame at once.
//
//   fire   one lane per touched frame walks the firing table of the frame's function; an
//          entry fires when its sources are present under that tag (Section 2.2).  Call_i
//          entries emit <i:t,d> tokens, the function output emits the Return token, vector
//          operators append to the schedule log and yield a row reference.
//   match  one lane per token.  Call tokens find-or-insert the key (parent frame, label) in
//          the tag-hash table (Section 3: Call_i <t,d> = <i:t,d>; Section 5.1: a new frame
//          that stores the label); Return tokens read the frame's key back, which is the
//          label check of Return_i, and deliver the value to the caller's frame (Return_i
//          <i:t,d> = <t,d>).  Frames that received a token are compacted into the touched
//          list with wave ballots and one counter bump per wave.
#include "engine.h"

namespace tdf {

namespace {

constexpr int FIRE_BLOCK = 128;
constexpr int MATCH_BLOCK = 256;

__device__ __forceinline__ void raise(Ctrl* c, int status) {
  atomicCAS(&c->status, 0u, (uint32_t)(-status));
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
  h->touched = 0;
  h->depth = 0;
  e.touched[b] = f;
  if (b == 0) e.ctrl->touched_count[0] = e.n_inst;
}

// ---- fire --------------------------------------------------------------------------------
struct Src {
  long long v;
  bool p, d;   // present, dead
};

// One pass over the touched frames [0, n): lane `first + tid` takes frame i, i + stride, ...
// regs is the block's value file in LDS, [value][lane of the block].
__device__ void fire_pass(const DevProgram& P, const Engine& e, uint32_t n, uint32_t first, uint32_t stride,
                          long long* regs) {
  Ctrl* c = e.ctrl;
  const int tid = threadIdx.x;
  const int FIRE_BLOCK = blockDim.x;
  for (uint32_t base = first; base < n; base += stride) {
    const uint32_t i = base + tid;
    const bool active = i < n;
    const uint32_t frame = active ? e.touched[i] : 0;
    FrameHdr* h = frame_at(e, P.frame_stride, frame);
    long long* slots = frame_slots(h);
    unsigned long long fired = 0;
    uint32_t present = 0;
    int myfn = -1;
    if (active) {
      fired = h->fired;
      // present_fn is updated with atomics by the match pass: read it the same way
      const uint32_t pf = __atomic_load_n(&h->present_fn, __ATOMIC_RELAXED);
      present = pf & 0xFFFFFFu;
      myfn = (int)(pf >> 24);
    }
    const unsigned long long fired_in = fired;
    const uint32_t present_in = present;

    for (int f = 0; f < P.n_fn; ++f) {
      const bool on = myfn == f;
      if (__ballot(on) == 0) continue;
      const int first = P.fn[f].first, count = P.fn[f].count;
      const bool is_result = f == P.result_fn;
      unsigned long long pres = 0, dead = 0;   // over value ids

      for (int ip = 0; ip < count; ++ip) {
        const Instr I = P.instr[first + ip];
        const unsigned long long ibit = 1ull << ip;
        auto src = [&](int k) -> Src {
          const uint8_t s = I.src[k];
          if (s == SRC_IMM) return Src{I.imm, true, false};
          return Src{regs[(int)s * FIRE_BLOCK + tid], ((pres >> s) & 1) != 0, ((dead >> s) & 1) != 0};
        };
        auto put = [&](int dst, long long v, bool p, bool d) {
          regs[dst * FIRE_BLOCK + tid] = v;
          if (p) pres |= 1ull << dst;
          if (d) dead |= 1ull << dst;
        };
        bool live = false;   // this entry holds a live value under this tag
        switch (I.op) {
          case D_IN: {
            const bool p = on && ((present >> I.aux) & 1);
            put(I.dst, p ? slots[I.aux] : 0, p, false);
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
            put(I.dst, p ? slots[I.aux] : 0, p || is_dead, is_dead);
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
              } else if (I.op == D_ISLEAF) r = e.left[a.v] < 0;
              else if (I.op == D_LEFT) r = e.left[a.v];
              else if (I.op == D_RIGHT) r = e.right[a.v];
              else r = e.token[a.v];
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
            const Src a = src(0);
            const bool go = on && a.p && !a.d && !(fired & ibit);
            const uint32_t pos = wave_alloc(go, &c->q_count);
            if (go) {
              if (pos < e.q_cap)
                e.queue[pos] = Token{frame, 0x80000000u | I.aux | ((uint32_t)I.aux2 << 8), a.v};
              else
                raise(c, TDF_ERR_TABLE_FULL);
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
              const uint32_t pos = wave_alloc(go, &c->q_count);
              if (go) {
                if (pos < e.q_cap) e.queue[pos] = Token{frame, 0u, a.v};
                else raise(c, TDF_ERR_TABLE_FULL);
              }
            }
            live = on && a.p && !a.d;
            break;
          }
          case D_EMBED: {
            const Src a = src(0);
            const bool had = on && ((present >> I.aux) & 1);
            const bool go = on && a.p && !a.d && !had;
            const uint32_t idx = wave_alloc(go, &c->n_leaf);
            const uint32_t row = wave_alloc(go, &c->n_rows);
            long long r = had ? slots[I.aux] : 0;
            bool ok = go;
            if (go) {
              if (row < e.row_cap && idx < e.row_cap && a.v >= 0) {
                e.leaf_row[idx] = row;
                e.leaf_tok[idx] = (uint32_t)a.v;
                r = (long long)row;   // level 0
                slots[I.aux] = r;
                present |= 1u << I.aux;
              } else {
                raise(c, a.v < 0 ? TDF_ERR_BAD_ARG : TDF_ERR_TABLE_FULL);
                ok = false;
              }
            }
            put(I.dst, r, had || ok, false);
            live = had || ok;
            break;
          }
          case D_CELL: {
            const Src a = src(0), b = src(1);
            const bool had = on && ((present >> I.aux) & 1);
            const bool go = on && a.p && b.p && !a.d && !b.d && !had;
            const uint32_t j = wave_alloc(go, &c->n_cell);
            const uint32_t row = wave_alloc(go, &c->n_rows);
            long long r = had ? slots[I.aux] : 0;
            bool ok = go;
            uint32_t lvl = 0;
            if (go) {
              if (row < e.row_cap && j < e.row_cap) {
                const uint32_t la = (uint32_t)(a.v >> 32), lb = (uint32_t)(b.v >> 32);
                lvl = 1 + (la > lb ? la : lb);
                e.cell_out[j] = row;
                e.cell_l[j] = (uint32_t)a.v;
                e.cell_r[j] = (uint32_t)b.v;
                e.cell_lvl[j] = lvl;
                r = (long long)row | ((long long)lvl << 32);
                slots[I.aux] = r;
                present |= 1u << I.aux;
              } else {
                raise(c, TDF_ERR_TABLE_FULL);
                ok = false;
              }
            }
            if (__ballot(go)) wave_max(ok ? lvl : 0, &c->max_level);
            put(I.dst, r, had || ok, false);
            live = had || ok;
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
            (void)wave_alloc(go, &c->n_head);
            put(I.dst, had ? slots[I.aux] : (long long)(frame - e.cap), had || go, false);
            live = had || go;
            break;
          }
          default: break;
        }
        // live firings per static-graph node: counted the first time the entry is live
        const bool first_time = live && !(fired & ibit);
        if (first_time) fired |= ibit;
        const uint16_t st = P.stat_idx[first + ip];
        if (st != 0xFFFF) wave_count(first_time, &e.fire_count[st]);
      }
    }
    if (active && (fired != fired_in || present != present_in)) {
      h->fired = fired;
      if (present != present_in) atomicOr(&h->present_fn, present & ~present_in);
    }
  }
}

// A step is "small" when its touched frames fit a few passes of one workgroup; small steps
// run in k_steps_small, the others in the grid-wide k_fire / k_match pair.
__device__ __forceinline__ bool step_is_small(const Engine& e, uint32_t n) { return n <= e.small_limit; }

__global__ void k_fire(DevProgram P, Engine e) {
  extern __shared__ long long regs[];
  Ctrl* c = e.ctrl;
  const uint32_t n = __atomic_load_n(&c->touched_count[c->step & 1], __ATOMIC_RELAXED);
  if (c->done || n == 0 || step_is_small(e, n)) return;
  fire_pass(P, e, n, blockIdx.x * blockDim.x, gridDim.x * blockDim.x, regs);
}

// ---- step bookkeeping: reset the consumed lists, count the step, detect the end -------------
__device__ void advance(const Engine& e, int parity) {
  Ctrl* c = e.ctrl;
  const uint32_t next = __atomic_load_n(&c->touched_count[parity ^ 1], __ATOMIC_RELAXED);
  const unsigned long long n_tags = __atomic_load_n(&c->n_tags, __ATOMIC_RELAXED);
  uint32_t status = __atomic_load_n(&c->status, __ATOMIC_RELAXED);
  __atomic_store_n(&c->q_count, 0u, __ATOMIC_RELAXED);
  __atomic_store_n(&c->touched_count[parity], 0u, __ATOMIC_RELAXED);
  c->step += 1;
  if (n_tags > e.max_tags && status == 0) status = (uint32_t)(-TDF_ERR_TABLE_FULL);
  if (c->step >= e.step_limit && next != 0 && status == 0) status = (uint32_t)(-TDF_ERR_STEP_LIMIT);
  if (status != 0) {
    __atomic_store_n(&c->status, status, __ATOMIC_RELAXED);
    __atomic_store_n(&c->touched_count[parity ^ 1], 0u, __ATOMIC_RELAXED);   // drain: nothing more fires
    c->done = 1;
  } else if (next == 0) {
    c->done = 1;
  }
}

// ---- match -------------------------------------------------------------------------------
// One pass over the tokens [0, n) of the queue.
__device__ void match_pass(const DevProgram& P, const Engine& e, int parity, uint32_t n, uint32_t stamp,
                           uint32_t first, uint32_t lane_stride) {
  Ctrl* c = e.ctrl;
  const int stride = P.frame_stride;
  for (uint32_t base = first; base < n; base += lane_stride) {
    const uint32_t i = base + threadIdx.x;
    const bool active = i < n;
    bool inserted = false, deliver = false;
    uint32_t target = 0, probes = 0, depth = 0;
    if (active) {
      const Token t = e.queue[i];
      if (t.b & 0x80000000u) {
        // Call_i: <t,d> -> <i:t,d>.  The tag i:t is the key (frame of t, i).
        const uint32_t label = t.b & 0xFFu, param = (t.b >> 8) & 0xFFu;
        const unsigned long long key = ((unsigned long long)(t.a + 1u) << 32) | (label + 1u);
        uint32_t s = (uint32_t)mix64(key) & e.cap_mask;
        bool found = false;
        const uint32_t probe_limit = e.cap < 8192u ? e.cap : 8192u;
        for (probes = 1; probes <= probe_limit; ++probes) {
          FrameHdr* h = frame_at(e, stride, s);
          unsigned long long cur = __atomic_load_n(&h->key, __ATOMIC_RELAXED);
          if (cur == 0) {
            cur = atomicCAS(&h->key, 0ull, key);
            if (cur == 0) {
              inserted = found = true;
              break;
            }
          }
          if (cur == key) {
            found = true;
            break;
          }
          s = (s + 1) & e.cap_mask;
        }
        if (found) {
          FrameHdr* h = frame_at(e, stride, s);
          const uint32_t fn = P.label_callee[label];
          if (inserted) {
            depth = frame_at(e, stride, t.a)->depth + 1;
            h->depth = depth;
          }
          frame_slots(h)[param] = t.value;
          atomicOr(&h->present_fn, (1u << param) | (fn << 24));
          target = s;
          deliver = true;
        } else {
          raise(c, TDF_ERR_TABLE_FULL);
        }
      } else {
        // Return_i: <i:t,d> -> <t,d>.  The frame's own key names its label i and the frame
        // of t, so only the Return_i of the call that created the frame produces output.
        const unsigned long long key = __atomic_load_n(&frame_at(e, stride, t.a)->key, __ATOMIC_RELAXED);
        const uint32_t parent = (uint32_t)(key >> 32) - 1u, label = (uint32_t)key - 1u;
        FrameHdr* h = frame_at(e, stride, parent);
        const uint32_t slot = P.label_ret_slot[label];
        frame_slots(h)[slot] = t.value;
        atomicOr(&h->present_fn, 1u << slot);
        target = parent;
        deliver = true;
      }
    }
    // ready-frame compaction: the first token to reach a frame in this step appends it
    bool first = false;
    if (deliver) first = atomicExch(&frame_at(e, stride, target)->touched, stamp) != stamp;
    const uint32_t pos = wave_alloc(first, &c->touched_count[parity ^ 1]);
    if (first) {
      if (pos < e.touched_cap) e.touched[pos] = target;
      else raise(c, TDF_ERR_TABLE_FULL);
    }
    wave_count(inserted, &c->n_tags);
    wave_count(active, &c->n_tokens);
    if (__ballot(inserted)) {
      wave_max(inserted ? probes : 0, &c->max_probe);
      wave_max(depth, &c->max_depth);
    }
  }
}

__global__ void __launch_bounds__(MATCH_BLOCK) k_match(DevProgram P, Engine e) {
  Ctrl* c = e.ctrl;
  const uint32_t step = c->step;
  const int parity = (int)(step & 1);
  const uint32_t n_touched = __atomic_load_n(&c->touched_count[parity], __ATOMIC_RELAXED);
  if (c->done || n_touched == 0 || step_is_small(e, n_touched)) return;   // same test as k_fire
  const uint32_t n = __atomic_load_n(&c->q_count, __ATOMIC_RELAXED);
  match_pass(P, e, parity, n, step + 1, blockIdx.x * blockDim.x, gridDim.x * blockDim.x);
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
    __atomic_store_n(&c->blocks_done, 0u, __ATOMIC_RELAXED);
    advance(e, parity);
  }
}

// Small steps: one workgroup runs fire and match back to back, step after step, with workgroup
// barriers only.  Returns when the recursion is finished, when a step is too large for one
// workgroup, or after max_steps steps.
__global__ void k_steps_small(DevProgram P, Engine e, int max_steps) {
  extern __shared__ long long regs[];
  __shared__ uint32_t sh[3];
  Ctrl* c = e.ctrl;
  for (int it = 0; it < max_steps; ++it) {
    if (threadIdx.x == 0) {
      const uint32_t step = c->step;
      sh[0] = step;
      sh[1] = __atomic_load_n(&c->touched_count[step & 1], __ATOMIC_RELAXED);
      sh[2] = c->done;
    }
    __syncthreads();
    const uint32_t step = sh[0], n = sh[1], stop = sh[2];
    __syncthreads();
    if (stop || n == 0 || !step_is_small(e, n)) return;
    const int parity = (int)(step & 1);
    fire_pass(P, e, n, 0, blockDim.x, regs);
    __threadfence();
    __syncthreads();
    const uint32_t qn = __atomic_load_n(&c->q_count, __ATOMIC_RELAXED);
    match_pass(P, e, parity, qn, step + 1, 0, blockDim.x);
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) advance(e, parity);
    __syncthreads();
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

// One round of the tag machine: as many small steps as fit (one workgroup), then one
// grid-wide step if the next step is large.  Each kernel decides on the device whether the
// current step is its own.
void launch_round(const DevProgram& P, const Engine& e, int max_values, int blocks, int small_block,
                  int small_steps, hipStream_t s) {
  const size_t small_lds = (size_t)max_values * small_block * sizeof(long long);
  if (small_lds > 48 * 1024)   // large value files need the LDS opt-in
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_steps_small),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_lds);
  hipLaunchKernelGGL(k_steps_small, dim3(1), dim3(small_block), small_lds, s, P, e, small_steps);
  hipLaunchKernelGGL(k_fire, dim3(blocks), dim3(FIRE_BLOCK), (size_t)max_values * FIRE_BLOCK * sizeof(long long), s, P, e);
  hipLaunchKernelGGL(k_match, dim3(blocks), dim3(MATCH_BLOCK), 0, s, P, e);
}

void launch_levels(const Engine& e, uint32_t n_cell, hipStream_t s) {
  int g = grid_for(n_cell, 256, 2048);
  hipLaunchKernelGGL(k_level_hist, dim3(g), dim3(256), 0, s, e);
  hipLaunchKernelGGL(k_level_scan, dim3(1), dim3(1024), 0, s, e);
  hipLaunchKernelGGL(k_level_scatter, dim3(g), dim3(256), 0, s, e);
}

}  // namespace tdf
