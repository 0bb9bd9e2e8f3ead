// Device-side data layout of one evaluation, shared by the tag machine (tag_machine.hip),
// the vector kernels (cells.hip) and the host driver (eval.hip).
#pragma once
#ifndef __HIPCC_RTC__ /* the run-time compiler provides the HIP device API implicitly */
#include <hip/hip_runtime.h>
#endif
#include <stdint.h>

#include "tdf_tables.h"

namespace tdf {

// Control block of one tag machine, at the head of the workspace.  Counters are bumped with
// device-scope atomics; everything else is ordered by kernel boundaries.  One 128-byte line per
// machine: machines run on different dies and must not share a line.
struct alignas(128) Ctrl {
  uint32_t touched_count[2]; // frames that received a token (double-buffered by step parity)
  uint32_t step;
  uint32_t n_leaf;           // EMBED firings
  uint32_t n_cell;           // cell firings
  uint32_t n_head;           // CE_HEAD firings
  uint32_t status;           // 0, or -(tdf_status) raised on the device
  uint32_t done;
  uint32_t n_alloc;          // frames handed out so far: the next free record of this machine's part
  // Frames given back by finished tags (forward evaluation of integer programs): a ring of frame
  // ids.  A step takes from the head only what was given back before the step began (up to
  // free_limit) and gives back at the tail, so takers and givers never meet on an entry.
  uint32_t free_head, free_tail, free_limit;   // monotone counters, ring index = counter % part
  uint32_t max_depth, max_level;
  uint32_t bar_count;        // grid barrier of the grid-wide step kernel: arrivals (monotone)
  uint32_t bar_gen;          // ... and completed barriers
  uint32_t wbar_count, wbar_gen;   // the same for the device-wide kernel (another number of workgroups)
  uint32_t xcc_mask;         // accelerator dies that ran a die-local grid-wide step kernel
  uint32_t prev_count;       // frames of the previous step
  uint32_t peak_count;       // ... and of the largest step so far
  uint32_t same_steps;       // steps in a row, before this one, with exactly as many frames as their predecessor
  unsigned long long n_tags, n_tokens;
};

// Frame record = one call-context tag (Section 5.1: a frame holds the label i of the Call_i that
// created it and a reference to the previous scope).  The key packs (parent frame + 1, iteration
// counter, label + 1): a tag of the paper is (iteration number, pointer into the frame stack), and
// a loop scope is pushed on the same stack as a function scope (Section 5.1).  Enter is the push
// of a scope with counter 0, so the frame of a call is the frame of "iteration 0" of its label;
// Next keeps parent and label and adds one to the counter; Exit pops like Return.
//
// The match table is keyed by (frame of t, i) and needs no probing: all Call_i tokens of one
// call come from sweeps of the caller's frame, so the entry for (frame of t, i) is a child link
// inside that frame's own record, one per call site of its function (and one for the next
// iteration of a loop).  The first token of a call finds the link empty, takes the next free
// record of its machine (wave ballot + prefix sum, one counter bump per wave) and writes the
// link; later tokens of the same call follow the link.  Records are handed out in creation
// order: frames that are created together, and completed together, share cache lines.  The lane
// that creates a frame writes its header; records beyond the machine's counter are never read.
//
// Tokens delivered during step s set bits in the arrival word of step s+1; the sweep of step
// s+1 takes that word (exchange with 0) and folds it into present_fn, which only the sweeping
// lane writes.  The delivery that finds the word empty is the first to reach the frame in that
// step and puts it on the next list.  Values delivered in one step are read in a later one, so
// only arrived[] is ever accessed concurrently and needs atomics.
struct FrameHdr {
  unsigned long long key;     // (parent + 1) << 32 | iteration << 8 | (label + 1)
  unsigned long long fired;   // firing-table entries that have fired live under this tag
  uint32_t present_fn;        // bits 0..23: stored values present; bits 24..31: function
  uint32_t depth;             // length of the tag: call labels and iteration counters below the root
  uint32_t arrived[2];        // same layout as present_fn, by parity of the consuming step
  // followed by int64 stored[max_stored], then uint32 link[n_links] (frame id + 1 of the scope opened at
  // each site, 0 = not opened yet)
};
static_assert(sizeof(FrameHdr) == 32, "FrameHdr must be 32 bytes");

constexpr uint32_t LEVEL_KEY_DIES = 8;
constexpr uint32_t STEP_LOG_CAP = 8192;   // steps per machine whose size and time are recorded on request

// Pointers into the workspace and to the caller's buffers, passed to kernels by value.
//
// The instances of a batch never exchange tokens (their tags differ in the root), so the batch
// is dealt to n_dies independent tag machines, instance b to machine b % n_dies.  A machine
// has its own control block, its own part of the frame records (plus the root records of its
// instances), its own touched lists and its own schedule log; nothing it touches during the
// steps is touched by another machine.  Each machine runs
// on one accelerator die (XCD), so its atomics and step boundaries stay inside that die's L2.
// Kernels receive the description of the whole engine and take the view of their machine
// (die_view); after the last step the logs of the machines are merged.
struct Engine {
  const DevProgram* prog;           // firing tables in the workspace (copied there once per call)
  Ctrl* ctrl;                       // [n_dies]; in a machine's view: its own block
  uint32_t n_dies;                  // machines: 1, 2, 4 or 8
  uint32_t die;                     // view: this machine
  uint32_t key_base, part;          // view: first frame record of this machine's part; records per part
  // per-machine schedule logs [n_dies][log_cap] (with one machine they are the merged logs below)
  uint32_t *m_leaf_row, *m_leaf_tok, *m_cell_out, *m_cell_l, *m_cell_r, *m_cell_lvl;
  unsigned long long* fire_count;   // [TDF_STATS_MAX_COUNTS]
  char* frames;                     // (cap + B) records of frame_stride bytes: n_dies parts, then the root records
  uint4* step_log;                  // per machine STEP_LOG_CAP records {frames of the step, frames handed out so far, 100 MHz clock
                                    // at the step's end, 0}, or null (statistics level 2)
  uint32_t* free_ring;              // per machine `part` frame ids (see Ctrl::free_head); null: frames are kept until the call ends
  uint32_t reclaim;                 // 1: a frame is given back once its tag has finished (Section 5.1: Return_i deallocates)
  uint32_t cap, n_inst, max_tags;   // cap = n_dies * part
  uint32_t* touched;                // per machine two lists of touched_cap frame ids, by step parity
  uint32_t touched_cap;
  uint32_t step_limit;
  uint32_t small_limit;             // steps with at most this many touched frames run in one workgroup
  uint32_t wide_limit;              // 0, or: a machine's steps with more frames than this run in the device-wide kernel
                                    // on every die's compute units (batches that leave dies without a machine)
  uint32_t follow_limit;            // in single-workgroup steps with at most this many frames a lane goes on with the frame it created
  // forest
  const int32_t *left, *right, *token;
  int32_t n_tree_nodes;
  int32_t vocab;                    // rows of the embedding table: EMBED rejects token ids beyond it
  // program inputs / outputs
  const long long* args;
  int32_t n_args;
  long long* out_i64;
  uint32_t* root_ref;               // [B] row of the vector result of instance b
  uint32_t* root_lvl;               // [B] dependency level of that row: the height of instance b's recursion
  uint32_t* inst_class;             // [B] 1: a deep instance, scheduled apart (set after the tag machine; null: one class)
  // schedule log written by the step kernels; a vector value is named by the frame that produced it
  // until the rows are numbered
  uint32_t log_cap;                 // entries of the leaf / cell logs (0: no vector operators)
  uint32_t *leaf_row, *leaf_tok;    // [n_leaf]
  uint32_t *cell_out, *cell_l, *cell_r, *cell_lvl;   // [n_cell], in firing order; cell_lvl holds the sort key
  uint32_t *head_row, *head_label;  // [B]
  // cells bucketed by dependency level
  // The log's sort key is level * LEVEL_KEY_DIES + machine: a level is one contiguous range of
  // the sorted log, and inside it the cells of every machine (die) are contiguous too.
  uint32_t *level_count, *level_off, *level_fill;    // [(max_levels + 2) * LEVEL_KEY_DIES]
  uint32_t max_levels;
  uint32_t *q_out, *q_l, *q_r;      // [n_cell], sorted by level: producing frame, then (after the rows are numbered) the children's rows
  // State rows are numbered by the sorted schedule, not by frame: leaf i of the leaf log has row i,
  // the cell at position q of the sorted log has row row0 + q (row0 = number of leaves).  Every
  // level then reads scattered child rows but writes one contiguous block, and the state arrays
  // hold only rows that exist.
  uint32_t row0;                    // first cell row (set by the host once the tag machine has finished)
  uint32_t* row_of;                 // [cap + n_inst]: row of the value a frame produced (valid for logged frames)
  uint32_t* row_node;               // [cap + n_inst]: tree node whose loss term the frame's row gets (CE_NODE), ~0: none
  uint32_t* node_of_row;            // [rows]: the same by row
};

// The engine as machine d sees it.
inline __host__ __device__ Engine die_view(const Engine& e, uint32_t d) {
  Engine v = e;
  v.die = d;
  v.ctrl = e.ctrl + d;
  v.key_base = d * e.part;
  v.touched = e.touched + (size_t)d * 2 * e.touched_cap;
  v.free_ring = e.free_ring ? e.free_ring + (size_t)d * e.part : nullptr;
  v.step_log = e.step_log ? e.step_log + (size_t)d * STEP_LOG_CAP : nullptr;
  const size_t o = (size_t)d * e.log_cap;
  v.leaf_row = e.m_leaf_row + o;
  v.leaf_tok = e.m_leaf_tok + o;
  v.cell_out = e.m_cell_out + o;
  v.cell_l = e.m_cell_l + o;
  v.cell_r = e.m_cell_r + o;
  v.cell_lvl = e.m_cell_lvl + o;
  return v;
}
inline __device__ FrameHdr* frame_at(const Engine& e, int stride, uint32_t f) {
  return reinterpret_cast<FrameHdr*>(e.frames + (size_t)f * stride);
}
inline __device__ long long* frame_slots(FrameHdr* h) {
  return reinterpret_cast<long long*>(h + 1);
}
inline __device__ uint32_t* frame_links(FrameHdr* h, int links_off) {
  return reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(h) + links_off);
}

// ---- wave-level helpers (64-wide wavefronts) ------------------------------------------------
inline __device__ unsigned lane_id() { return __lane_id(); }

inline __device__ unsigned long long lanemask_lt() {
  return (1ull << lane_id()) - 1ull;
}

// Wave-level compaction: lanes with `take` get consecutive positions from *counter.
// Must be reached by every lane of the wave.
inline __device__ uint32_t wave_alloc(bool take, uint32_t* counter) {
  unsigned long long m = __ballot(take);
  if (m == 0) return 0;
  int leader = __ffsll((long long)m) - 1;
  uint32_t base = 0;
  if ((int)lane_id() == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
  base = __shfl(base, leader);
  return base + (uint32_t)__popcll(m & lanemask_lt());
}

// Frame records for the new scopes of a wave (two requests per lane at once).  With `ring` set,
// frames that finished tags gave back before this step are taken first (one bump of the ring's head
// per wave), the rest comes from the machine's part (one bump of its counter).  f0 / f1: record index
// inside the part, or >= part where the part is exhausted.
template <int SCOPE>
inline __device__ void wave_take_frames(bool take0, bool take1, uint32_t* n_alloc, uint32_t* free_head, const uint32_t* free_limit,
                                        const uint32_t* ring, uint32_t part, uint32_t& f0, uint32_t& f1) {
  const unsigned long long m0 = __ballot(take0), m1 = __ballot(take1);
  f0 = f1 = 0;
  if ((m0 | m1) == 0) return;
  const int leader = __ffsll((long long)(m0 | m1)) - 1;
  const uint32_t n = (uint32_t)(__popcll(m0) + __popcll(m1));
  uint32_t h = 0, got = 0, base = 0;
  if ((int)lane_id() == leader) {
    if (ring) {
      const uint32_t limit = __hip_atomic_load(free_limit, __ATOMIC_RELAXED, SCOPE);
      if ((int)(limit - __hip_atomic_load(free_head, __ATOMIC_RELAXED, SCOPE)) > 0) {
        h = __hip_atomic_fetch_add(free_head, n, __ATOMIC_RELAXED, SCOPE);
        const int avail = (int)(limit - h);
        got = avail <= 0 ? 0u : ((uint32_t)avail < n ? (uint32_t)avail : n);
      }
    }
    if (got < n) base = __hip_atomic_fetch_add(n_alloc, n - got, __ATOMIC_RELAXED, SCOPE);
  }
  h = __shfl(h, leader);
  got = __shfl(got, leader);
  base = __shfl(base, leader);
  const uint32_t r0 = (uint32_t)__popcll(m0 & lanemask_lt());
  const uint32_t r1 = (uint32_t)__popcll(m0) + (uint32_t)__popcll(m1 & lanemask_lt());
  // (ring entries were written in earlier steps, maybe by another compute unit: read past the L1)
  if (take0) f0 = r0 < got ? __hip_atomic_load(&ring[(h + r0) % part], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : base + (r0 - got);
  if (take1) f1 = r1 < got ? __hip_atomic_load(&ring[(h + r1) % part], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : base + (r1 - got);
}

// Lanes with `take` get unique consecutive positions in counters[key]; lanes of the wave
// that share a key are served by one atomic.  Must be reached by every lane of the wave.
inline __device__ uint32_t wave_alloc_keyed(bool take, uint32_t key, uint32_t* counters) {
  uint32_t pos = 0;
  unsigned long long todo = __ballot(take);
  while (todo) {
    const int leader = __ffsll((long long)todo) - 1;
    const uint32_t k0 = __shfl(key, leader);
    const unsigned long long same = __ballot(take && key == k0) & todo;
    uint32_t base = 0;
    if ((int)lane_id() == leader) base = atomicAdd(&counters[k0], (uint32_t)__popcll(same));
    base = __shfl(base, leader);
    if ((same >> lane_id()) & 1) pos = base + (uint32_t)__popcll(same & lanemask_lt());
    todo &= ~same;
  }
  return pos;
}

template <int SCOPE>
inline __device__ uint32_t wave_alloc_scoped(bool take, uint32_t* counter) {
  unsigned long long m = __ballot(take);
  if (m == 0) return 0;
  int leader = __ffsll((long long)m) - 1;
  uint32_t base = 0;
  if ((int)lane_id() == leader) base = __hip_atomic_fetch_add(counter, (uint32_t)__popcll(m), __ATOMIC_RELAXED, SCOPE);
  base = __shfl(base, leader);
  return base + (uint32_t)__popcll(m & lanemask_lt());
}

inline __device__ void wave_count32(bool take, uint32_t* counter) {
  unsigned long long m = __ballot(take);
  if (m && (int)lane_id() == __ffsll((long long)m) - 1) atomicAdd(counter, (uint32_t)__popcll(m));
}

inline __device__ void wave_count(bool take, unsigned long long* counter) {
  unsigned long long m = __ballot(take);
  if (m && (int)lane_id() == __ffsll((long long)m) - 1)
    atomicAdd(counter, (unsigned long long)__popcll(m));
}

// Maximum over the 64 lanes of a wave (row-wise DPP shifts, then row broadcasts; lane 63 holds
// the result).  Must be reached by every lane of the wave; lanes without a value pass 0.
template <int CTRL, int ROW_MASK>
inline __device__ uint32_t dpp_umax(uint32_t x) {
  const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xf, false);
  return o > x ? o : x;
}
inline __device__ uint32_t wave_umax(uint32_t v) {
  v = dpp_umax<0x111, 0xf>(v);   // row_shr:1
  v = dpp_umax<0x112, 0xf>(v);   // row_shr:2
  v = dpp_umax<0x114, 0xf>(v);   // row_shr:4
  v = dpp_umax<0x118, 0xf>(v);   // row_shr:8
  v = dpp_umax<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v = dpp_umax<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// ---- vector side ----------------------------------------------------------------------
struct VecArgs {
  int dtype;        // tdf_dtype
  int cell_kind;    // 1 RNN, 2 LSTM
  int H, Hp;        // hidden size and padded row stride (multiple of 64)
  int N, Np;        // gate rows of W: H or 5H; padded: Hp or 5*Hp
  int Kp;           // 2*Hp
  int vocab, n_classes;
  const void* E;
  const void* W;
  const float* b;
  const float *U, *u0;
  void* Hs;         // state rows [rows x Hp], dtype (rows: capacity max_tags)
  float* Cs;        // LSTM cell state [rows x Hp]
  void* Wp;         // packed W [Np x Kp], dtype (k contiguous)
  float* bp;        // [Np]
  // gradient side
  float* dH;        // [rows x Hp]
  float* dC;        // [rows x Hp]
  void* gates;      // LSTM activations (i,f_l,f_r,o,u) [n_cell x Np], dtype, by level order q
  void* Dz;         // pre-activation gradients [n_cell x Np], dtype, by q
  void* DzT;        // [Np x q_stride]
  void* XT;         // [Kp x q_stride]  (gathered [h_l;h_r] transposed)
  void* WpT;        // packed W transposed [Kp x Np]
  void* Wf;         // Wp and WpT in MFMA operand order, for the small-level kernel
  void* WfT;
  float* dW_part;   // split partial sums [n_split x Np x Kp]
  uint32_t q_stride;
  float* loss;      // [B]
  uint32_t* gmark;  // [rows] gradient runs: how often the gradient body of a row's tag has fired (cleared per call)
  float* dHn;       // [rows x Hp] gradient of each row's own loss term (CE_NODE, gradient runs; else null):
                    // whoever reads a row of dH adds the row of dHn
  int wide_offsets; // only the build for the tests sets it: kernels with a 32-bit and a 64-bit offset path take the latter
};

}  // namespace tdf
