// Kernels and launchers of the tag machine.  The step logic itself is in step_device.h; this
// file instantiates it with the table interpreter and adds the seed, the post-run firing
// counts and the bucketing of the cell log by dependency level.
#include <stdlib.h>

#include "bucket.h"
#include "step_device.h"
#include "tdf_internal.h"

namespace tdf {

namespace {

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
  h->depth = 0;
  h->fired = 0;
  h->present_fn = ((1u << np) - 1u) | ((uint32_t)P.result_fn << 24);
  h->arrived[0] = h->arrived[1] = 0;
  for (int k = 0; k < P.n_links; ++k) frame_links(h, P.links_off)[k] = 0u;
  if (P.inst_off) *frame_links(h, P.inst_off) = b;
  // instance b belongs to machine b % n_dies
  const uint32_t d = b % e.n_dies, pos = b / e.n_dies;
  e.touched[(size_t)d * 2 * e.touched_cap + pos] = f;
  if (pos == 0) e.ctrl[d].touched_count[0] = (e.n_inst - d + e.n_dies - 1) / e.n_dies;
}

// ---- after the last step: the machines' schedule logs, one after the other ------------------
struct LogOffsets {
  uint32_t leaf[9], cell[9];   // first entry of machine d in the merged logs; [n_dies] = totals
};
__global__ void k_merge_logs(Engine e, LogOffsets o) {
  const uint32_t d = blockIdx.y;
  const Engine m = die_view(e, d);
  const uint32_t n_leaf = o.leaf[d + 1] - o.leaf[d], n_cell = o.cell[d + 1] - o.cell[d];
  for (uint32_t j = blockIdx.x * blockDim.x + threadIdx.x; j < n_leaf; j += gridDim.x * blockDim.x) {
    e.leaf_row[o.leaf[d] + j] = m.leaf_row[j];
    e.leaf_tok[o.leaf[d] + j] = m.leaf_tok[j];
  }
  for (uint32_t j = blockIdx.x * blockDim.x + threadIdx.x; j < n_cell; j += gridDim.x * blockDim.x) {
    e.cell_out[o.cell[d] + j] = m.cell_out[j];
    e.cell_l[o.cell[d] + j] = m.cell_l[j];
    e.cell_r[o.cell[d] + j] = m.cell_r[j];
    e.cell_lvl[o.cell[d] + j] = m.cell_lvl[j];
  }
}

template <int NV, bool LOCAL>
__global__ void __launch_bounds__(LOCAL ? LOCAL_BLOCK : STEP_BLOCK) k_steps_grid(Engine e, int max_steps, long long spin_ticks) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ DevProgram P;
  __shared__ uint32_t sh[4];
  steps_grid<LOCAL, InterpSweep<NV>>(e, max_steps, spin_ticks, lds, &P, sh);
}

template <int NV>
__global__ void __launch_bounds__(512) k_steps_small(Engine e, int max_steps) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ DevProgram P;
  __shared__ Ctrl lc;
  steps_small<InterpSweep<NV>>(e, max_steps, lds, &P, &lc);
}

// ---- statistics: live firings per static-graph node, counted from the fired masks -------------
__global__ void k_count_fired(DevProgram P, Engine e) {
  __shared__ uint32_t cnt[MAX_INSTR];
  for (int i = threadIdx.x; i < MAX_INSTR; i += blockDim.x) cnt[i] = 0;
  __syncthreads();
  const uint32_t total = e.cap + e.n_inst;
  for (uint32_t f = blockIdx.x * blockDim.x + threadIdx.x; f < total; f += gridDim.x * blockDim.x) {
    if (f < e.cap && f % e.part >= e.ctrl[f / e.part].n_alloc) continue;   // not handed out: the record holds stale bytes
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
__global__ void k_level_hist(Engine e, uint32_t n) {
  for (uint32_t base = blockIdx.x * blockDim.x; base < n; base += gridDim.x * blockDim.x) {
    const uint32_t j = base + threadIdx.x;
    (void)wave_alloc_keyed(j < n, j < n ? e.cell_lvl[j] : 0, e.level_count);
  }
}

struct LevelSink {   // the level-sorted copy of the cell log
  Engine e;
  __device__ void operator()(uint32_t j, uint32_t q) const {
    e.q_out[q] = e.cell_out[j];
    e.q_l[q] = e.cell_l[j];
    e.q_r[q] = e.cell_r[j];
  }
};

__global__ void k_level_scan(Engine e, uint32_t n_keys) {
  // single block; exclusive scan over the sort keys
  __shared__ uint32_t carry;
  __shared__ uint32_t buf[1024];
  const uint32_t L = n_keys;
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

__global__ void k_level_scatter(Engine e, uint32_t n) {
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

// Workgroup size of a generated kernel: `name` in the environment (a multiple of 64 up to the
// kernel's launch bound), else `def`.
static int env_block(const char* name, int def, int max) {
  const char* e = getenv(name);
  const int v = e ? atoi(e) : def;
  return v >= 64 && v <= max && v % 64 == 0 ? v : def;
}

// Lanes of the single-workgroup kernel: as many as the per-lane LDS footprint allows.
int tag_machine_small_block(const DevProgram& P, bool jit) {
  const Sizes z = sizes_of(P);
  const bool lds_values = !jit && !fits_registers(z);
  int rb = 512;
  if (jit) rb = env_block("TDF_SMALL_BLOCK", 512, GEN_SMALL_BLOCK);
  // generated kernels are module functions, launched without an LDS opt-in: 64 KB at most
  const size_t lds_limit = jit ? 64 * 1024 : 120 * 1024;
  while (rb > 64 && step_lds_bytes(z, rb, lds_values) > lds_limit) rb >>= 1;
  return rb;
}

// One round of the tag machine: a run of small steps (one workgroup), then a run of grid-wide
// steps.  Each kernel decides on the device whether the current step is its own and returns at
// once if not.  The workgroups of the grid-wide kernel must all be resident at once: one per
// compute unit (`cus`); with `local` one per compute unit of a single accelerator die, which is
// every eighth workgroup of a launch eight times as large.  jit: kernels generated for this
// program by the run-time compiler (used when all handles are set), else the table
// interpreter.  spin_ticks bounds the wait at the grid barrier (100 MHz ticks).
tdf_status launch_round(const DevProgram& P, const Engine& e, int cus, bool local, int small_block, int max_steps,
                        long long spin_ticks, const JitKernels& jit, hipStream_t s) {
  const Sizes z = sizes_of(P);
  const int per_die = cus / (int)XCDS > 0 ? cus / (int)XCDS : 1;
  const int grid = local ? per_die * (int)XCDS : cus / (int)e.n_dies * (int)e.n_dies;
  const bool also_wide = local && e.wide_limit != 0;   // a third kernel for the steps too wide for one die
  const int wide_grid = cus / (int)e.n_dies * (int)e.n_dies;
  if (jit.small && jit.step && jit.step_local) {
    Engine ev = e;
    int ms = max_steps;
    long long st = spin_ticks;
    void* a_small[] = {&ev, &ms};
    void* a_step[] = {&ev, &ms, &st};
    int gb = local ? env_block("TDF_LOCAL_BLOCK", 256, GEN_LOCAL_BLOCK) : STEP_BLOCK;
    while (gb > 64 && step_lds_bytes(z, gb, false) > 64 * 1024) gb >>= 1;   // no LDS opt-in for module functions
    hipError_t r = hipModuleLaunchKernel((hipFunction_t)jit.small, e.n_dies, 1, 1, small_block, 1, 1,
                                         (unsigned)step_lds_bytes(z, small_block, false), s, a_small, nullptr);
    if (r == hipSuccess)
      r = hipModuleLaunchKernel((hipFunction_t)(local ? jit.step_local : jit.step), grid, 1, 1, gb, 1, 1,
                                (unsigned)step_lds_bytes(z, gb, false), s, a_step, nullptr);
    if (r == hipSuccess && also_wide) {
      int wb = STEP_BLOCK;
      while (wb > 64 && step_lds_bytes(z, wb, false) > 64 * 1024) wb >>= 1;
      r = hipModuleLaunchKernel((hipFunction_t)jit.step, wide_grid, 1, 1, wb, 1, 1, (unsigned)step_lds_bytes(z, wb, false), s, a_step,
                                nullptr);
    }
    if (r != hipSuccess) {
      set_error(std::string("launch of a generated step kernel failed: ") + hipGetErrorString(r));
      return TDF_ERR_DEVICE;
    }
    return TDF_OK;
  }
  const bool in_regs = fits_registers(z);
  const size_t small_lds = step_lds_bytes(z, small_block, !in_regs);
  if (small_lds > 48 * 1024)   // large value files need the LDS opt-in
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_steps_small<0>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_lds);
  if (in_regs) {
    hipLaunchKernelGGL(k_steps_small<16>, dim3(e.n_dies), dim3(small_block), small_lds, s, e, max_steps);
    if (local)
      hipLaunchKernelGGL((k_steps_grid<16, true>), dim3(grid), dim3(LOCAL_BLOCK), step_lds_bytes(z, LOCAL_BLOCK, false), s, e,
                         max_steps, spin_ticks);
    if (!local || also_wide)
      hipLaunchKernelGGL((k_steps_grid<16, false>), dim3(wide_grid), dim3(STEP_BLOCK), step_lds_bytes(z, STEP_BLOCK, false), s, e,
                         max_steps, spin_ticks);
  } else {
    // the LDS value file limits the workgroup to 128 lanes (at most 90 KB)
    const size_t grid_lds = step_lds_bytes(z, 128, true);
    if (grid_lds > 48 * 1024) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_steps_grid<0, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)grid_lds);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_steps_grid<0, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)grid_lds);
    }
    hipLaunchKernelGGL(k_steps_small<0>, dim3(e.n_dies), dim3(small_block), small_lds, s, e, max_steps);
    if (local)
      hipLaunchKernelGGL((k_steps_grid<0, true>), dim3(grid), dim3(128), grid_lds, s, e, max_steps, spin_ticks);
    if (!local || also_wide)
      hipLaunchKernelGGL((k_steps_grid<0, false>), dim3(wide_grid), dim3(128), grid_lds, s, e, max_steps, spin_ticks);
  }
  return TDF_OK;
}

// Copies the machines' logs into the merged logs; leaf_off / cell_off: n_dies + 1 prefix sums.
void launch_merge_logs(const Engine& e, const uint32_t* leaf_off, const uint32_t* cell_off, hipStream_t s) {
  if (e.n_dies <= 1) return;   // one machine writes the merged logs directly
  LogOffsets o{};
  for (uint32_t d = 0; d <= e.n_dies; ++d) {
    o.leaf[d] = leaf_off[d];
    o.cell[d] = cell_off[d];
  }
  hipLaunchKernelGGL(k_merge_logs, dim3(64, e.n_dies), dim3(256), 0, s, e, o);
}

void launch_count_fired(const DevProgram& P, const Engine& e, hipStream_t s) {
  hipLaunchKernelGGL(k_count_fired, dim3(grid_for(e.cap + e.n_inst, 256, 1024)), dim3(256), 0, s, P, e);
}

// Deep instances apart: an instance whose recursion is at least deep_level high gets its cells' sort
// keys moved behind all keys of the other instances (key + deep_base), so the sorted log holds first
// the shallow instances' cells by (level, machine), then the deep instances' by (level, machine).
__global__ void k_class_keys(Engine e, DevProgram P, uint32_t n_cell, uint32_t deep_level, uint32_t deep_base) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < e.n_inst) e.inst_class[i] = e.root_lvl[i] >= deep_level ? 1u : 0u;
  for (uint32_t j = i; j < n_cell; j += gridDim.x * blockDim.x) {
    const uint32_t inst = *frame_links(frame_at(e, P.frame_stride, e.cell_out[j]), P.inst_off);
    if (inst < e.n_inst && e.root_lvl[inst] >= deep_level) e.cell_lvl[j] += deep_base;
  }
}
void launch_class_keys(const DevProgram& P, const Engine& e, uint32_t n_cell, uint32_t deep_level, uint32_t deep_base, hipStream_t s) {
  const uint32_t n = n_cell > e.n_inst ? n_cell : e.n_inst;
  hipLaunchKernelGGL(k_class_keys, dim3(grid_for(n, 256, 1 << 20)), dim3(256), 0, s, e, P, n_cell, deep_level, deep_base);
}

// Counting sort of the cell log by sort key (n_keys keys); level_off[k] = first cell of key k.
void launch_levels(const Engine& e, uint32_t n_cell, uint32_t n_keys, hipStream_t s) {
  // (the two arrays lie one behind the other in the workspace: one fill)
  if (e.level_fill > e.level_count) {
    (void)hipMemsetAsync(e.level_count, 0, (size_t)((char*)(e.level_fill + n_keys) - (char*)e.level_count), s);
  } else {
    (void)hipMemsetAsync(e.level_count, 0, sizeof(uint32_t) * n_keys, s);
    (void)hipMemsetAsync(e.level_fill, 0, sizeof(uint32_t) * n_keys, s);
  }
  if (bucket_fits(n_keys)) {
    const size_t lds = (size_t)n_keys * 4;
    bucket_lds_opt_in(reinterpret_cast<const void*>(&k_bucket_count), n_keys);
    bucket_lds_opt_in(reinterpret_cast<const void*>(&k_bucket_place<LevelSink>), n_keys);
    hipLaunchKernelGGL(k_bucket_count, dim3(BUCKET_BLOCKS), dim3(BUCKET_THREADS), lds, s, e.cell_lvl, n_cell, n_keys,
                       e.level_count);
    hipLaunchKernelGGL(k_level_scan, dim3(1), dim3(1024), 0, s, e, n_keys);
    hipLaunchKernelGGL(k_bucket_place<LevelSink>, dim3(BUCKET_BLOCKS), dim3(BUCKET_THREADS), lds, s, e.cell_lvl, n_cell,
                       n_keys, e.level_off, e.level_fill, LevelSink{e});
    return;
  }
  int g = grid_for(n_cell, 256, 2048);
  hipLaunchKernelGGL(k_level_hist, dim3(g), dim3(256), 0, s, e, n_cell);
  hipLaunchKernelGGL(k_level_scan, dim3(1), dim3(1024), 0, s, e, n_keys);
  hipLaunchKernelGGL(k_level_scatter, dim3(g), dim3(256), 0, s, e, n_cell);
}

}  // namespace tdf
