// Run-time specialisation of the step kernels: the firing tables of a program are turned into
// straight-line HIP source (one block of code per table entry, values in named variables) and
// compiled for the current GPU with hiprtc.  The generated sweep replaces the table interpreter
// inside the same step logic (step_device.h), so both produce identical results.  hiprtc is
// loaded lazily; without it, or with TDF_NO_JIT=1, the interpreter is used.
#include <dlfcn.h>
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <mutex>
#include <sstream>
#include <string>
#include <vector>

#include "tdf_internal.h"

// headers of the device code as string literals, written by the build script
#include "embedded_headers.inc"

namespace tdf {

namespace {

// ---- the subset of the hiprtc API that is used, resolved with dlsym ------------------------------
typedef void* rtcProgram;
struct Rtc {
  int (*create)(rtcProgram*, const char*, const char*, int, const char* const*, const char* const*) = nullptr;
  int (*compile)(rtcProgram, int, const char* const*) = nullptr;
  int (*log_size)(rtcProgram, size_t*) = nullptr;
  int (*log)(rtcProgram, char*) = nullptr;
  int (*code_size)(rtcProgram, size_t*) = nullptr;
  int (*code)(rtcProgram, char*) = nullptr;
  int (*destroy)(rtcProgram*) = nullptr;
  bool ok = false;
};

Rtc& rtc() {
  static Rtc r;
  static std::once_flag once;
  std::call_once(once, [] {
    void* h = dlopen("libhiprtc.so.7", RTLD_NOW | RTLD_LOCAL);
    if (!h) h = dlopen("libhiprtc.so", RTLD_NOW | RTLD_LOCAL);
    if (!h) return;
    r.create = (decltype(r.create))dlsym(h, "hiprtcCreateProgram");
    r.compile = (decltype(r.compile))dlsym(h, "hiprtcCompileProgram");
    r.log_size = (decltype(r.log_size))dlsym(h, "hiprtcGetProgramLogSize");
    r.log = (decltype(r.log))dlsym(h, "hiprtcGetProgramLog");
    r.code_size = (decltype(r.code_size))dlsym(h, "hiprtcGetCodeSize");
    r.code = (decltype(r.code))dlsym(h, "hiprtcGetCode");
    r.destroy = (decltype(r.destroy))dlsym(h, "hiprtcDestroyProgram");
    r.ok = r.create && r.compile && r.log_size && r.log && r.code_size && r.code && r.destroy;
  });
  return r;
}

// ---- source generation ------------------------------------------------------------------------
struct Gen {
  std::ostringstream o;
  const DevProgram& P;
  explicit Gen(const DevProgram& p) : P(p) {}

  // value / present / dead expressions of source k of an entry
  static std::string val(const Instr& I, int k) {
    if (I.src[k] == SRC_IMM) return "(long long)" + std::to_string((unsigned long long)I.imm) + "ULL";
    return "v" + std::to_string(I.src[k]);
  }
  static std::string pre(const Instr& I, int k) { return I.src[k] == SRC_IMM ? "true" : "p" + std::to_string(I.src[k]); }
  static std::string ded(const Instr& I, int k) { return I.src[k] == SRC_IMM ? "false" : "d" + std::to_string(I.src[k]); }

  void function(int f) {
    const DevFn& fn = P.fn[f];
    o << "    {  // function " << f << "\n";
    o << "      const bool on = x.myfn == " << f << ";\n";
    o << "      if (__ballot(on) != 0) {\n";
    for (int v = 0; v < fn.n_values; ++v)
      o << "        long long v" << v << " = 0; bool p" << v << " = false, d" << v << " = false;\n";
    o << "        bool live = false, all_in = true;\n";
    for (int ip = 0; ip < fn.count; ++ip) {
      const Instr& I = P.instr[fn.first + ip];
      const std::string bit = "(1ull << " + std::to_string(ip) + ")";
      const std::string D = std::to_string(I.dst);
      o << "        {  // entry " << ip << " op " << (int)I.op << "\n";
      switch (I.op) {
        case D_IN:
          o << "          p" << D << " = on && ((x.present >> " << (int)I.aux << ") & 1); v" << D << " = x.sv[" << (int)I.aux
            << "]; live = p" << D << "; all_in = all_in && p" << D << ";\n";
          break;
        case D_RET: {
          std::string all_p = "true", any_d = "false";
          bool any_arg = false;
          for (int k = 0; k < 4; ++k) {
            if (I.src[k] == SRC_NONE) continue;
            any_arg = true;
            all_p += " && p" + std::to_string(I.src[k]);
            any_d += " || d" + std::to_string(I.src[k]);
          }
          o << "          const bool p = on && ((x.present >> " << (int)I.aux << ") & 1);\n";
          o << "          const bool is_dead = on && !p && " << (any_arg ? "true" : "false") << " && (" << all_p << ") && (" << any_d
            << ");\n";
          o << "          v" << D << " = x.sv[" << (int)I.aux << "]; p" << D << " = p || is_dead; d" << D << " = is_dead; live = p;\n";
          o << "          all_in = all_in && p" << D << ";\n";
          break;
        }
        case D_ADD: case D_SUB: case D_MUL: case D_EQ: case D_LT: {
          const std::string a = val(I, 0), b = val(I, 1);
          o << "          const bool p = on && " << pre(I, 0) << " && " << pre(I, 1) << "; const bool d = " << ded(I, 0) << " || "
            << ded(I, 1) << ";\n";
          if (I.op == D_ADD) o << "          v" << D << " = (long long)((unsigned long long)" << a << " + (unsigned long long)" << b << ");\n";
          if (I.op == D_SUB) o << "          v" << D << " = (long long)((unsigned long long)" << a << " - (unsigned long long)" << b << ");\n";
          if (I.op == D_MUL) o << "          v" << D << " = (long long)((unsigned long long)" << a << " * (unsigned long long)" << b << ");\n";
          if (I.op == D_EQ) o << "          v" << D << " = " << a << " == " << b << ";\n";
          if (I.op == D_LT) o << "          v" << D << " = " << a << " < " << b << ";\n";
          o << "          p" << D << " = p; d" << D << " = p && d; live = p && !d;\n";
          break;
        }
        case D_ID:
          o << "          v" << D << " = " << val(I, 0) << "; p" << D << " = on && " << pre(I, 0) << "; d" << D << " = p" << D << " && "
            << ded(I, 0) << "; live = p" << D << " && !d" << D << ";\n";
          break;
        case D_ISLEAF: case D_LEFT: case D_RIGHT: case D_TOKEN:
          o << "          const bool p = on && " << pre(I, 0) << "; bool d = " << ded(I, 0) << "; long long r = 0;\n";
          o << "          if (p && !d) r = sw_tree(x, " << val(I, 0) << ", " << (I.op - D_ISLEAF) << ", d);\n";
          o << "          v" << D << " = r; p" << D << " = p; d" << D << " = p && d; live = p && !d;\n";
          break;
        case D_CE_NODE:
          o << "          const bool p = on && " << pre(I, 0) << " && " << pre(I, 1) << "; bool d = " << ded(I, 0) << " || " << ded(I, 1)
            << ";\n";
          o << "          if (p && !d) sw_ce_node(x, " << val(I, 0) << ", " << val(I, 1) << ", d);\n";
          o << "          v" << D << " = " << val(I, 0) << "; p" << D << " = p; d" << D << " = p && d; live = p && !d;\n";
          break;
        case D_SWITCH: {
          const std::string D1 = std::to_string(I.dst + 1);
          o << "          const bool p = on && " << pre(I, 0) << " && " << pre(I, 1) << "; const bool d = " << ded(I, 0) << " || "
            << ded(I, 1) << "; const bool t = " << val(I, 0) << " != 0;\n";
          o << "          v" << D << " = " << val(I, 1) << "; p" << D << " = p; d" << D << " = p && (d || !t);\n";
          o << "          v" << D1 << " = " << val(I, 1) << "; p" << D1 << " = p; d" << D1 << " = p && (d || t);\n";
          o << "          live = p && !d;\n";
          break;
        }
        case D_MERGE: {
          o << "          bool any_live = false, all_p = true; long long r = 0;\n";
          for (int k = 0; k < 4; ++k) {
            if (I.src[k] == SRC_NONE) continue;
            o << "          if (" << pre(I, k) << " && !" << ded(I, k) << " && !any_live) { any_live = true; r = " << val(I, k) << "; }\n";
            o << "          all_p = all_p && " << pre(I, k) << ";\n";
          }
          o << "          const bool p = on && (any_live || all_p);\n";
          o << "          v" << D << " = r; p" << D << " = p; d" << D << " = p && !any_live; live = on && any_live;\n";
          break;
        }
        case D_CALL:
          o << "          sw_emit(x, on && " << pre(I, 0) << " && !" << ded(I, 0) << " && !(x.fired & " << bit << "), "
            << (0x80000000u | I.aux | ((uint32_t)I.aux2 << 8)) << "u, " << val(I, 0) << ");\n";
          o << "          live = on && " << pre(I, 0) << " && !" << ded(I, 0) << ";\n";
          break;
        case D_NEXT:
          o << "          sw_emit(x, on && " << pre(I, 0) << " && !" << ded(I, 0) << " && !(x.fired & " << bit << "), "
            << (0xC0000000u | ((uint32_t)I.aux2 << 8)) << "u, " << val(I, 0) << ");\n";
          o << "          live = on && " << pre(I, 0) << " && !" << ded(I, 0) << ";\n";
          break;
        case D_OUT:
          o << "          const bool go = on && " << pre(I, 0) << " && !" << ded(I, 0) << " && !(x.fired & " << bit << ");\n";
          if (f == P.result_fn) o << "          sw_result(x, go, " << (int)I.aux << ", " << val(I, 0) << ");\n";
          else o << "          sw_emit(x, go, 0u, " << val(I, 0) << ");\n";
          o << "          live = on && " << pre(I, 0) << " && !" << ded(I, 0) << ";\n";
          break;
        case D_EMBED:
          o << "          sw_embed(x, on, " << (int)I.aux << ", x.sv[" << (int)I.aux << "], " << pre(I, 0) << ", " << ded(I, 0) << ", "
            << val(I, 0) << ", v" << D << ", p" << D << ", live);\n";
          break;
        case D_CELL:
          o << "          sw_cell(x, on, " << (int)I.aux << ", x.sv[" << (int)I.aux << "], " << pre(I, 0) << ", " << ded(I, 0) << ", "
            << val(I, 0) << ", " << pre(I, 1) << ", " << ded(I, 1) << ", " << val(I, 1) << ", v" << D << ", p" << D << ", live);\n";
          break;
        case D_HEAD:
          o << "          sw_head(x, on, " << (int)I.aux << ", " << pre(I, 0) << ", " << ded(I, 0) << ", " << val(I, 0) << ", " << pre(I, 1)
            << ", " << ded(I, 1) << ", " << val(I, 1) << ", v" << D << ", p" << D << ", live);\n";
          break;
        default: break;
      }
      o << "          if (live) x.fired |= " << bit << ";\n";
      o << "        }\n";
    }
    o << "        if (on) x.complete = all_in;\n";
    o << "      }\n    }\n";
  }

  std::string source() {
    o << "#include \"step_device.h\"\n";
    o << "namespace tdf {\n";
    o << "struct GeneratedSweep {\n";
    o << "  static constexpr bool kLdsValues = false;\n";
    o << "  static __device__ void run(LaneCtx& x, const DevProgram& P) {\n";
    o << "    (void)P;\n";
    for (int f = 0; f < P.n_fn; ++f) function(f);
    o << "  }\n};\n}  // namespace tdf\n";
    o << "extern \"C\" __global__ void __launch_bounds__(256) tdf_generated_step(tdf::Engine e, int max_steps, long long spin_ticks) {\n";
    o << "  extern __shared__ __attribute__((aligned(16))) char lds[];\n";
    o << "  __shared__ tdf::DevProgram P;\n  __shared__ uint32_t sh[4];\n";
    o << "  tdf::steps_grid<false, tdf::GeneratedSweep>(e, max_steps, spin_ticks, lds, &P, sh);\n}\n";
    o << "extern \"C\" __global__ void __launch_bounds__(tdf::GEN_LOCAL_BLOCK) tdf_generated_step_local(tdf::Engine e, int max_steps, long long spin_ticks) {\n";
    o << "  extern __shared__ __attribute__((aligned(16))) char lds[];\n";
    o << "  __shared__ tdf::DevProgram P;\n  __shared__ uint32_t sh[4];\n";
    o << "  tdf::steps_grid<true, tdf::GeneratedSweep>(e, max_steps, spin_ticks, lds, &P, sh);\n}\n";
    o << "extern \"C\" __global__ void __launch_bounds__(tdf::GEN_SMALL_BLOCK) tdf_generated_small(tdf::Engine e, int max_steps) {\n";
    o << "  extern __shared__ __attribute__((aligned(16))) char lds[];\n";
    o << "  __shared__ tdf::DevProgram P;\n  __shared__ tdf::Ctrl lc;\n";
    o << "  tdf::steps_small<tdf::GeneratedSweep>(e, max_steps, lds, &P, &lc);\n}\n";
    return o.str();
  }
};

// compiled code objects by firing-table contents: graphs with equal programs share the compile
struct CacheEntry {
  std::vector<char> code;
};
std::mutex g_cache_mutex;
std::map<std::string, CacheEntry> g_cache;

}  // namespace

// Code object of the generated kernels for `arch`, compiled once per (arch, firing tables).
static bool jit_code(const DevProgram& P, const std::string& arch, std::vector<char>& code, std::string& log) {
  for (int f = 0; f < P.n_fn; ++f)
    if (P.fn[f].n_stored > 8) {
      log = "a function keeps more than 8 stored values";
      return false;
    }
  const std::string key = arch + '\n' + std::string(reinterpret_cast<const char*>(&P), sizeof(DevProgram));
  {
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    auto it = g_cache.find(key);
    if (it != g_cache.end()) {
      code = it->second.code;
      return true;
    }
  }
  Rtc& r = rtc();
  if (!r.ok) {
    log = "hiprtc is not available";
    return false;
  }
  Gen gen(P);
  const std::string src = gen.source();
  if (getenv("TDF_JIT_DUMP")) fprintf(stderr, "%s\n", src.c_str());
  rtcProgram prog = nullptr;
  if (r.create(&prog, src.c_str(), "tdf_generated.hip", kEmbeddedCount, kEmbeddedSources, kEmbeddedNames) != 0) {
    log = "hiprtcCreateProgram failed";
    return false;
  }
  const std::string arch_opt = "--offload-arch=" + arch;
  const char* opts[] = {arch_opt.c_str(), "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  const int rc = r.compile(prog, 7, opts);
  size_t ls = 0;
  r.log_size(prog, &ls);
  if (ls > 1) {
    log.resize(ls);
    r.log(prog, &log[0]);
  }
  if (rc != 0) {
    r.destroy(&prog);
    return false;
  }
  size_t cs = 0;
  r.code_size(prog, &cs);
  code.resize(cs);
  r.code(prog, code.data());
  r.destroy(&prog);
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  g_cache[key].code = code;
  return true;
}

bool jit_compile(const DevProgram& P, JitKernels& out, std::string& log) {
  const char* off = getenv("TDF_NO_JIT");
  if (off && off[0] == '1') {
    log = "disabled by TDF_NO_JIT";
    return false;
  }
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    log = "no device";
    return false;
  }
  std::vector<char> code;
  if (!jit_code(P, prop.gcnArchName, code, log)) return false;   // e.g. gfx950:sramecc+:xnack-
  hipModule_t mod = nullptr;
  if (hipModuleLoadData(&mod, code.data()) != hipSuccess) {
    log = "hipModuleLoadData failed";
    return false;
  }
  hipFunction_t f_step = nullptr, f_small = nullptr, f_local = nullptr;
  if (hipModuleGetFunction(&f_step, mod, "tdf_generated_step") != hipSuccess ||
      hipModuleGetFunction(&f_local, mod, "tdf_generated_step_local") != hipSuccess ||
      hipModuleGetFunction(&f_small, mod, "tdf_generated_small") != hipSuccess) {
    (void)hipModuleUnload(mod);
    log = "generated kernels not found in the module";
    return false;
  }
  out.module = mod;
  out.step = f_step;
  out.step_local = f_local;
  out.small = f_small;
  return true;
}

void jit_release(JitKernels& k) {
  if (k.module) (void)hipModuleUnload((hipModule_t)k.module);
  k = JitKernels{};
}

}  // namespace tdf

extern "C" tdf_status tdf_graph_precompile(const tdf_graph* graph, const char* arch, size_t* code_bytes) {
  if (!graph || !arch || !arch[0]) {
    tdf::set_error("tdf_graph_precompile: graph and arch are required");
    return TDF_ERR_BAD_ARG;
  }
  std::vector<char> code;
  std::string log;
  if (!tdf::jit_code(graph->g.prog, arch, code, log)) {
    tdf::set_error("run-time compilation failed: " + log);
    return TDF_ERR_UNSUPPORTED;
  }
  if (code_bytes) *code_bytes = code.size();
  return TDF_OK;
}
