// Tile kernels compiled for one plan at run time (plan option compile=1).
//
// Section 4 of the paper builds, once per layer and before training starts, a meta-kernel that
// runs the layer's operators one after the other, and compiles it at run time.  Here the
// template is the tile kernel itself (fbx_tile.hip): the same source is compiled again with the
// numbers that the plan and the tile size fix written in as literals, which is worth several per
// cent of its time.  The compiler is the HIP run-time compilation library, loaded when first
// needed; whatever goes wrong (no library, no sources beside this library, a compile error)
// leaves the call on the generic kernel and says why in the call's note.
#include <dlfcn.h>
#include <dirent.h>

#include <algorithm>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <sstream>

#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>

#include "fbx_device.h"

namespace fbx {

namespace {

struct Rtc {
  void* lib = nullptr;
  hiprtcResult (*create)(hiprtcProgram*, const char*, const char*, int, const char**, const char**) = nullptr;
  hiprtcResult (*compile)(hiprtcProgram, int, const char**) = nullptr;
  hiprtcResult (*log_size)(hiprtcProgram, size_t*) = nullptr;
  hiprtcResult (*log)(hiprtcProgram, char*) = nullptr;
  hiprtcResult (*code_size)(hiprtcProgram, size_t*) = nullptr;
  hiprtcResult (*code)(hiprtcProgram, char*) = nullptr;
  hiprtcResult (*destroy)(hiprtcProgram*) = nullptr;
  std::string why;  // why it is not usable
  bool ok = false;
};

const Rtc& rtc() {
  static Rtc r;
  static std::once_flag once;
  std::call_once(once, [] {
    for (const char* name : {"libhiprtc.so", "libhiprtc.so.7", "/opt/rocm/lib/libhiprtc.so"}) {
      r.lib = dlopen(name, RTLD_NOW | RTLD_LOCAL);
      if (r.lib) break;
    }
    if (!r.lib) { r.why = "the run-time compilation library could not be loaded"; return; }
    auto sym = [&](const char* n) { return dlsym(r.lib, n); };
    r.create = reinterpret_cast<decltype(r.create)>(sym("hiprtcCreateProgram"));
    r.compile = reinterpret_cast<decltype(r.compile)>(sym("hiprtcCompileProgram"));
    r.log_size = reinterpret_cast<decltype(r.log_size)>(sym("hiprtcGetProgramLogSize"));
    r.log = reinterpret_cast<decltype(r.log)>(sym("hiprtcGetProgramLog"));
    r.code_size = reinterpret_cast<decltype(r.code_size)>(sym("hiprtcGetCodeSize"));
    r.code = reinterpret_cast<decltype(r.code)>(sym("hiprtcGetCode"));
    r.destroy = reinterpret_cast<decltype(r.destroy)>(sym("hiprtcDestroyProgram"));
    r.ok = r.create && r.compile && r.log_size && r.log && r.code_size && r.code && r.destroy;
    if (!r.ok) r.why = "the run-time compilation library lacks an entry point";
  });
  return r;
}

bool readable(const std::string& path) {
  FILE* f = fopen(path.c_str(), "rb");
  if (f) fclose(f);
  return f != nullptr;
}

// The kernel sources lie beside this library (csrc/, ../include/) unless the environment
// variable FBX_KERNEL_SOURCES names the directory that holds csrc/ and include/; the compiler's
// own headers lie under the ROCm tree.
struct Paths {
  std::string csrc, include, rocm_include, clang_include, why;
  bool ok = false;
};

const Paths& paths() {
  static Paths p;
  static std::once_flag once;
  std::call_once(once, [] {
    Dl_info info;
    if (!dladdr(reinterpret_cast<const void*>(&paths), &info) || !info.dli_fname) { p.why = "this library's own path is unknown"; return; }
    std::string dir(info.dli_fname);
    const size_t slash = dir.rfind('/');
    dir = slash == std::string::npos ? std::string(".") : dir.substr(0, slash);
    p.csrc = dir + "/csrc";
    p.include = dir + "/../include";
    if (const char* moved = getenv("FBX_KERNEL_SOURCES")) {  // a library installed away from its sources: <dir>/csrc, <dir>/include
      if (*moved) { p.csrc = std::string(moved) + "/csrc"; p.include = std::string(moved) + "/include"; }
    }
    if (!readable(p.csrc + "/fbx_tile.hip") || !readable(p.include + "/fbx.h")) { p.why = "the kernel sources are not beside the library"; return; }
    const char* env = getenv("ROCM_PATH");
    const std::string rocm = env && *env ? env : "/opt/rocm";
    p.rocm_include = rocm + "/include";
    const std::string clang = rocm + "/lib/llvm/lib/clang";
    if (DIR* d = opendir(clang.c_str())) {
      while (dirent* e = readdir(d)) {
        if (e->d_name[0] == '.') continue;
        const std::string cand = clang + "/" + e->d_name + "/include";
        if (readable(cand + "/stddef.h")) p.clang_include = cand;
      }
      closedir(d);
    }
    if (p.clang_include.empty()) { p.why = "the compiler's headers were not found under " + rocm; return; }
    p.ok = true;
  });
  return p;
}

#define FBX_FIELD_VALUE(name) v.push_back(P.name);
std::vector<uint32_t> fixed_values(const TileParams& P) {
  std::vector<uint32_t> v;
  FBX_TILE_FIXED_FIELDS(FBX_FIELD_VALUE)
  return v;
}
#undef FBX_FIELD_VALUE

#define FBX_FIELD_ASSIGN(name) os << " P." #name " = " << P.name << "u;";
void braces(std::ostringstream& os, const uint32_t* v, size_t n) {
  os << "{";
  for (size_t i = 0; i < n; ++i) os << (i ? ", " : "") << v[i] << "u";
  os << "}";
}

std::string program_text(const TileParams& P, int mode, const PlanHost& h, uint32_t threads, uint32_t lane_ops) {
  std::ostringstream os;
  os << "#define FBX_TILE_THREADS " << threads << "\n";
  // (tuning: the environment variable FBX_EXP defines the macro of that name for the compiled kernel, so that
  // two variants of a piece of kernel code, written under #if FBX_EXP & <bit>, can be timed in one process
  // environment after the other on the same device; no committed code path depends on it)
  if (const char* x = getenv("FBX_EXP")) os << "#define FBX_EXP " << atoi(x) << "\n";
  os << "#define FBX_FIXED_MODE " << mode << "\n#define FBX_FIXED_NAME fbx_tile_fixed_" << mode << "\n#define FBX_FIXED_ASSIGN";
  FBX_TILE_FIXED_FIELDS(FBX_FIELD_ASSIGN)
  // wavefronts per SIMD the kernel must leave registers for: as many workgroups as the LDS admits
  const uint32_t groups = std::max(1u, std::min(4u, tile_max_lds() / std::max(P.lds_bytes, 1u)));
  os << "\n#define FBX_FIXED_WAVES " << std::max(4u, groups * (threads / 64u) / 4u);
  os << "\n#define FBX_FIXED_LIST_BEGIN ";
  braces(os, h.tile_list_begin.data(), h.tile_list_begin.size());
  // (the table of derived counts starts with the first entry of every layer, padded to four words)
  const uint32_t none = 0;
  const size_t head = h.derive_tab.empty() ? 0 : 4u * ((h.n_layers + 3u) / 4u);
  os << "\n#define FBX_FIXED_RNR_HEAD ";
  braces(os, head ? h.derive_tab.data() : &none, head ? head : 1);
  if (P.log2T != 6u) lane_ops = 0;
  os << "\n#define FBX_LANE_OPS " << lane_ops;
  if (lane_ops == 2u) {
    // Tiles of 64 records: a wavefront runs one single-sign operator at a time, one record per lane.
    // Those operators become straight-line code with their numbers written in, one case each:
    // single-valued buckets and hashes of layer 1 (in the order of their work lists: a unit of
    // work is an operator), and per later layer the crosses of two single signs.
    auto hex = [&](uint64_t v) { os << "0x" << std::hex << v << std::dec << "ull"; };
    uint32_t u = 0;
    os << "\n#define FBX_GEN_L1";
    for (uint32_t list : {(uint32_t)TL_BUCKET1, (uint32_t)TL_HASH1}) {
      for (uint32_t i = h.tile_list_begin[list]; i < h.tile_list_begin[list + 1]; ++i, ++u) {
        const uint32_t op = h.tile_lists[i];
        const OpDesc& d = h.ops[op].d;
        os << " case " << u << "u: ";
        if (list == TL_BUCKET1) {
          os << "lane_bucket1(" << d.field << "u, here(";
          hex(d.key);
          os << "), " << d.aux_off << "u, " << d.aux_len << "u, values_of(" << op << "u), " << d.stage << "u); break;";
        } else {
          os << "lane_hash1(" << d.field << "u, here(";
          hex(d.key);
          os << "), values_of(" << op << "u), " << d.stage << "u); break;";
        }
      }
    }
    os << "\n#define FBX_GEN_X11";
    for (uint32_t layer = 2; layer <= h.n_layers; ++layer) {
      const uint32_t list = TL_LAYER + 2u * (layer - 2u);
      os << " case " << layer << "u: switch (u) {";
      u = 0;
      for (uint32_t i = h.tile_list_begin[list]; i < h.tile_list_begin[list + 1]; ++i, ++u) {
        const uint32_t op = h.tile_lists[i];
        const OpDesc& d = h.ops[op].d;
        os << " case " << u << "u: lane_x11(" << h.ops[d.a].d.stage << "u, " << h.ops[d.b].d.stage << "u, here(";
        hex(d.key);
        os << "), values_of(" << op << "u), " << d.stage << "u); break;";
      }
      os << " } break;";
    }
  }
  os << "\n#include \"fbx_tile.hip\"\n";
  return os.str();
}
#undef FBX_FIELD_ASSIGN

}  // namespace

std::string tile_kernel_source(const TileParams& P, int mode, const PlanHost& h, uint32_t threads, uint32_t lane_ops) {
  return program_text(P, mode, h, threads, lane_ops);
}

TileJit::~TileJit() { release(); }

void TileJit::release() {
  for (FixedTileKernel& k : kernels_)
    if (k.module) (void)hipModuleUnload(reinterpret_cast<hipModule_t>(k.module));
  kernels_.clear();
}

const FixedTileKernel* TileJit::get(const TileParams& P, int mode, const PlanHost& h, uint32_t threads, uint32_t lane_ops) {
  std::vector<uint32_t> key = fixed_values(P);
  key.push_back(threads | (lane_ops << 16));
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = 0; }
  key.push_back(static_cast<uint32_t>(dev));  // (a loaded kernel belongs to one device)
  for (const FixedTileKernel& k : kernels_)
    if (k.mode == mode && k.key == key) return k.function ? &k : nullptr;
  if (kernels_.size() >= kMaxKernels) {  // batches of ever new shapes: stop compiling for them
    note_ = "compile=1: more tile shapes than compiled kernels are kept for; the generic kernel runs";
    return nullptr;
  }
  FixedTileKernel k;
  k.mode = mode;
  k.key = key;
  k.threads = threads;
  k.lane_ops = lane_ops;
  auto fail = [&](const std::string& why) -> const FixedTileKernel* {
    note_ = "compile=1: " + why + "; the generic kernel runs";
    kernels_.push_back(k);  // (remembered, so that the attempt is not made again)
    return nullptr;
  };
  const Rtc& r = rtc();
  if (!r.ok) return fail(r.why);
  const Paths& p = paths();
  if (!p.ok) return fail(p.why);
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return fail("the device's architecture is unknown");
  std::string arch(prop.gcnArchName);
  arch = arch.substr(0, arch.find(':'));

  const auto t0 = std::chrono::steady_clock::now();
  const std::string text = program_text(P, mode, h, threads, lane_ops);
  hiprtcProgram prog = nullptr;
  if (r.create(&prog, text.c_str(), "fbx_tile_fixed.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS) return fail("the program could not be created");
  const std::string o_arch = "--offload-arch=" + arch, i0 = "-I" + p.csrc, i1 = "-I" + p.include, i2 = "-I" + p.rocm_include,
                    i3 = "-I" + p.clang_include;
  // the same code generation options as the library's own build
  const char* opts[] = {o_arch.c_str(), "-O3", "-std=c++17", i0.c_str(), i1.c_str(), i2.c_str(), i3.c_str(),
                        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                        "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
#ifdef FBX_TILE_PROF
                        "-DFBX_TILE_PROF",  // (a tuning build of the library compiles tuning kernels)
#endif
  };
  const hiprtcResult rc = r.compile(prog, static_cast<int>(sizeof(opts) / sizeof(opts[0])), opts);
  if (rc != HIPRTC_SUCCESS) {
    size_t n = 0;
    std::string log;
    if (r.log_size(prog, &n) == HIPRTC_SUCCESS && n > 1) {
      log.resize(n);
      (void)r.log(prog, &log[0]);
      if (log.size() > 400) log.resize(400);
    }
    (void)r.destroy(&prog);
    return fail("the kernel did not compile (" + log + ")");
  }
  size_t n = 0;
  std::vector<char> code;
  if (r.code_size(prog, &n) != HIPRTC_SUCCESS || n == 0) { (void)r.destroy(&prog); return fail("the compiler returned no code"); }
  code.resize(n);
  const hiprtcResult got = r.code(prog, code.data());
  (void)r.destroy(&prog);
  if (got != HIPRTC_SUCCESS) return fail("the compiler returned no code");
  hipModule_t module = nullptr;
  hipFunction_t fn = nullptr;
  if (hipModuleLoadData(&module, code.data()) != hipSuccess) { (void)hipGetLastError(); return fail("the compiled code did not load"); }
  const std::string name = "fbx_tile_fixed_" + std::to_string(mode);
  if (hipModuleGetFunction(&fn, module, name.c_str()) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipModuleUnload(module);
    return fail("the compiled code has no kernel");
  }
  int per_cu = 0;
  if (hipModuleOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, (int)threads, P.lds_bytes) != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    per_cu = 1;
  }
  k.module = module;
  k.function = fn;
  k.per_cu = static_cast<uint32_t>(per_cu);
  compile_ms_ += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
  ++compiled_;
  kernels_.push_back(k);
  return &kernels_.back();
}

hipError_t launch_tile_fixed(const FixedTileKernel& k, const TileParams& P, hipStream_t st) {
  if (P.n_tiles == 0) return hipSuccess;
  std::vector<uint32_t> now = fixed_values(P);
  now.push_back(k.threads | (k.lane_ops << 16));
  now.push_back(k.key.back());
  if (now != k.key) return hipErrorInvalidValue;  // (a kernel compiled for other numbers)
  uint32_t capacity = tile_cu_count() * k.per_cu;  // as many workgroups as run at the same time
  if (P.grid && P.grid < capacity) capacity = P.grid;
  TileParams Q = P;
  void* args[] = {&Q};
  const uint32_t grid = std::min(P.n_tiles, capacity);
  return hipModuleLaunchKernel(reinterpret_cast<hipFunction_t>(k.function), grid, 1, 1, k.threads, 1, 1, P.lds_bytes, st, args,
                               nullptr);
}

}  // namespace fbx
