// Run-time side of the generated kernels: compiles HIP source for gfx950 with the HIP
// run-time compiler (loaded with dlopen, so the library still loads where it is absent and
// the generic path then stays with the interpreter), keeps the code objects in a
// process-wide cache keyed by the source, loads a code object as a module on the device it
// is first launched on, and launches it.  Host code only.
#include <dlfcn.h>
#include <unistd.h>
#include <hip/hip_runtime.h>
#include <hip/hiprtc.h>

#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>

#include "launch.hpp"

namespace fs {

namespace {

constexpr int kMaxDevices = 16;

struct Rtc {
  void* lib = nullptr;
  hiprtcResult (*create)(hiprtcProgram*, const char*, const char*, int, const char* const*, const char* const*) = nullptr;
  hiprtcResult (*compile)(hiprtcProgram, int, const char* const*) = nullptr;
  hiprtcResult (*log_size)(hiprtcProgram, size_t*) = nullptr;
  hiprtcResult (*log)(hiprtcProgram, char*) = nullptr;
  hiprtcResult (*code_size)(hiprtcProgram, size_t*) = nullptr;
  hiprtcResult (*code)(hiprtcProgram, char*) = nullptr;
  hiprtcResult (*destroy)(hiprtcProgram*) = nullptr;
  const char* (*error_string)(hiprtcResult) = nullptr;
  bool ok = false;
};

const Rtc& rtc() {
  static const Rtc r = [] {
    Rtc t;
    // the copy the process already holds (PyTorch ships one beside its HIP runtime) wins over the system's
    const char* names[] = {"libhiprtc.so.7", "libhiprtc.so", "/opt/rocm/lib/libhiprtc.so"};
    for (const char* n : names)
      if (!t.lib) t.lib = dlopen(n, RTLD_NOW | RTLD_NOLOAD);
    for (const char* n : names)
      if (!t.lib) t.lib = dlopen(n, RTLD_NOW | RTLD_LOCAL);
    if (!t.lib) return t;
    auto sym = [&](const char* name) { return dlsym(t.lib, name); };
    t.create = reinterpret_cast<decltype(t.create)>(sym("hiprtcCreateProgram"));
    t.compile = reinterpret_cast<decltype(t.compile)>(sym("hiprtcCompileProgram"));
    t.log_size = reinterpret_cast<decltype(t.log_size)>(sym("hiprtcGetProgramLogSize"));
    t.log = reinterpret_cast<decltype(t.log)>(sym("hiprtcGetProgramLog"));
    t.code_size = reinterpret_cast<decltype(t.code_size)>(sym("hiprtcGetCodeSize"));
    t.code = reinterpret_cast<decltype(t.code)>(sym("hiprtcGetCode"));
    t.destroy = reinterpret_cast<decltype(t.destroy)>(sym("hiprtcDestroyProgram"));
    t.error_string = reinterpret_cast<decltype(t.error_string)>(sym("hiprtcGetErrorString"));
    t.ok = t.create && t.compile && t.log_size && t.log && t.code_size && t.code && t.destroy && t.error_string;
    return t;
  }();
  return r;
}

// Value of an unsigned integer entry `key` of the kernel's metadata note (MessagePack, as the
// AMDGPU code-object format defines it): the key's bytes are searched for and the integer that
// follows is decoded.  -1 if absent.
int64_t metadata_uint(const std::string& code, const char* key) {
  const size_t klen = strlen(key);
  size_t at = 0;
  while ((at = code.find(key, at)) != std::string::npos) {
    const size_t v = at + klen;
    if (at == 0 || v >= code.size()) return -1;
    // the key must be a MessagePack string of exactly this length (fixstr 0xa0|len or str8 0xd9 len)
    const unsigned char before = (unsigned char)code[at - 1];
    const bool fixstr = klen < 32 && before == (0xa0u | klen);
    const bool str8 = at >= 2 && (unsigned char)code[at - 2] == 0xd9 && before == klen;
    if (fixstr || str8) {
      const unsigned char t = (unsigned char)code[v];
      auto be = [&](int n) -> int64_t {
        if (v + 1 + n > code.size()) return -1;
        int64_t x = 0;
        for (int i = 0; i < n; ++i) x = (x << 8) | (unsigned char)code[v + 1 + i];
        return x;
      };
      if (t <= 0x7f) return t;
      if (t == 0xcc) return be(1);
      if (t == 0xcd) return be(2);
      if (t == 0xce) return be(4);
      if (t == 0xcf) return be(8);
    }
    at = v;
  }
  return -1;
}

std::mutex& big_lock() {
  static std::mutex m;
  return m;
}

// Optional on-disk cache of code objects, for processes that start often: FS_CODEGEN_CACHE_DIR names a directory
// (it must exist); a file there is named by a 64-bit hash of the source and holds the source's length, the source
// and the code object, so a hash collision or a damaged file reads as a miss.  Unset: nothing is read or written.
uint64_t fnv1a64(const std::string& text) {
  uint64_t h = 1469598103934665603ull;
  for (unsigned char ch : text) h = (h ^ ch) * 1099511628211ull;
  return h;
}
std::string cache_path(const std::string& source) {
  const char* dir = getenv("FS_CODEGEN_CACHE_DIR");
  if (!dir || !dir[0]) return std::string();
  char name[64];
  // the compiler settings are part of the key (the source alone would survive a change of them)
  snprintf(name, sizeof name, "/fs_gfx950_%016llx.co", (unsigned long long)fnv1a64("gfx950|O3|c++17|no-packed-fp32|" + source));
  return std::string(dir) + name;
}
bool cache_read(const std::string& source, std::string* code) {
  const std::string path = cache_path(source);
  if (path.empty()) return false;
  FILE* f = fopen(path.c_str(), "rb");
  if (!f) return false;
  bool ok = false;
  uint64_t n_source = 0, n_code = 0;
  if (fread(&n_source, 8, 1, f) == 1 && fread(&n_code, 8, 1, f) == 1 && n_source == source.size() && n_code > 0 && n_code < (1ull << 28)) {
    std::string stored(n_source, '\0');
    code->assign(n_code, '\0');
    ok = fread(&stored[0], 1, n_source, f) == n_source && stored == source && fread(&(*code)[0], 1, n_code, f) == n_code;
  }
  fclose(f);
  return ok;
}
void cache_write(const std::string& source, const std::string& code) {
  const std::string path = cache_path(source);
  if (path.empty()) return;
  const std::string tmp = path + ".tmp" + std::to_string((long)getpid());
  FILE* f = fopen(tmp.c_str(), "wb");
  if (!f) return;
  const uint64_t n_source = source.size(), n_code = code.size();
  const bool ok = fwrite(&n_source, 8, 1, f) == 1 && fwrite(&n_code, 8, 1, f) == 1 && fwrite(source.data(), 1, n_source, f) == n_source &&
                  fwrite(code.data(), 1, n_code, f) == n_code;
  fclose(f);
  if (!ok || rename(tmp.c_str(), path.c_str()) != 0) remove(tmp.c_str());   // complete files only, whoever wins the race
}

}  // namespace

struct GenKernel {
  std::string entry;
  std::string code;                      // the code object
  int32_t vgprs = 0, static_lds = 0, scratch_bytes = 0, spilled_vgprs = 0;
  std::atomic<hipFunction_t> fn[kMaxDevices];
  GenKernel() {
    for (auto& f : fn) f.store(nullptr, std::memory_order_relaxed);
  }
};

namespace {

std::map<std::string, std::shared_ptr<GenKernel>>& cache() {
  static std::map<std::string, std::shared_ptr<GenKernel>> c;
  return c;
}

// the function on the current device; the module is loaded on first use there and stays loaded
int function_here(GenKernel* k, hipFunction_t* out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  hipFunction_t f = k->fn[dev].load(std::memory_order_acquire);
  if (!f) {
    std::lock_guard<std::mutex> guard(big_lock());
    f = k->fn[dev].load(std::memory_order_acquire);
    if (!f) {
      hipModule_t mod = nullptr;
      e = hipModuleLoadData(&mod, k->code.data());
      if (e != hipSuccess) return (int)e;
      e = hipModuleGetFunction(&f, mod, k->entry.c_str());
      if (e != hipSuccess) return (int)e;
      k->fn[dev].store(f, std::memory_order_release);
    }
  }
  *out = f;
  return 0;
}

}  // namespace

bool gen_available() { return rtc().ok; }

int gen_compile(const std::string& source, const char* entry, std::shared_ptr<GenKernel>* out, std::string* log) {
  const Rtc& r = rtc();
  if (!r.ok) {
    if (log) *log = "the HIP run-time compiler (libhiprtc) could not be loaded";
    return (int)hipErrorNotSupported;
  }
  if (const char* inject = getenv("FS_CODEGEN_INJECT_FAILURE"); inject && inject[0] == '1') {
    // for tests of the fall-back paths: behave as if the compiler had rejected the source
    if (log) *log = "compilation failure injected by FS_CODEGEN_INJECT_FAILURE";
    return (int)hipErrorUnknown;
  }
  std::lock_guard<std::mutex> guard(big_lock());
  auto it = cache().find(source);
  if (it != cache().end()) {
    *out = it->second;
    return 0;
  }
  auto finish = [&](const std::shared_ptr<GenKernel>& k) {
    const int64_t vg = metadata_uint(k->code, ".vgpr_count"), lds = metadata_uint(k->code, ".group_segment_fixed_size"),
                  scratch = metadata_uint(k->code, ".private_segment_fixed_size"), spill = metadata_uint(k->code, ".vgpr_spill_count");
    k->vgprs = vg > 0 ? (int32_t)vg : 0;
    k->static_lds = lds > 0 ? (int32_t)lds : 0;
    k->scratch_bytes = scratch > 0 ? (int32_t)scratch : 0;
    k->spilled_vgprs = spill > 0 ? (int32_t)spill : 0;
    cache()[source] = k;
    *out = k;
  };
  {
    auto k = std::make_shared<GenKernel>();
    k->entry = entry;
    if (cache_read(source, &k->code)) {
      finish(k);
      return 0;
    }
  }
  hiprtcProgram prog = nullptr;
  hiprtcResult rc = r.create(&prog, source.c_str(), "fs_generated.hip", 0, nullptr, nullptr);
  if (rc != HIPRTC_SUCCESS) {
    if (log) *log = r.error_string(rc);
    return (int)hipErrorUnknown;
  }
  // same code generation settings as the library's own kernels; packed-fp32 VALU ops stay off
  const char* opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
  rc = r.compile(prog, (int)(sizeof opts / sizeof opts[0]), opts);
  if (log) {
    size_t n = 0;
    if (r.log_size(prog, &n) == HIPRTC_SUCCESS && n > 1) {
      log->assign(n, '\0');
      r.log(prog, &(*log)[0]);
      while (!log->empty() && log->back() == '\0') log->pop_back();
    }
    if (rc != HIPRTC_SUCCESS && log->empty()) *log = r.error_string(rc);
  }
  if (rc != HIPRTC_SUCCESS) {
    r.destroy(&prog);
    return (int)hipErrorUnknown;
  }
  auto k = std::make_shared<GenKernel>();
  k->entry = entry;
  size_t n = 0;
  rc = r.code_size(prog, &n);
  if (rc == HIPRTC_SUCCESS) {
    k->code.assign(n, '\0');
    rc = r.code(prog, &k->code[0]);
  }
  r.destroy(&prog);
  if (rc != HIPRTC_SUCCESS || k->code.empty()) {
    if (log) *log = "the run-time compiler returned no code object";
    return (int)hipErrorUnknown;
  }
  cache_write(source, k->code);
  finish(k);
  return 0;
}

GenResources gen_resources(const GenKernel* k) {
  GenResources r;
  r.vgprs = k->vgprs;
  r.static_lds = k->static_lds;
  r.scratch_bytes = k->scratch_bytes;
  r.spilled_vgprs = k->spilled_vgprs;
  r.code_bytes = (int64_t)k->code.size();
  return r;
}

int gen_preload(GenKernel* k) {
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) {
    (void)hipGetLastError();   // no device here: the module is loaded by the first launch
    return 0;
  }
  hipFunction_t f;
  return function_here(k, &f);
}

int gen_launch(GenKernel* k, const void* args, size_t args_bytes, const LaunchShape& s, void* stream) {
  hipFunction_t f = nullptr;
  const int e = function_here(k, &f);
  if (e != 0) return e;
  void* config[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, const_cast<void*>(args), HIP_LAUNCH_PARAM_BUFFER_SIZE, &args_bytes, HIP_LAUNCH_PARAM_END};
  return (int)hipModuleLaunchKernel(f, s.grid[0], s.grid[1], s.grid[2], s.block[0], s.block[1], s.block[2], s.lds_bytes,
                                    static_cast<hipStream_t>(stream), nullptr, config);
}

}  // namespace fs
