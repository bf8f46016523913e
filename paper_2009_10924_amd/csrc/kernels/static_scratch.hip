// fs_execute_static: fs_execute for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid it).  The plan's scratch -- the
// partial column sums that the workgroups of one launch hand to the fold launch -- lives in a
// fixed array in the library's own device image instead of a caller-provided workspace.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../fs_internal.hpp"

namespace {

// One copy per GPU, loaded with the code object and held until the process ends.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[FS_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU; null = not looked up yet

// Address of this GPU's copy of `scratch`.  The array's name in host code is only a handle for the
// runtime, not a device address: the address comes from hipGetSymbolAddress, once per device with that
// device current, and everything below uses the looked-up pointer.
fs_status scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fs::fail(FS_ERR_HIP, "fs_execute_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fs::fail(FS_ERR_INVALID_ARG, "fs_execute_static: device %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return fs::fail(FS_ERR_HIP, "fs_execute_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FS_OK;
}

}  // namespace

extern "C" fs_status fs_execute_static(const fs_plan* p, const void* const* inputs, void* const* outputs, void* hip_stream) try {
  fs::clear_error();
  const fs_status s = fs::check_execute_args(p, inputs, outputs, "fs_execute_static");
  if (s != FS_OK) return s;
  const fs::Candidate& c = p->candidates[p->chosen];
  if (c.info.workspace_bytes > (int64_t)FS_STATIC_SCRATCH_BYTES)
    return fs::fail(FS_ERR_WORKSPACE, "fs_execute_static: the plan needs %lld bytes of scratch, the static array holds %lld; use fs_execute with a workspace",
                    (long long)c.info.workspace_bytes, (long long)FS_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (c.info.workspace_bytes > 0) {
    const fs_status a = scratch_of_current_device(&ws);
    if (a != FS_OK) return a;
  }
  // Nothing has to start at zero: every kernel that reads the scratch reads what a launch of the same call
  // wrote there before it (the fold reads the partial sums of the launch in front of it).
  return fs::run_launches(p, inputs, outputs, ws, hip_stream, c.launches.size());
} catch (...) {
  return fs::fail_caught("fs_execute_static");
}
