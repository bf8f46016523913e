// Kernel dispatch: every kernel takes its device pointers first and its parameter
// block (by value) last, so one launcher serves all families.
#include <hip/hip_runtime.h>

#include "kernel_table.hpp"

namespace fs {

namespace {
struct KernelDesc {
  const char* name;
  int n_ptrs;
};
const KernelDesc kDesc[K_COUNT] = {
    {"unary", 2},          {"binary", 3},          {"reduce_row", 2},     {"reduce_mid", 2},
    {"transpose_rows", 2}, {"transpose_tile", 2},  {"copy", 2},           {"softmax_wave", 3},
    {"softmax_block", 3},  {"layernorm_wave", 8},  {"layernorm_block", 8}, {"bias_gelu", 3},
    {"bias_gelu_dbias", 5}, {"colfold", 3},        {"tchain_wave", 3},    {"tchain_lds", 3},
    {"row_wave", 6},       {"row_block", 6},       {"row_program", 0},    {"layernorm_bwd", 7},
    {"row_generated", 0},
};

const void* symbol_for(int32_t kernel, const KernelArgs& a) {
  switch (kernel) {
    case K_UNARY: case K_BINARY: case K_REDUCE_ROW: case K_REDUCE_MID:
    case K_TRANSPOSE_ROWS: case K_TRANSPOSE_TILE: case K_COPY:
      return unfused_kernel_symbol(kernel, a);
    case K_SOFTMAX_WAVE: case K_SOFTMAX_BLOCK:
      return softmax_kernel_symbol(kernel, a);
    case K_LAYERNORM_WAVE: case K_LAYERNORM_BLOCK: case K_LAYERNORM_BWD:
      return layernorm_kernel_symbol(kernel, a);
    case K_BIAS_GELU: case K_BIAS_GELU_DBIAS: case K_COLFOLD:
      return gelu_kernel_symbol(kernel, a);
    case K_TCHAIN_WAVE: case K_TCHAIN_LDS:
      return tchain_kernel_symbol(kernel, a);
    case K_ROW_WAVE: case K_ROW_BLOCK:
      return rowops_kernel_symbol(kernel, a);
    case K_ROW_PROGRAM:
      return rowprog_kernel_symbol(kernel, a);
    default:
      return nullptr;
  }
}
}  // namespace

const char* kernel_name(int32_t kernel) {
  return (kernel >= 0 && kernel < K_COUNT) ? kDesc[kernel].name : "?";
}

const char* hip_error_text(int err) { return hipGetErrorString(static_cast<hipError_t>(err)); }

int launch_kernel(int32_t kernel, const KernelArgs& args, const LaunchShape& s, void* stream) {
  if (kernel < 0 || kernel >= K_COUNT) return (int)hipErrorInvalidValue;
  const void* sym = symbol_for(kernel, args);
  if (!sym) return (int)hipErrorInvalidDeviceFunction;
  if (kernel == K_ROW_PROGRAM) {
    // one by-value argument: pointers by class, then the program
    ProgArgs pa;
    for (int i = 0; i < kProgMaxOperands; ++i) {
      pa.full[i] = args.p[kSlotFull + i];
      pa.col[i] = args.p[kSlotCol + i];
      pa.rscal[i] = args.p[kSlotRscal + i];
      pa.out[i] = args.p[kSlotOut + i];
      pa.rout[i] = args.p[kSlotRout + i];
    }
    pa.p = args.u.prog;
    if (s.lds_bytes > 64u * 1024u) {
      // more dynamic LDS than the default cap: the limit is a per-kernel attribute
      if (s.lds_bytes > (uint32_t)kProgMaxLdsBytes) return (int)hipErrorInvalidValue;
      const hipError_t e = hipFuncSetAttribute(sym, hipFuncAttributeMaxDynamicSharedMemorySize, (int)s.lds_bytes);
      if (e != hipSuccess) return (int)e;
    }
    void* one[1] = {&pa};
    return (int)hipLaunchKernel(sym, dim3(s.grid[0], s.grid[1], s.grid[2]), dim3(s.block[0], s.block[1], s.block[2]),
                                one, s.lds_bytes, static_cast<hipStream_t>(stream));
  }
  KernelArgs a = args;   // hipLaunchKernel wants addresses of mutable argument storage
  void* argv[kMaxPtrs + 1];
  const int n = kDesc[kernel].n_ptrs;
  for (int i = 0; i < n; ++i) argv[i] = &a.p[i];
  argv[n] = &a.u;        // every member of the union starts at the union's address
  return (int)hipLaunchKernel(sym, dim3(s.grid[0], s.grid[1], s.grid[2]), dim3(s.block[0], s.block[1], s.block[2]),
                              argv, s.lds_bytes, static_cast<hipStream_t>(stream));
}

KernelResources kernel_resources(int32_t kernel, const KernelArgs& args) {
  KernelResources r;
  const void* sym = (kernel >= 0 && kernel < K_COUNT) ? symbol_for(kernel, args) : nullptr;
  if (!sym) return r;
  hipFuncAttributes attr;
  if (hipFuncGetAttributes(&attr, sym) == hipSuccess) {
    r.vgprs = attr.numRegs;
    r.static_lds = (int32_t)attr.sharedSizeBytes;
    r.from_device = true;
  } else {
    (void)hipGetLastError();   // no device: the caller falls back to its own estimate
  }
  return r;
}

}  // namespace fs
