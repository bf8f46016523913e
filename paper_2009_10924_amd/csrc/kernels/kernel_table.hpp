// Per-family lookup of the compiled kernel variant for a (kernel id, parameter block).
#pragma once
#include "launch.hpp"

namespace fs {
const void* unfused_kernel_symbol(int32_t kernel, const KernelArgs& a);
const void* softmax_kernel_symbol(int32_t kernel, const KernelArgs& a);
const void* layernorm_kernel_symbol(int32_t kernel, const KernelArgs& a);
const void* gelu_kernel_symbol(int32_t kernel, const KernelArgs& a);
const void* tchain_kernel_symbol(int32_t kernel, const KernelArgs& a);
const void* rowops_kernel_symbol(int32_t kernel, const KernelArgs& a);
const void* rowprog_kernel_symbol(int32_t kernel, const KernelArgs& a);
}  // namespace fs
