// Kernel packing (paper Section 4.1) across fusion patterns that have no data dependence
// on each other (Section 5.2, remote fusion: patterns that are not adjacent in the graph
// still share one kernel): up to 32 independent row patterns run as ONE launch.  Each
// workgroup finds the member it serves from a table carried in the kernel arguments,
// then runs that member's pattern on the generic row skeleton exactly as a stand-alone
// launch would: a lane group (or the workgroup) owns a row, intermediates stay in
// registers.  Members differ in pattern, dtype, shape and lanes per row; nothing is
// exchanged between members.  What packing removes is the per-launch cost, which
// dominates subgraphs whose own run time is a few microseconds.
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include "row_skeleton.hpp"

namespace fsk {

template <typename Spec, typename T, typename TO, int K>
__device__ __forceinline__ void run_member(const PackEntry& e, float* slots, uint32_t vblock) {
  RowCtx<T, TO, Spec::NI, Spec::NV, K, false, MODE_RUNTIME> c(e.p, slots, vblock);
  const T* in[Spec::NI];
  const T* vec[Spec::NV > 0 ? Spec::NV : 1] = {nullptr};
#pragma unroll
  for (int i = 0; i < Spec::NI; ++i) in[i] = static_cast<const T*>(e.in[i]);
#pragma unroll
  for (int i = 0; i < Spec::NV; ++i) vec[i] = static_cast<const T*>(e.vec[i]);
  c.load(in, vec);
  Spec::run(c, static_cast<TO*>(e.out));
}

template <typename Spec, typename T, typename TO>
__device__ __forceinline__ void run_member_k(const PackEntry& e, float* slots, uint32_t vblock, int k_log2) {
  switch (k_log2) {
    case 0: run_member<Spec, T, TO, 1>(e, slots, vblock); break;
    case 1: run_member<Spec, T, TO, 2>(e, slots, vblock); break;
    default: run_member<Spec, T, TO, 4>(e, slots, vblock); break;
  }
}

template <typename Spec, bool MIXED>
__device__ __forceinline__ void run_member_t(const PackEntry& e, float* slots, uint32_t vblock, int types, int k_log2) {
  switch (types) {
    case PT_F32: run_member_k<Spec, float, float>(e, slots, vblock, k_log2); break;
    case PT_F16: run_member_k<Spec, f16_t, f16_t>(e, slots, vblock, k_log2); break;
    case PT_BF16: run_member_k<Spec, bf16_t, bf16_t>(e, slots, vblock, k_log2); break;
    default:
      if constexpr (MIXED) run_member_k<Spec, float, bf16_t>(e, slots, vblock, k_log2);
      break;
  }
}

// The table is read straight from the kernel-argument segment (constant memory) with
// wave-uniform addresses; indexing the by-value parameter itself would make the compiler
// copy the whole table to per-lane scratch first.
typedef const PackTable __attribute__((address_space(4))) * ConstTable;

__global__ void __launch_bounds__(256) k_pack(const PackTable table_in_kernarg) {
  __shared__ float slots[16];
  ConstTable tab = (ConstTable)__builtin_amdgcn_kernarg_segment_ptr();
  const uint32_t b = blockIdx.x;
  int i = -1;
#pragma unroll
  for (int j = 0; j < kPackMaxMembers; ++j) i += b >= tab->first_block[j] ? 1 : 0;   // first_block[0] = 0
  i = __builtin_amdgcn_readfirstlane(i);
  PackEntry e;
  __builtin_memcpy(&e, &tab->e[i], sizeof(PackEntry));
  const uint32_t vblock = b - tab->first_block[i];
  const int k_log2 = e.variant % 3, types = (e.variant / 3) % PT_COUNT, spec = e.variant / (3 * PT_COUNT);
  switch (spec) {
    case PACK_SOFTMAX: run_member_t<SoftmaxSpec, false>(e, slots, vblock, types, k_log2); break;
    case PACK_SOFTMAX_BWD: run_member_t<SoftmaxBwdSpec, false>(e, slots, vblock, types, k_log2); break;
    case PACK_RMSNORM: run_member_t<RmsNormSpec, false>(e, slots, vblock, types, k_log2); break;
    case PACK_LN_FULL: run_member_t<LayerNormSpec<true>, true>(e, slots, vblock, types, k_log2); break;
    case PACK_LN_PLAIN: run_member_t<LayerNormSpec<false>, true>(e, slots, vblock, types, k_log2); break;
    case PACK_BIAS_GELU: run_member_t<BiasGeluSpec, false>(e, slots, vblock, types, k_log2); break;
    default: break;
  }
}

}  // namespace fsk

namespace fs {

int launch_pack(const PackTable& table, void* stream) {
  if (table.n < 1 || table.n > kPackMaxMembers || table.total_blocks == 0) return (int)hipErrorInvalidValue;
  PackTable t = table;
  void* argv[1] = {&t};
  return (int)hipLaunchKernel((const void*)fsk::k_pack, dim3(table.total_blocks), dim3(256), argv, 0,
                              static_cast<hipStream_t>(stream));
}

KernelResources pack_kernel_resources() {
  KernelResources r;
  hipFuncAttributes attr;
  if (hipFuncGetAttributes(&attr, (const void*)fsk::k_pack) == hipSuccess) {
    r.vgprs = attr.numRegs;
    r.static_lds = (int32_t)attr.sharedSizeBytes;
    r.from_device = true;
  } else {
    (void)hipGetLastError();
  }
  return r;
}

}  // namespace fs
