// Stand-alone kernels of the generic row-stitched skeleton: one launch serves one pattern
// over one row tensor, in the wave form (a lane group per row) or the block form (a
// workgroup per row).
#include <hip/hip_runtime.h>

#include "kernel_table.hpp"
#include "row_skeleton.hpp"

namespace fsk {

template <typename Spec, typename T, typename Ctx>
__device__ __forceinline__ void run_row_pattern(Ctx& c, const T* in0, const T* in1, const T* vec0, const T* vec1, T* out0) {
  const T* all_in[2] = {in0, in1};
  const T* all_vec[2] = {vec0, vec1};
  const T* in[Spec::NI];
  const T* vec[Spec::NV > 0 ? Spec::NV : 1] = {nullptr};
#pragma unroll
  for (int i = 0; i < Spec::NI; ++i) in[i] = all_in[i];
#pragma unroll
  for (int i = 0; i < Spec::NV; ++i) vec[i] = all_vec[i];
  c.load(in, vec);
  Spec::run(c, out0);
}

template <typename Spec, typename T, int K, bool FAST>
__global__ void __launch_bounds__(256) k_row_wave(const T* __restrict__ in0, const T* __restrict__ in1,
                                                  const T* __restrict__ vec0, const T* __restrict__ vec1,
                                                  T* __restrict__ out0, T* __restrict__ out1, RowP p) {
  RowCtx<T, T, Spec::NI, Spec::NV, K, FAST, MODE_WAVE> c(p, nullptr, blockIdx.x);
  run_row_pattern<Spec, T>(c, in0, in1, vec0, vec1, out0);
}

template <typename Spec, typename T, int K, bool FAST>
__global__ void __launch_bounds__(256) k_row_block(const T* __restrict__ in0, const T* __restrict__ in1,
                                                   const T* __restrict__ vec0, const T* __restrict__ vec1,
                                                   T* __restrict__ out0, T* __restrict__ out1, RowP p) {
  __shared__ float slots[16];
  RowCtx<T, T, Spec::NI, Spec::NV, K, FAST, MODE_BLOCK> c(p, slots, blockIdx.x);
  run_row_pattern<Spec, T>(c, in0, in1, vec0, vec1, out0);
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename Spec, typename T>
const void* row_sym(int32_t kernel, int K, bool fast) {
  if (kernel == K_ROW_BLOCK) {
    switch (K) {
      case 1: return fast ? (const void*)k_row_block<Spec, T, 1, true> : (const void*)k_row_block<Spec, T, 1, false>;
      case 2: return fast ? (const void*)k_row_block<Spec, T, 2, true> : (const void*)k_row_block<Spec, T, 2, false>;
      case 4: return fast ? (const void*)k_row_block<Spec, T, 4, true> : (const void*)k_row_block<Spec, T, 4, false>;
      default: return nullptr;
    }
  }
#define FS_ROW_CASE(KK) \
  case KK: return fast ? (const void*)k_row_wave<Spec, T, KK, true> : (const void*)k_row_wave<Spec, T, KK, false>;
  switch (K) {
    FS_ROW_CASE(1) FS_ROW_CASE(2) FS_ROW_CASE(4) FS_ROW_CASE(8)
    default: return nullptr;
  }
#undef FS_ROW_CASE
}
template <typename Spec>
const void* row_sym_dt(int32_t kernel, const RowP& p) {
  switch (p.dt) {
    case DT_F32: return row_sym<Spec, float>(kernel, p.vecs_per_lane, p.fast != 0);
    case DT_F16: return row_sym<Spec, f16_t>(kernel, p.vecs_per_lane, p.fast != 0);
    default: return row_sym<Spec, bf16_t>(kernel, p.vecs_per_lane, p.fast != 0);
  }
}
}  // namespace

const void* rowops_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  const RowP& p = a.u.row;
  switch (p.pattern) {
    case ROW_SOFTMAX_BWD: return row_sym_dt<SoftmaxBwdSpec>(kernel, p);
    case ROW_RMSNORM: return row_sym_dt<RmsNormSpec>(kernel, p);
    default: return nullptr;
  }
}

}  // namespace fs
