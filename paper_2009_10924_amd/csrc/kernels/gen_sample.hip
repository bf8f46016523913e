// Build-time check of the generated kernels' support header: fixed kernels written the way the
// code generator writes them, so that the header is compiled (and its templates instantiated for
// every storage type, both step widths and both row forms) whenever the library is built.  They
// are never launched.
#include <hip/hip_runtime.h>

#include "gen_support.hpp"

using namespace fsk;

template <typename TI, typename TO, int VEC, int K, uint32_t L, bool BLOCK>
__device__ __forceinline__ void sample_body(const GenArgs& a) {
  typedef GenRow<1000u, 64u * VEC * K, VEC, K, L, BLOCK> Row;
  constexpr int KV = Row::KV;
  __shared__ float slots[8];
  const Row row(blockIdx.x);
  const auto raw_full0 = row.template load<TI, true>(a.full[0], (size_t)row.row_c);
  const auto raw_col0 = row.template load<float, false>(a.col[0], 0);
  float acc[KV], c0[KV], sacc;
  row.template unpack_to<float>(raw_col0, c0);
  row.template unpack_to<TI>(raw_full0, acc);
  sacc = row.template reduce<OpSum, false, true>(acc, slots);
  sacc = fast_rsqrt(sacc * (1.0f / (64 * VEC * K)) + 1e-6f);
#pragma unroll
  for (int j = 0; j < KV; ++j) acc[j] = gen_round<2>(acc[j] * sacc) * c0[j];
  row.template store<TO>(a.out[0], acc);
  sacc = row.template reduce<OpMax, true, false>(acc, slots + 4);
  row.template store_scalar<TO>(a.rout[0], sacc);
}

extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_wave_f32(const GenArgs a) { sample_body<float, bf16_t, 4, 2, 32u, false>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_wave_f16(const GenArgs a) { sample_body<f16_t, float, 8, 1, 64u, false>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_block_bf16(const GenArgs a) { sample_body<bf16_t, f16_t, 8, 4, 256u, true>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_wide_f32(const GenArgs a) { sample_body<float, float, 8, 1, 8u, false>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_half_width_bf16(const GenArgs a) { sample_body<bf16_t, bf16_t, 4, 2, 16u, false>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_half_width_f16(const GenArgs a) { sample_body<f16_t, f16_t, 4, 1, 256u, true>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_element_f32(const GenArgs a) { sample_body<float, float, 1, 5, 64u, false>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_element_bf16(const GenArgs a) { sample_body<bf16_t, f16_t, 1, 3, 32u, false>(a); }
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_element_f16(const GenArgs a) { sample_body<f16_t, bf16_t, 1, 7, 256u, true>(a); }

// a pattern with a column sum: two rows per lane group, partial sums through LDS to the workspace
extern "C" __global__ void __launch_bounds__(256) fs_gen_sample_colsum(const GenArgs a) {
  typedef GenRow<1000u, 96u, 4, 3, 8u, false, 2u> Row;
  constexpr int KV = Row::KV;
  __shared__ float colred[1][4 * Row::PADDED_COLS];
  float cs0[KV];
#pragma unroll
  for (int j = 0; j < KV; ++j) cs0[j] = 0.0f;
#pragma unroll 1
  for (uint32_t it = 0; it < 2u; ++it) {
    const Row row(it * gridDim.x + blockIdx.x);
    const auto raw_full0 = row.load<float, true>(a.full[0], (size_t)row.row_c);
    float acc[KV];
    row.unpack_to<float>(raw_full0, acc);
    row.store<float>(a.out[0], acc);
    row.colsum_add(acc, cs0);
  }
  Row::colsum_flush(cs0, colred[0], static_cast<float*>(a.ws) + (size_t)blockIdx.x * 96u);
}
