// Stitched row softmax with optional scale and additive mask:
//     y = softmax_lastaxis(scale * x + mask)
// i.e. (scale) -> (add mask) -> row max -> subtract -> exp -> row sum -> divide as ONE
// kernel.  Each input element is read once, each output written once; the two row
// reductions are reused by every lane of the row without leaving the chip:
//   * wave variant  (warp composition, paper Section 4.1): a row lives in the
//     registers of an aligned group of L lanes of one wavefront; reductions are
//     DPP / permute all-reduces, so every lane ends up holding the reduced value.
//   * block variant (block composition): a row lives in the registers of one
//     workgroup; per-wave results meet in LDS.
//   * generic variant: any row length / alignment, block per row, three passes
//     over the row (the later ones hit L2), reduced values through LDS.
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "kernel_table.hpp"

namespace fsk {
using namespace fs;

// Loads the row segment of one lane.  Every load is issued before any value is used:
// out-of-range vectors and rows are clamped to a valid address and blanked afterwards,
// so no branch separates the loads and all of them are in flight together.
// FAST: the row fills the lanes exactly, the rows fill the workgroups exactly and a mask,
// if any, varies along the row: clamps, padding masks and flag tests fold away.
template <typename T, int K, bool HAS_MASK, bool FAST>
__device__ __forceinline__ void softmax_load(const T* __restrict__ x, const T* __restrict__ mask, const SoftmaxP& p,
                                             uint32_t row, uint32_t lane, uint32_t stride,
                                             float (&v)[K][Elem<T>::VEC]) {
  constexpr int VEC = Elem<T>::VEC;
  const uint32_t nvec = p.cols / VEC;
  const uint32_t r = FAST ? row : min(row, p.rows - 1);
  const T* xr = x + (size_t)r * p.cols;
  auto vec_at = [&](int k) { return FAST ? lane + k * stride : min(lane + k * stride, nvec - 1); };
  const bool mask_inner = FAST || p.mask_inner;
  u32x4 raw[K], rawm[K];
  float mscalar = 0.0f;
#pragma unroll
  for (int k = 0; k < K; ++k) raw[k] = load_raw_nt(xr + vec_at(k) * VEC);
  if constexpr (HAS_MASK) {
    const uint32_t r1 = fast_div(r, p.od[2]);
    const uint32_t c2 = r - r1 * p.od[2].d;
    const uint32_t c0 = fast_div(r1, p.od[1]);
    const uint32_t c1 = r1 - c0 * p.od[1].d;
    const T* mrow = mask + (c0 * p.ms[0] + c1 * p.ms[1] + c2 * p.ms[2]);
    if (mask_inner) {
#pragma unroll
      for (int k = 0; k < K; ++k) rawm[k] = load_raw(mrow + vec_at(k) * VEC);
    } else {
      mscalar = load1(mrow);
    }
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    unpack(raw[k], v[k], (const T*)nullptr);
    if constexpr (HAS_MASK) {
      float m[VEC];
      if (mask_inner) {
        unpack(rawm[k], m, (const T*)nullptr);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) m[e] = mscalar;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k][e] = v[k][e] * p.scale + m[e];
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k][e] *= p.scale;
    }
    if (!FAST && lane + k * stride >= nvec) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k][e] = -INFINITY;
    }
  }
}

template <int K, int VEC>
__device__ __forceinline__ float local_max(const float (&v)[K][VEC]) {
  float m = -INFINITY;
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int e = 0; e < VEC; ++e) m = fmaxf(m, v[k][e]);
  return m;
}

template <int K, int VEC>
__device__ __forceinline__ float exp_and_sum(float (&v)[K][VEC], float m) {
  const float mb = m * kLog2e;
  float s = 0.0f;
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      v[k][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(v[k][e], kLog2e, -mb));
      s += v[k][e];
    }
  return s;
}

template <typename T, int K, bool FAST>
__device__ __forceinline__ void softmax_store(T* __restrict__ out, const SoftmaxP& p, uint32_t row, bool row_ok,
                                              uint32_t lane, uint32_t stride, float (&v)[K][Elem<T>::VEC], float inv) {
  constexpr int VEC = Elem<T>::VEC;
  const uint32_t nvec = p.cols / VEC;
  T* orow = out + (size_t)row * p.cols;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const uint32_t j = lane + k * stride;
    if (FAST || (row_ok && j < nvec)) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k][e] *= inv;
      store_vec_nt(orow + j * VEC, v[k]);
    }
  }
}

// ---- wave variant ------------------------------------------------------------------
template <typename T, int K, bool HAS_MASK, bool FAST>
__global__ void __launch_bounds__(256) k_softmax_wave(const T* __restrict__ x, const T* __restrict__ mask,
                                                      T* __restrict__ out, SoftmaxP p) {
  constexpr int VEC = Elem<T>::VEC;
  const uint32_t L = p.lanes_per_row;            // power of two, <= 64
  const uint32_t group = threadIdx.x >> p.lanes_log2;
  const uint32_t lane = threadIdx.x & (L - 1);
  const uint32_t row = blockIdx.x * (256u >> p.lanes_log2) + group;
  const bool row_ok = row < p.rows;
  float v[K][VEC];
  softmax_load<T, K, HAS_MASK, FAST>(x, mask, p, row, lane, L, v);
  const float m = group_allreduce<OpMax>(local_max<K, VEC>(v), L);
  const float s = group_allreduce<OpSum>(exp_and_sum<K, VEC>(v, m), L);
  softmax_store<T, K, FAST>(out, p, row, row_ok, lane, L, v, fast_rcp(s));
}

// ---- block variant -----------------------------------------------------------------
template <typename T, int K, bool HAS_MASK, bool FAST>
__global__ void __launch_bounds__(256) k_softmax_block(const T* __restrict__ x, const T* __restrict__ mask,
                                                       T* __restrict__ out, SoftmaxP p) {
  constexpr int VEC = Elem<T>::VEC;
  __shared__ float slot_max[4], slot_sum[4];
  const uint32_t row = blockIdx.x;
  const uint32_t n_waves = blockDim.x >> 6;
  float v[K][VEC];
  softmax_load<T, K, HAS_MASK, FAST>(x, mask, p, row, threadIdx.x, blockDim.x, v);
  const float m = block_allreduce<OpMax>(local_max<K, VEC>(v), slot_max, n_waves);
  const float s = block_allreduce<OpSum>(exp_and_sum<K, VEC>(v, m), slot_sum, n_waves);
  softmax_store<T, K, FAST>(out, p, row, true, threadIdx.x, blockDim.x, v, fast_rcp(s));
}

// ---- generic variant ---------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_softmax_generic(const T* __restrict__ x, const T* __restrict__ mask,
                                                         T* __restrict__ out, SoftmaxP p) {
  __shared__ float slot_max[4], slot_sum[4];
  const uint32_t row = blockIdx.x;
  uint32_t moff = 0;
  if (p.has_mask) {
    const uint32_t r1 = fast_div(row, p.od[2]);
    const uint32_t c0 = fast_div(r1, p.od[1]);
    moff = c0 * p.ms[0] + (r1 - c0 * p.od[1].d) * p.ms[1] + (row - r1 * p.od[2].d) * p.ms[2];
  }
  const T* xr = x + (size_t)row * p.cols;
  auto value = [&](uint32_t c) {
    float a = load1(xr + c) * p.scale;
    if (p.has_mask) a += load1(mask + moff + (p.mask_inner ? c : 0u));
    return a;
  };
  float m = -INFINITY;
  for (uint32_t c = threadIdx.x; c < p.cols; c += 256u) m = fmaxf(m, value(c));
  m = block_allreduce<OpMax>(m, slot_max, 4);
  float s = 0.0f;
  for (uint32_t c = threadIdx.x; c < p.cols; c += 256u) s += fast_exp(value(c) - m);
  s = block_allreduce<OpSum>(s, slot_sum, 4);
  const float inv = fast_rcp(s);
  T* orow = out + (size_t)row * p.cols;
  for (uint32_t c = threadIdx.x; c < p.cols; c += 256u) store1(orow + c, fast_exp(value(c) - m) * inv);
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename T, bool M, bool F>
const void* wave_sym(int K) {
  switch (K) {
    case 1: return (const void*)k_softmax_wave<T, 1, M, F>;
    case 2: return (const void*)k_softmax_wave<T, 2, M, F>;
    case 4: return (const void*)k_softmax_wave<T, 4, M, F>;
    default: return (const void*)k_softmax_wave<T, 8, M, F>;
  }
}
template <typename T, bool M, bool F>
const void* block_sym(int K) {
  switch (K) {
    case 1: return (const void*)k_softmax_block<T, 1, M, F>;
    case 2: return (const void*)k_softmax_block<T, 2, M, F>;
    case 4: return (const void*)k_softmax_block<T, 4, M, F>;
    default: return (const void*)k_softmax_block<T, 8, M, F>;
  }
}
template <typename T, bool M>
const void* sym_mf(int32_t kernel, const SoftmaxP& p) {
  if (kernel == K_SOFTMAX_WAVE) return p.fast ? wave_sym<T, M, true>(p.vecs_per_lane) : wave_sym<T, M, false>(p.vecs_per_lane);
  return p.fast ? block_sym<T, M, true>(p.vecs_per_lane) : block_sym<T, M, false>(p.vecs_per_lane);
}
template <typename T>
const void* sym_for(int32_t kernel, const SoftmaxP& p) {
  if (p.vecs_per_lane == 0) return (const void*)k_softmax_generic<T>;
  return p.has_mask ? sym_mf<T, true>(kernel, p) : sym_mf<T, false>(kernel, p);
}
}  // namespace

const void* softmax_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  const SoftmaxP& p = a.u.softmax;
  switch (p.in_dt) {
    case DT_F32: return sym_for<float>(kernel, p);
    case DT_F16: return sym_for<f16_t>(kernel, p);
    default: return sym_for<bf16_t>(kernel, p);
  }
}

}  // namespace fs
