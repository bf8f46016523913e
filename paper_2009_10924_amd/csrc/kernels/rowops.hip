// Generic row-stitched skeleton (warp composition, paper Section 4.1): a lane group of L
// lanes owns one row in registers; a pattern is a small functor that reads the row's
// inputs, asks for row reductions (cross-lane all-reduces) and writes outputs.  The
// skeleton does what every row kernel needs and is easy to get wrong: all 128-bit loads
// issued up front, clamped addresses instead of branches for padding lanes / rows,
// padding blanked before use, streaming stores.  A new element-wise / row-reduce /
// element-wise pattern is one `Spec` struct, not a new kernel.
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "kernel_table.hpp"

namespace fsk {
using namespace fs;

// BLOCK = false: a lane group of L lanes of one wavefront owns the row (warp composition).
// BLOCK = true : the whole workgroup owns the row, per-wave partial results meet in LDS
//                (block composition); each reduction of a pattern uses its own LDS slot.
template <typename T, int NI, int NV, int K, bool FAST, bool BLOCK>
struct RowCtx {
  static constexpr int VEC = Elem<T>::VEC;
  float x[NI][K][VEC];      // row inputs, padding slots hold 0
  float cv[NV > 0 ? NV : 1][K][VEC];   // column vectors (one value per column, shared by all rows)
  uint32_t row, lane, L, nvec;
  bool row_ok;
  const RowP& p;
  float* slots;             // BLOCK: [4 reductions][4 waves]
  int next_slot = 0;

  __device__ __forceinline__ RowCtx(const RowP& params, float* lds_slots) : p(params), slots(lds_slots) {
    if (BLOCK) {
      L = blockDim.x;
      lane = threadIdx.x;
      row = blockIdx.x;
    } else {
      L = p.lanes_per_row;
      lane = threadIdx.x & (L - 1);
      row = blockIdx.x * (256u >> p.lanes_log2) + (threadIdx.x >> p.lanes_log2);
    }
    nvec = p.cols / VEC;
    row_ok = FAST || row < p.rows;
  }
  __device__ __forceinline__ bool valid(int k) const { return FAST || lane + k * L < nvec; }
  __device__ __forceinline__ uint32_t vec_at(int k) const { return FAST ? lane + k * L : min(lane + k * L, nvec - 1); }

  __device__ __forceinline__ void load(const T* const (&in)[NI], const T* const (&vec)[NV > 0 ? NV : 1]) {
    const size_t base = (size_t)(FAST ? row : min(row, p.rows - 1)) * p.cols;
    u32x4 raw[NI][K], rawv[NV > 0 ? NV : 1][K];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int k = 0; k < K; ++k) raw[i][k] = load_raw_nt(in[i] + base + vec_at(k) * VEC);
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int k = 0; k < K; ++k) rawv[i][k] = load_raw(vec[i] + vec_at(k) * VEC);
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int k = 0; k < K; ++k) unpack(rawv[i][k], cv[i][k], (const T*)nullptr);
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int k = 0; k < K; ++k) {
        unpack(raw[i][k], x[i][k], (const T*)nullptr);
        if (!valid(k)) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) x[i][k][e] = 0.0f;
        }
      }
  }
  // sum over the row of f(k, e); padding slots must contribute 0 (inputs there are 0)
  template <typename F>
  __device__ __forceinline__ float row_sum(F f) {
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += f(k, e);
    if (BLOCK) return block_allreduce<OpSum>(s, slots + 4 * (next_slot++), (int)(blockDim.x >> 6));
    return group_allreduce<OpSum>(s, (int)L);
  }
  template <typename F>
  __device__ __forceinline__ void store(T* __restrict__ out, F f) const {
    const size_t base = (size_t)row * p.cols;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = f(k, e);
      if (row_ok && valid(k)) store_vec_nt(out + base + (lane + k * L) * VEC, v);
    }
  }
};

// ---- patterns ------------------------------------------------------------------------
// softmax backward: dx = y * (dy - sum_j y_j dy_j);   in0 = y, in1 = dy
struct SoftmaxBwdSpec {
  static constexpr int NI = 2, NV = 0;
  template <typename Ctx, typename T>
  __device__ __forceinline__ static void run(Ctx& c, T* out0, T*) {
    const float s = c.row_sum([&](int k, int e) { return c.x[0][k][e] * c.x[1][k][e]; });
    c.store(out0, [&](int k, int e) { return c.x[0][k][e] * (c.x[1][k][e] - s); });
  }
};

// RMS normalisation: out = x * rsqrt(mean(x^2) + eps) * gamma;   in0 = x, vec0 = gamma, f[0] = eps, f[1] = 1/cols
struct RmsNormSpec {
  static constexpr int NI = 1, NV = 1;
  template <typename Ctx, typename T>
  __device__ __forceinline__ static void run(Ctx& c, T* out0, T*) {
    const float ss = c.row_sum([&](int k, int e) { return c.x[0][k][e] * c.x[0][k][e]; });
    const float r = fast_rsqrt(ss * c.p.f[1] + c.p.f[0]);
    c.store(out0, [&](int k, int e) { return c.x[0][k][e] * r * c.cv[0][k][e]; });
  }
};

template <typename Spec, typename T, int K, bool FAST>
__global__ void __launch_bounds__(256) k_row_wave(const T* __restrict__ in0, const T* __restrict__ in1,
                                                  const T* __restrict__ vec0, const T* __restrict__ vec1,
                                                  T* __restrict__ out0, T* __restrict__ out1, RowP p) {
  RowCtx<T, Spec::NI, Spec::NV, K, FAST, false> c(p, nullptr);
  const T* all_in[2] = {in0, in1};
  const T* all_vec[2] = {vec0, vec1};
  const T* in[Spec::NI];
  const T* vec[Spec::NV > 0 ? Spec::NV : 1] = {nullptr};
#pragma unroll
  for (int i = 0; i < Spec::NI; ++i) in[i] = all_in[i];
#pragma unroll
  for (int i = 0; i < Spec::NV; ++i) vec[i] = all_vec[i];
  c.load(in, vec);
  Spec::run(c, out0, out1);
}

template <typename Spec, typename T, int K, bool FAST>
__global__ void __launch_bounds__(256) k_row_block(const T* __restrict__ in0, const T* __restrict__ in1,
                                                   const T* __restrict__ vec0, const T* __restrict__ vec1,
                                                   T* __restrict__ out0, T* __restrict__ out1, RowP p) {
  __shared__ float slots[16];
  RowCtx<T, Spec::NI, Spec::NV, K, FAST, true> c(p, slots);
  const T* all_in[2] = {in0, in1};
  const T* all_vec[2] = {vec0, vec1};
  const T* in[Spec::NI];
  const T* vec[Spec::NV > 0 ? Spec::NV : 1] = {nullptr};
#pragma unroll
  for (int i = 0; i < Spec::NI; ++i) in[i] = all_in[i];
#pragma unroll
  for (int i = 0; i < Spec::NV; ++i) vec[i] = all_vec[i];
  c.load(in, vec);
  Spec::run(c, out0, out1);
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
