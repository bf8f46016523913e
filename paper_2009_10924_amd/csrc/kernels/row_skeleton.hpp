// Generic row-stitched skeleton (paper Section 4.1, warp and block composition): a lane
// group of L lanes of one wavefront -- or a whole workgroup -- owns one row in registers; a
// pattern is a small functor (`Spec`) that reads the row's inputs, asks for row reductions
// (cross-lane / cross-wave all-reduces) and writes outputs.  The skeleton does what every
// row kernel needs and is easy to get wrong: all 128-bit loads issued up front, clamped
// addresses instead of branches for padding lanes / rows, padding blanked before use,
// streaming stores.  A new element-wise / row-reduce / element-wise pattern is one `Spec`
// struct, not a new kernel.
#pragma once
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "launch.hpp"

namespace fsk {
using namespace fs;

// MODE_WAVE   : a lane group of L lanes of one wavefront owns the row (warp composition).
// MODE_BLOCK  : the whole workgroup owns the row, per-wave partial results meet in LDS
//               (block composition); each reduction of a pattern uses its own LDS slot.
// MODE_RUNTIME: lanes_per_row > 64 selects the block form at run time (packed launches,
//               where one kernel serves members of either form).
enum RowMode : int { MODE_WAVE = 0, MODE_BLOCK = 1, MODE_RUNTIME = 2 };

template <typename T, typename TO, int NI, int NV, int K, bool FAST, int MODE>
struct RowCtx {
  static constexpr int VEC = Elem<T>::VEC;
  float x[NI][K][VEC];                 // row inputs, padding slots hold 0
  float cv[NV > 0 ? NV : 1][K][VEC];   // column vectors (one value per column, shared by all rows)
  uint32_t row, lane, L, nvec;
  bool row_ok, block_mode;
  const RowP& p;
  float* slots;                        // block form: [4 reductions][4 waves]
  int next_slot = 0;

  // vblock: index of this workgroup among the workgroups that serve this row tensor
  __device__ __forceinline__ RowCtx(const RowP& params, float* lds_slots, uint32_t vblock)
      : p(params), slots(lds_slots) {
    block_mode = MODE == MODE_BLOCK || (MODE == MODE_RUNTIME && params.lanes_per_row > 64);
    if (block_mode) {
      L = blockDim.x;
      lane = threadIdx.x;
      row = vblock;
    } else {
      L = p.lanes_per_row;
      lane = threadIdx.x & (L - 1);
      row = vblock * (256u >> p.lanes_log2) + (threadIdx.x >> p.lanes_log2);
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
  template <typename OP>
  __device__ __forceinline__ float reduce(float s) {
    if (MODE == MODE_BLOCK) return block_allreduce<OP>(s, slots + 4 * (next_slot++), (int)(blockDim.x >> 6));
    if (MODE == MODE_RUNTIME && block_mode) return block_allreduce<OP>(s, slots + 4 * (next_slot++), (int)(blockDim.x >> 6));
    return group_allreduce<OP>(s, (int)L);
  }
  // sum over the row of f(k, e); padding slots must contribute 0 (inputs there are 0)
  template <typename F>
  __device__ __forceinline__ float row_sum(F f) {
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += f(k, e);
    return reduce<OpSum>(s);
  }
  // max over the row of f(k, e); padding slots are left out
  template <typename F>
  __device__ __forceinline__ float row_max(F f) {
    float m = -INFINITY;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const bool ok = valid(k);
#pragma unroll
      for (int e = 0; e < VEC; ++e) m = fmaxf(m, ok ? f(k, e) : -INFINITY);
    }
    return reduce<OpMax>(m);
  }
  template <typename F>
  __device__ __forceinline__ void store(TO* __restrict__ out, F f) const {
    const size_t base = (size_t)row * p.cols;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = f(k, e);
      if (row_ok && valid(k)) StoreN<TO, VEC>::run(out + base + (size_t)(lane + k * L) * VEC, v);
    }
  }
};

// ---- patterns ------------------------------------------------------------------------
// NI row inputs in0.., NV column vectors vec0.., scalars in RowP::f.

// softmax backward: dx = y * (dy - sum_j y_j dy_j);   in0 = y, in1 = dy
struct SoftmaxBwdSpec {
  static constexpr int NI = 2, NV = 0;
  template <typename Ctx, typename TO>
  __device__ __forceinline__ static void run(Ctx& c, TO* out0) {
    const float s = c.row_sum([&](int k, int e) { return c.x[0][k][e] * c.x[1][k][e]; });
    c.store(out0, [&](int k, int e) { return c.x[0][k][e] * (c.x[1][k][e] - s); });
  }
};

// RMS normalisation: out = x * rsqrt(mean(x^2) + eps) * gamma;   in0 = x, vec0 = gamma, f[0] = eps, f[1] = 1/cols
struct RmsNormSpec {
  static constexpr int NI = 1, NV = 1;
  template <typename Ctx, typename TO>
  __device__ __forceinline__ static void run(Ctx& c, TO* out0) {
    const float ss = c.row_sum([&](int k, int e) { return c.x[0][k][e] * c.x[0][k][e]; });
    const float r = fast_rsqrt(ss * c.p.f[1] + c.p.f[0]);
    c.store(out0, [&](int k, int e) { return c.x[0][k][e] * r * c.cv[0][k][e]; });
  }
};

// softmax over the row of f[0] * x;   in0 = x
struct SoftmaxSpec {
  static constexpr int NI = 1, NV = 0;
  template <typename Ctx, typename TO>
  __device__ __forceinline__ static void run(Ctx& c, TO* out0) {
    const float sc = c.p.f[0] * kLog2e;                       // exp(a - m) = exp2(a log2e - m log2e)
    const float m = c.row_max([&](int k, int e) { return c.x[0][k][e] * sc; });
    const float s = c.row_sum([&](int k, int e) {
      const float v = c.valid(k) ? __builtin_amdgcn_exp2f(__builtin_fmaf(c.x[0][k][e], sc, -m)) : 0.0f;
      c.x[0][k][e] = v;
      return v;
    });
    const float inv = fast_rcp(s);
    c.store(out0, [&](int k, int e) { return c.x[0][k][e] * inv; });
  }
};

// LayerNorm with affine output, two-pass variance on the register-resident row.
//   RES_BIAS: h = x + res + bias; in0 = x, in1 = res, vec0 = bias, vec1 = gamma, vec2 = beta
//   else    : h = x;              in0 = x,            vec0 = gamma, vec1 = beta
//   f[0] = eps, f[1] = 1/cols
template <bool RES_BIAS>
struct LayerNormSpec {
  static constexpr int NI = RES_BIAS ? 2 : 1, NV = RES_BIAS ? 3 : 2;
  template <typename Ctx, typename TO>
  __device__ __forceinline__ static void run(Ctx& c, TO* out0) {
    constexpr int G = RES_BIAS ? 1 : 0;
    const float mean = c.p.f[1] * c.row_sum([&](int k, int e) {
      if (RES_BIAS) c.x[0][k][e] = c.valid(k) ? c.x[0][k][e] + c.x[NI - 1][k][e] + c.cv[0][k][e] : 0.0f;
      return c.x[0][k][e];
    });
    const float var = c.p.f[1] * c.row_sum([&](int k, int e) {
      const float d = c.valid(k) ? c.x[0][k][e] - mean : 0.0f;
      c.x[0][k][e] = d;
      return d * d;
    });
    const float rstd = fast_rsqrt(var + c.p.f[0]);
    c.store(out0, [&](int k, int e) { return __builtin_fmaf(c.x[0][k][e] * rstd, c.cv[G][k][e], c.cv[G + 1][k][e]); });
  }
};

// y = gelu_tanh(x + bias): no reduction, the row form only gives the column index;   in0 = x, vec0 = bias
struct BiasGeluSpec {
  static constexpr int NI = 1, NV = 1;
  template <typename Ctx, typename TO>
  __device__ __forceinline__ static void run(Ctx& c, TO* out0) {
    c.store(out0, [&](int k, int e) { return gelu_fwd(c.x[0][k][e] + c.cv[0][k][e]); });
  }
};

}  // namespace fsk
