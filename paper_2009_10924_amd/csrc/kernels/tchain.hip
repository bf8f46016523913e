// Stitched transpose + per-head scale + L2 normalisation of the last axis:
//     t = transpose(x, (0,2,1,3));  u = t * scale[h];  out = u * rsqrt(sum_d u^2 + eps)
// x is [B,S,H,D], out is [B,H,S,D]; 7 ops, one kernel.  The permutation keeps the
// innermost axis, so a row of D elements moves as a unit; its sum of squares is a
// cross-lane all-reduce over the L lanes that hold it (warp composition).
//   * wave variant: a workgroup walks the rows of an [s_tile, H] slab in input order
//     (reads contiguous), each lane group stores its row straight to its transposed
//     position (D-element contiguous pieces).
//   * LDS variant (block composition): the normalised slab is parked in LDS and
//     written out in output order, so both HBM sides see long contiguous runs.
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "kernel_table.hpp"

namespace fsk {
using namespace fs;

template <typename T, int K>
__device__ __forceinline__ void tchain_row(const T* __restrict__ xrow, float scale, float eps, uint32_t lane,
                                           uint32_t L, uint32_t nvec, bool ok, float (&v)[K][Elem<T>::VEC]) {
  constexpr int VEC = Elem<T>::VEC;
  float ss = 0.0f;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const uint32_t j = lane + k * L;
    if (ok && j < nvec) {
      load_vec(xrow + j * VEC, v[k]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        v[k][e] *= scale;
        ss = __builtin_fmaf(v[k][e], v[k][e], ss);
      }
    } else {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[k][e] = 0.0f;
    }
  }
  ss = group_allreduce<OpSum>(ss, L);
  const float r = fast_rsqrt(ss + eps);
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[k][e] *= r;
}

template <typename T, int K>
__global__ void __launch_bounds__(256) k_tchain_wave(const T* __restrict__ x, const T* __restrict__ scale,
                                                     T* __restrict__ out, TChainP p) {
  constexpr int VEC = Elem<T>::VEC;
  const uint32_t L = p.lanes_per_row;
  const uint32_t groups = 256u / L;
  const uint32_t group = threadIdx.x / L, lane = threadIdx.x & (L - 1);
  const uint32_t nvec = p.D / VEC;
  const uint32_t s_tiles = (p.S + p.s_tile - 1) / p.s_tile;
  const uint32_t b = blockIdx.x / s_tiles;
  const uint32_t s0 = (blockIdx.x % s_tiles) * p.s_tile;
  const uint32_t s_cnt = min((uint32_t)p.s_tile, p.S - s0);
  const uint32_t n_rows = s_cnt * p.H;                    // rows of this slab, input order (s, h)
  const uint32_t passes = (p.s_tile * p.H + groups - 1) / groups;
  for (uint32_t it = 0; it < passes; ++it) {
    const uint32_t idx = it * groups + group;
    const bool ok = idx < n_rows;
    const uint32_t sl = idx / p.H, h = idx % p.H;
    float v[K][VEC];
    const T* xrow = x + ((size_t)(b * p.S + s0 + sl) * p.H + h) * p.D;
    const float sc = ok ? load1(scale + h) : 0.0f;
    tchain_row<T, K>(xrow, sc, p.eps, lane, L, nvec, ok, v);
    T* orow = out + ((size_t)(b * p.H + h) * p.S + s0 + sl) * p.D;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const uint32_t j = lane + k * L;
      if (ok && j < nvec) store_vec(orow + j * VEC, v[k]);
    }
  }
}

template <typename T, int K>
__global__ void __launch_bounds__(256) k_tchain_lds(const T* __restrict__ x, const T* __restrict__ scale,
                                                    T* __restrict__ out, TChainP p) {
  constexpr int VEC = Elem<T>::VEC;
  extern __shared__ float slab[];                          // [s_tile * H][pitch] float32
  const uint32_t L = p.lanes_per_row;
  const uint32_t groups = 256u / L;
  const uint32_t group = threadIdx.x / L, lane = threadIdx.x & (L - 1);
  const uint32_t nvec = p.D / VEC;
  const uint32_t pitch = p.D + 4;                          // skew rows across LDS banks
  const uint32_t s_tiles = (p.S + p.s_tile - 1) / p.s_tile;
  const uint32_t b = blockIdx.x / s_tiles;
  const uint32_t s0 = (blockIdx.x % s_tiles) * p.s_tile;
  const uint32_t s_cnt = min((uint32_t)p.s_tile, p.S - s0);
  const uint32_t n_rows = s_cnt * p.H;
  const uint32_t passes = (p.s_tile * p.H + groups - 1) / groups;
  for (uint32_t it = 0; it < passes; ++it) {
    const uint32_t idx = it * groups + group;
    const bool ok = idx < n_rows;
    const uint32_t sl = idx / p.H, h = idx % p.H;
    float v[K][VEC];
    const T* xrow = x + ((size_t)(b * p.S + s0 + sl) * p.H + h) * p.D;
    const float sc = ok ? load1(scale + h) : 0.0f;
    tchain_row<T, K>(xrow, sc, p.eps, lane, L, nvec, ok, v);
    if (ok) {
      float* dst = slab + (h * p.s_tile + sl) * pitch;     // parked in output order (h, s)
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const uint32_t j = lane + k * L;
        if (j < nvec) {
#pragma unroll
          for (int e = 0; e < VEC; e += 4) {
            f32x4 t = {v[k][e], v[k][e + 1], v[k][e + 2], v[k][e + 3]};
            *reinterpret_cast<f32x4*>(dst + j * VEC + e) = t;
          }
        }
      }
    }
  }
  __syncthreads();
  // write phase: for each head the s_cnt rows are contiguous in the output
  const uint32_t vec_per_head = s_cnt * nvec;
  for (uint32_t i = threadIdx.x; i < p.H * vec_per_head; i += 256u) {
    const uint32_t h = i / vec_per_head, rem = i % vec_per_head;
    const uint32_t sl = rem / nvec, j = rem % nvec;
    const float* src = slab + (h * p.s_tile + sl) * pitch + j * VEC;
    float v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; e += 4) {
      f32x4 t = *reinterpret_cast<const f32x4*>(src + e);
      v[e] = t.x; v[e + 1] = t.y; v[e + 2] = t.z; v[e + 3] = t.w;
    }
    store_vec(out + ((size_t)(b * p.H + h) * p.S + s0 + sl) * p.D + j * VEC, v);
  }
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename T>
const void* tc_sym(int32_t kernel, int K) {
#define FS_TC_CASE(KK) \
  case KK: return kernel == K_TCHAIN_WAVE ? (const void*)k_tchain_wave<T, KK> : (const void*)k_tchain_lds<T, KK>;
  switch (K) {
    FS_TC_CASE(1) FS_TC_CASE(2) FS_TC_CASE(4)
    default: return nullptr;
  }
#undef FS_TC_CASE
}
}  // namespace

const void* tchain_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  const TChainP& p = a.u.tchain;
  switch (p.dt) {
    case DT_F32: return tc_sym<float>(kernel, p.vecs_per_lane);
    case DT_F16: return tc_sym<f16_t>(kernel, p.vecs_per_lane);
    default: return tc_sym<bf16_t>(kernel, p.vecs_per_lane);
  }
}

}  // namespace fs
