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

// One workgroup owns the [s_tile, H] slab of rows at (b, s0); lane group g handles rows
// g, g + groups, ... (input order, so a wavefront reads consecutive rows).  PASSES rows
// per lane group are loaded up front so that all loads are in flight together; rows
// past the slab are clamped to its last row and dropped at the store.
template <typename T, int K, int PASSES>
struct TChainTile {
  static constexpr int VEC = Elem<T>::VEC;
  float v[PASSES][K][VEC];
  uint32_t sl[PASSES], h[PASSES];
  bool ok[PASSES];

  __device__ __forceinline__ void run(const T* __restrict__ x, const T* __restrict__ scale, const TChainP& p,
                                      uint32_t b, uint32_t s0, uint32_t n_rows, uint32_t group, uint32_t groups,
                                      uint32_t lane, uint32_t L) {
    const uint32_t nvec = p.D / VEC;
    u32x4 raw[PASSES][K];
    float sc[PASSES];
#pragma unroll
    for (int it = 0; it < PASSES; ++it) {
      const uint32_t idx = it * groups + group;
      ok[it] = idx < n_rows;
      const uint32_t cidx = min(idx, n_rows - 1);
      sl[it] = fast_div(cidx, p.div_h);
      h[it] = cidx - sl[it] * p.H;
      const T* xrow = x + ((size_t)(b * p.S + s0 + sl[it]) * p.H + h[it]) * p.D;
#pragma unroll
      for (int k = 0; k < K; ++k) raw[it][k] = load_raw_nt(xrow + min(lane + k * L, nvec - 1) * VEC);
      sc[it] = load1(scale + h[it]);
    }
#pragma unroll
    for (int it = 0; it < PASSES; ++it) {
      float ss = 0.0f;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        unpack(raw[it][k], v[it][k], (const T*)nullptr);
        const float s = (lane + k * L < nvec) ? sc[it] : 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          v[it][k][e] *= s;
          ss = __builtin_fmaf(v[it][k][e], v[it][k][e], ss);
        }
      }
      ss = group_allreduce<OpSum>(ss, L);
      const float r = fast_rsqrt(ss + p.eps);
#pragma unroll
      for (int k = 0; k < K; ++k)
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[it][k][e] *= r;
    }
  }
};

template <typename T, int K, int PASSES>
__global__ void __launch_bounds__(256) k_tchain_wave(const T* __restrict__ x, const T* __restrict__ scale,
                                                     T* __restrict__ out, TChainP p) {
  constexpr int VEC = Elem<T>::VEC;
  const uint32_t L = p.lanes_per_row;
  const uint32_t groups = 256u >> p.lanes_log2;
  const uint32_t group = threadIdx.x >> p.lanes_log2, lane = threadIdx.x & (L - 1);
  const uint32_t nvec = p.D / VEC;
  const uint32_t b = fast_div(blockIdx.x, p.div_s_tiles);
  const uint32_t s0 = (blockIdx.x - b * p.div_s_tiles.d) * p.s_tile;
  const uint32_t s_cnt = min((uint32_t)p.s_tile, p.S - s0);
  TChainTile<T, K, PASSES> t;
  t.run(x, scale, p, b, s0, s_cnt * p.H, group, groups, lane, L);
#pragma unroll
  for (int it = 0; it < PASSES; ++it) {
    T* orow = out + ((size_t)(b * p.H + t.h[it]) * p.S + s0 + t.sl[it]) * p.D;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const uint32_t j = lane + k * L;
      if (t.ok[it] && j < nvec) store_vec_nt(orow + j * VEC, t.v[it][k]);
    }
  }
}

template <typename T, int K, int PASSES>
__global__ void __launch_bounds__(256) k_tchain_lds(const T* __restrict__ x, const T* __restrict__ scale,
                                                    T* __restrict__ out, TChainP p) {
  constexpr int VEC = Elem<T>::VEC;
  extern __shared__ float slab[];                          // [H][s_tile][pitch] float32, output order
  const uint32_t L = p.lanes_per_row;
  const uint32_t groups = 256u >> p.lanes_log2;
  const uint32_t group = threadIdx.x >> p.lanes_log2, lane = threadIdx.x & (L - 1);
  const uint32_t nvec = p.D / VEC;
  const uint32_t pitch = p.D + 4;                          // skew rows across LDS banks
  const uint32_t b = fast_div(blockIdx.x, p.div_s_tiles);
  const uint32_t s0 = (blockIdx.x - b * p.div_s_tiles.d) * p.s_tile;
  const uint32_t s_cnt = min((uint32_t)p.s_tile, p.S - s0);
  {
    TChainTile<T, K, PASSES> t;
    t.run(x, scale, p, b, s0, s_cnt * p.H, group, groups, lane, L);
#pragma unroll
    for (int it = 0; it < PASSES; ++it) {
      float* dst = slab + (t.h[it] * p.s_tile + t.sl[it]) * pitch;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        const uint32_t j = lane + k * L;
        if (t.ok[it] && j < nvec) {
#pragma unroll
          for (int e = 0; e < VEC; e += 4) {
            f32x4 q = {t.v[it][k][e], t.v[it][k][e + 1], t.v[it][k][e + 2], t.v[it][k][e + 3]};
            *reinterpret_cast<f32x4*>(dst + j * VEC + e) = q;
          }
        }
      }
    }
  }
  __syncthreads();
  // write phase: for each head the s_cnt rows are contiguous in the output
  const uint32_t vec_per_head = s_cnt * nvec;
  for (uint32_t i = threadIdx.x; i < p.H * vec_per_head; i += 256u) {
    const uint32_t h = i / vec_per_head, rem = i - h * vec_per_head;
    const uint32_t sl = rem / nvec, j = rem - sl * nvec;
    const float* src = slab + (h * p.s_tile + sl) * pitch + j * VEC;
    float v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; e += 4) {
      f32x4 q = *reinterpret_cast<const f32x4*>(src + e);
      v[e] = q.x; v[e + 1] = q.y; v[e + 2] = q.z; v[e + 3] = q.w;
    }
    store_vec_nt(out + ((size_t)(b * p.H + h) * p.S + s0 + sl) * p.D + j * VEC, v);
  }
}

}  // namespace fsk

namespace fs {
using namespace fsk;

namespace {
template <typename T, int K>
const void* tc_sym_kp(int32_t kernel, int passes) {
#define FS_TC_CASE(PP) \
  case PP: return kernel == K_TCHAIN_WAVE ? (const void*)k_tchain_wave<T, K, PP> : (const void*)k_tchain_lds<T, K, PP>;
  switch (passes) {
    FS_TC_CASE(1) FS_TC_CASE(2) FS_TC_CASE(3) FS_TC_CASE(4)
    default: return nullptr;
  }
#undef FS_TC_CASE
}
template <typename T>
const void* tc_sym(int32_t kernel, int K, int passes) {
  switch (K) {
    case 1: return tc_sym_kp<T, 1>(kernel, passes);
    case 2: return tc_sym_kp<T, 2>(kernel, passes);
    case 4: return tc_sym_kp<T, 4>(kernel, passes);
    default: return nullptr;
  }
}
}  // namespace

const void* tchain_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  const TChainP& p = a.u.tchain;
  switch (p.dt) {
    case DT_F32: return tc_sym<float>(kernel, p.vecs_per_lane, p.passes);
    case DT_F16: return tc_sym<f16_t>(kernel, p.vecs_per_lane, p.passes);
    default: return tc_sym<bf16_t>(kernel, p.vecs_per_lane, p.passes);
  }
}

}  // namespace fs
