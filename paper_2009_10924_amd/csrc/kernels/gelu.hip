// Stitched bias + tanh-GELU, alone (thread composition) or packed with the
// bias-gradient column reduction (kernel packing + a global hand-off):
//     z = x + bias;  y = gelu(z);  dbias = colsum(grad * gelu'(z))
// GELU and GELU' share one exp and one reciprocal per element (the computation-reuse
// rule of the paper's Section 4.5) and one read of x.
//
// The column reduction needs rows owned by other workgroups, which the paper's
// schemes exclude (Section 4.1, last paragraph: no inter-block communication).  Here
// it is one round trip through device memory: every workgroup writes its column
// partials to a [n_row_tiles, cols] float32 workspace, takes a ticket from a per
// column-tile counter, and the workgroup that draws the last ticket folds the
// partials in row-tile order.  The fold order is fixed, so results are bit-identical
// from run to run, and the counter is left at zero for the next launch.
#include <hip/hip_runtime.h>

#include "device_utils.hpp"
#include "kernel_table.hpp"

namespace fsk {
using namespace fs;

// ---- bias + GELU only ------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_bias_gelu(const T* __restrict__ x, const T* __restrict__ bias,
                                                   T* __restrict__ y, GeluP p) {
  constexpr int VEC = Elem<T>::VEC;
  const uint32_t vecs_per_row = p.cols / VEC;
  const uint32_t n_vec = p.rows * vecs_per_row;
  const uint32_t vi = blockIdx.x * 256u + threadIdx.x;
  if (vi >= n_vec) return;
  const uint32_t cv = vi % vecs_per_row;
  float v[VEC], b[VEC];
  load_vec(x + (size_t)vi * VEC, v);
  load_vec(bias + cv * VEC, b);
#pragma unroll
  for (int e = 0; e < VEC; ++e) v[e] = gelu_fwd(v[e] + b[e]);
  store_vec(y + (size_t)vi * VEC, v);
}

// ---- bias + GELU forward + bias-gradient column sum --------------------------------
// Workgroup = WAVES wavefronts over one tile of rows_per_block rows x (64*VEC) columns.
// Lane l of every wave owns columns [l*VEC, l*VEC+VEC) of the tile; wave w walks rows
// w, w+WAVES, ... of the tile, so each wave-wide access is 1 KB contiguous.
template <typename T, int WAVES>
__global__ void __launch_bounds__(WAVES * 64) k_bias_gelu_dbias(const T* __restrict__ x, const T* __restrict__ bias,
                                                                const T* __restrict__ grad, T* __restrict__ y,
                                                                float* __restrict__ dbias, float* __restrict__ partials,
                                                                uint32_t* __restrict__ counters, GeluP p) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int TILE_COLS = 64 * VEC;
  __shared__ float red[WAVES][TILE_COLS];
  __shared__ uint32_t ticket;
  const uint32_t n_col_tiles = (p.cols + TILE_COLS - 1) / TILE_COLS;
  const uint32_t ct = blockIdx.x % n_col_tiles;
  const uint32_t rt = blockIdx.x / n_col_tiles;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t col = ct * TILE_COLS + lane * VEC;
  const bool col_ok = col < p.cols;              // cols is a multiple of VEC
  const uint32_t r_begin = rt * p.rows_per_block;
  const uint32_t r_end = min(r_begin + p.rows_per_block, p.rows);

  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
  if (col_ok) {
    float b[VEC];
    load_vec(bias + col, b);
    constexpr uint32_t UNROLL = 2;
    uint32_t r = r_begin + wave;
    for (; r + (UNROLL - 1) * WAVES < r_end; r += UNROLL * WAVES) {
      float xv[UNROLL][VEC], gv[UNROLL][VEC];
#pragma unroll
      for (uint32_t u = 0; u < UNROLL; ++u) {
        const size_t off = (size_t)(r + u * WAVES) * p.cols + col;
        load_vec(x + off, xv[u]);
        load_vec(grad + off, gv[u]);
      }
#pragma unroll
      for (uint32_t u = 0; u < UNROLL; ++u) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float z = xv[u][e] + b[e];
          float s, d;
          gelu_parts(z, s, d);
          const float zs = z * s;
          xv[u][e] = zs;
          acc[e] = __builtin_fmaf(gv[u][e], __builtin_fmaf(zs * (1.0f - s), d, s), acc[e]);
        }
        store_vec(y + (size_t)(r + u * WAVES) * p.cols + col, xv[u]);
      }
    }
    for (; r < r_end; r += WAVES) {
      float xv[VEC], gv[VEC];
      const size_t off = (size_t)r * p.cols + col;
      load_vec(x + off, xv);
      load_vec(grad + off, gv);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float z = xv[e] + b[e];
        float s, d;
        gelu_parts(z, s, d);
        const float zs = z * s;
        xv[e] = zs;
        acc[e] = __builtin_fmaf(gv[e], __builtin_fmaf(zs * (1.0f - s), d, s), acc[e]);
      }
      store_vec(y + off, xv);
    }
  }

  // regional step: fold the waves of this workgroup through LDS, in wave order
#pragma unroll
  for (int e = 0; e < VEC; ++e) red[wave][lane * VEC + e] = acc[e];
  __syncthreads();
  for (uint32_t c = threadIdx.x; c < TILE_COLS; c += WAVES * 64) {
    float s = red[0][c];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) s += red[w][c];
    const uint32_t gc = ct * TILE_COLS + c;
    if (gc < p.cols) partials[(size_t)rt * p.cols + gc] = s;
  }

  // global step: publish, take a ticket, last workgroup of this column tile folds
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0)
    ticket = __hip_atomic_fetch_add(&counters[ct], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (ticket != p.n_row_tiles - 1) return;
  __threadfence();
  for (uint32_t c = threadIdx.x; c < TILE_COLS; c += WAVES * 64) {
    const uint32_t gc = ct * TILE_COLS + c;
    if (gc >= p.cols) continue;
    float s = 0.0f;
    const float* src = partials + gc;
    uint32_t t = 0;
    for (; t + 8 <= p.n_row_tiles; t += 8) {
      float q[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) q[u] = __builtin_nontemporal_load(src + (size_t)(t + u) * p.cols);
#pragma unroll
      for (int u = 0; u < 8; ++u) s += q[u];
    }
    for (; t < p.n_row_tiles; ++t) s += __builtin_nontemporal_load(src + (size_t)t * p.cols);
    dbias[gc] = s;
  }
  if (threadIdx.x == 0) __hip_atomic_store(&counters[ct], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace fsk

namespace fs {
using namespace fsk;

const void* gelu_kernel_symbol(int32_t kernel, const KernelArgs& a) {
  const GeluP& p = a.u.gelu;
  if (kernel == K_BIAS_GELU) {
    switch (p.dt) {
      case DT_F32: return (const void*)k_bias_gelu<float>;
      case DT_F16: return (const void*)k_bias_gelu<f16_t>;
      default: return (const void*)k_bias_gelu<bf16_t>;
    }
  }
  switch (p.dt) {
    case DT_F32: return (const void*)k_bias_gelu_dbias<float, 8>;
    case DT_F16: return (const void*)k_bias_gelu_dbias<f16_t, 8>;
    default: return (const void*)k_bias_gelu_dbias<bf16_t, 8>;
  }
}

}  // namespace fs
